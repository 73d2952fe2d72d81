// Loops 2-4 of Algorithm 1 (Lavin & Gray) in one kernel, fp32 F(4x4,3x3), second design: small
// workgroups that alternate transform and multiply phases, two per CU so that one multiplies while
// the other transforms, waits for memory or stores (on this chip MFMA and ordinary vector
// instructions of one SIMD do not overlap, so what a second workgroup can fill is the waiting).
//
// Workgroup = 4 wavefronts owning 32 filters x 32 tiles x 36 components (144 accumulators per lane).
// Per step of 8 channels:
//   1. transform phase: every thread owns one (tile, channel) pair.  Its 6 x 6 taps were requested
//      one step ahead, straight into registers, as buffer loads (per row one aligned 16-byte load
//      and the two outer columns): a tap outside the image -- the implicit zero padding of
//      Section 6 -- or in a channel past the last one is addressed beyond the buffer, for which
//      the hardware returns 0, so the loop holds no compare, no select and no address arithmetic.
//      v = B^T (d B) goes to LDS as [e][channel][tile]; then the taps of the next step are requested;
//      the step's transformed filters U[e][c][k] arrive as [e][channel][filter] by direct
//      global -> LDS loads (16 bytes per lane, no registers) requested right after the previous
//      multiply phase;
//   2. multiply phase: wavefront cg owns components 9 cg .. 9 cg + 8; lane (i, h) feeds channel
//      2 t + h of filter row i and tile column i to the t-th v_mfma_f32_32x32x2_f32 of a component
//      (LDS reads of 64 consecutive floats: conflict-free).
// After the last step the accumulators go through LDS in four pieces of 8 filters; every thread
// gathers the 36 components of one (filter, tile) pair, applies Y = A^T m A and writes the rows
// of its 4 x 4 outputs that are inside the image as 16-byte stores.
// Needs pad = 1, W % 4 == 0 and the images one workgroup touches (two, or 33 one-tile images) within 1 GiB.
#include "wino_internal.h"
#include "transforms.h"

namespace wino {

typedef float floatx16_l __attribute__((ext_vector_type(16)));
typedef float floatx4_l __attribute__((ext_vector_type(4)));
typedef unsigned uintx4_l __attribute__((ext_vector_type(4)));

constexpr int FL_K = 32, FL_P = 32, FL_C = 8, FL_T = 256;           // filters, tiles, channels per step, threads
constexpr int FL_U_FLOATS = 36 * FL_C * FL_K;                       // transformed filters of a step
constexpr int FL_V_FLOATS = 36 * FL_C * FL_P;                       // transformed tiles of a step
constexpr int FL_M_FLOATS = 36 * 8 * FL_P;                          // one piece of M in the epilogue
constexpr unsigned FL_MAX_BYTES = 0x40000000u;                      // longest stretch of D one workgroup's buffer covers
constexpr unsigned FL_ROW_OOB = 0x80000000u, FL_COL_OOB = 0x40000000u;   // offset markers of taps outside the image
static_assert(FL_U_FLOATS % (FL_T * 4) == 0, "every thread copies the same number of 16-byte words of U");
static_assert(FL_M_FLOATS <= FL_U_FLOATS + FL_V_FLOATS, "the epilogue reuses the operand area");

#define WINO_L_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define WINO_L_GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

// Barrier that orders LDS traffic only: global loads requested earlier stay in flight across it.
__device__ __forceinline__ void fl_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Barrier after which LDS that this workgroup has only READ may be overwritten: waits for this wavefront's LDS
// reads, not for global -> LDS copies in flight (a fence would wait for those too: they count as LDS writes).
__device__ __forceinline__ void fl_reads_done_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xc07f);      // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// CPAD: the channel count is not a multiple of 8, so the last step holds channel slots past the last channel.
template <bool CPAD>
__global__ __launch_bounds__(FL_T, 2) void fused_lds_kernel(const float *__restrict__ D, const float *__restrict__ U,
                                                            float *__restrict__ Y, Geo g, int n_kb, int n_items)
{
    __shared__ __attribute__((aligned(16))) float smem[FL_U_FLOATS + FL_V_FLOATS];
    float *Us = smem;
    float *Vs = smem + FL_U_FLOATS;
    const int tid = threadIdx.x;

    // A workgroup stays on its CU and walks a list of (tile block, filter block) items: the output stores of one
    // item drain while the next one is computed, and launch and index set-up are paid once.  Workgroups are dealt
    // to the 8 XCDs round-robin; each XCD takes one contiguous eighth of the items and its resident workgroups
    // stride through it together, so the filter blocks of one tile block (which read the same input) meet in one L2.
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8, slots = gridDim.x / 8;
    const int per_xcd = (n_items + 7) / 8;
    const int item_end = min((xcd + 1) * per_xcd, n_items);
    for (int item = xcd * per_xcd + slot; item < item_end; item += slots) {
    const int kb = item % n_kb, tb = item / n_kb;
    const int k0 = kb * FL_K, b0 = tb * FL_P;

    // ---- transform-phase role: (tile, channel slot of the step) ---------------------------------
    const int tl = tid & 31, cl = tid >> 5;
    const int b = b0 + tl;
    const bool tile_ok = b < g.P;
    int orow = 0;
    float *ybase = Y;
    // The buffer the taps are loaded from starts at the first image this workgroup touches, so the byte offsets
    // stay small whatever the size of D.  A row piece outside the image gets the offset FL_ROW_OOB, a column
    // outside gets FL_COL_OOB added instead of its distance from the middle piece: with the offsets of valid
    // taps below 2^30 (see fused_lds_eligible), every sum with one of the two markers in it lies beyond the
    // buffer (at most 2^30 bytes long), where a buffer load returns 0.
    const int tiles_per_image = g.Th * g.Tw;
    const int img0 = b0 / tiles_per_image;                     // uniform
    unsigned vo_m[6];                                          // byte offset of columns 1..4 of row p, channel slot cl, step 0
    unsigned adj_l, adj_r;
    {
        const int bb = tile_ok ? b : b0;
        const int ty = bb % g.Tw;
        const int t2 = bb / g.Tw;
        const int tx = t2 % g.Th;
        const int i = t2 / g.Th;
        const int x0 = 4 * tx - 1, y0 = 4 * ty - 1;
        orow = 4 * tx;
        ybase = Y + ((size_t)i * g.K * g.Ho + orow) * g.Wo + 4 * ty;
        adj_l = (y0 >= 0) ? 0xfffffffcu : FL_COL_OOB;             // -4 bytes
        adj_r = (y0 + 5 < g.W) ? 16u : FL_COL_OOB;
        const unsigned plane0 = (unsigned)((i - img0) * g.C + cl) * (unsigned)(g.H * g.W);
#pragma unroll
        for (int p = 0; p < 6; ++p) {
            const int x = x0 + p;
            const bool rok = tile_ok && x >= 0 && x < g.H;
            vo_m[p] = rok ? (plane0 + (unsigned)(x * g.W + y0 + 1)) * 4u : FL_ROW_OOB;   // column y0 + 1 = 4 ty
        }
    }
    const unsigned step_bytes = (unsigned)(FL_C * g.H * g.W) * 4u;
    const size_t image_floats = (size_t)g.C * g.H * g.W;
    const size_t left = ((size_t)g.N - img0) * image_floats * 4;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(D + (size_t)img0 * image_floats), 0, (unsigned)(left < FL_MAX_BYTES ? left : FL_MAX_BYTES), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_u =
        __builtin_amdgcn_make_buffer_rsrc((void *)U, 0, (unsigned)((size_t)36 * g.Cp * g.Kp * 4), 0x00020000);

    // ---- multiply-phase role -------------------------------------------------------------------
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int cg = wave;
    const int li = lane & 31, lh = lane >> 5;
    floatx16_l acc[9];
#pragma unroll
    for (int e = 0; e < 9; ++e)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[e][r] = 0.0f;

    const int nsteps = (g.C + FL_C - 1) / FL_C;      // U holds zeros for the channels between C and Cp

    // Transformed filters of a step: LDS float ((e * 8 + c) * 32 + k) <- U[(e * Cp + 8 step + c) * Kp + k0 + k];
    // thread t copies 16-byte word w = t + 256 j (j = 0..8): e = w / 64, c = (w / 8) % 8, k = 4 (w % 8)
    // (c and k do not depend on j, and e advances by 4 per j: one per-lane offset, the rest is uniform)
    constexpr int NCH = FL_U_FLOATS / (FL_T * 4);
    const unsigned uoff = (unsigned)(((tid / 64) * g.Cp + ((tid / 8) & 7)) * g.Kp + k0 + (tid & 7) * 4) * 4u;
    const unsigned ustep_bytes = (unsigned)(FL_C * g.Kp) * 4u, uj_bytes = (unsigned)(4 * g.Cp * g.Kp) * 4u;
    auto load_u = [&](int step) {
        const unsigned so = (unsigned)step * ustep_bytes;
#pragma unroll
        for (int j = 0; j < NCH; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_u, WINO_L_LDS_PTR(Us + (wave * 64 + FL_T * j) * 4), 16, uoff,
                                                     so + j * uj_bytes, 0, 0);
    };
    floatx4_l mid[6];
    float l[6], r[6];
    auto load_taps = [&](int step) {
        const unsigned so = (unsigned)step * step_bytes;
        const bool ch_ok = !CPAD || (step * FL_C + cl < g.C);
#pragma unroll
        for (int p = 0; p < 6; ++p) {
            const unsigned om = ch_ok ? vo_m[p] : FL_ROW_OOB;
            mid[p] = __builtin_bit_cast(floatx4_l, __builtin_amdgcn_raw_buffer_load_b128(rsrc, om, so, 0));
            l[p] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, om + adj_l, so, 0));
            r[p] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, om + adj_r, so, 0));
        }
    };

    const int a_off = lh * 32 + li;                // within one (e, t): channel 2 t + lh, row / column li
    // Order of the memory requests: taps of step s + 1 before the multiply phase of step s, filters of step s + 1
    // after it -- so the wait for the taps at the top of a step leaves the filter loads in flight.
    load_taps(0);
    load_u(0);
    for (int step = 0;; ++step) {
        // 1. this thread's tile: rows then columns (v = B^T (d B)), scatter to LDS
        {
            float t[6][6];
#pragma unroll
            for (int p = 0; p < 6; ++p) {
                const float d[6] = {l[p], mid[p][0], mid[p][1], mid[p][2], mid[p][3], r[p]};
                bt_mul<4>(d, t[p]);
            }
            float *dst = Vs + cl * FL_P + tl;
#pragma unroll
            for (int q = 0; q < 6; ++q) {
                const float col[6] = {t[0][q], t[1][q], t[2][q], t[3][q], t[4][q], t[5][q]};
                float o[6];
                bt_mul<4>(col, o);
#pragma unroll
                for (int p = 0; p < 6; ++p) dst[(p * 6 + q) * (FL_C * FL_P)] = o[p];
            }
        }
        const bool more = step + 1 < nsteps;
        // the filters of this step (requested right after the previous step's multiply phase) and the LDS stores
        // above must have landed
        __builtin_amdgcn_s_waitcnt(0x0070);      // vmcnt(0) lgkmcnt(0)
        fl_lds_barrier();
        // the taps of the next step: in flight during the multiply phase below, which needs few registers
        if (more) load_taps(step + 1);
        // 2. nine components x (32 filters x 32 tiles x 8 channels); the operands of the next component are read
        //    from LDS while the four MFMAs of the current one run
        {
            float a[2][4], bb[2][4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                a[0][t] = Us[cg * 9 * (FL_C * 32) + a_off + t * 64];
                bb[0][t] = Vs[cg * 9 * (FL_C * 32) + a_off + t * 64];
            }
#pragma unroll
            for (int e = 0; e < 9; ++e) {
                if (e + 1 < 9) {
                    const int eo = (cg * 9 + e + 1) * (FL_C * 32) + a_off;
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        a[(e + 1) & 1][t] = Us[eo + t * 64];
                        bb[(e + 1) & 1][t] = Vs[eo + t * 64];
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    acc[e] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e & 1][t], bb[e & 1][t], acc[e], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // every wavefront has read its operands (LDS reads only: the taps in flight stay in flight)
        fl_reads_done_barrier();
        if (!more) break;
        load_u(step + 1);
    }
    __syncthreads();

    // ---- inverse transform: four pieces of 8 filters -------------------------------------------
    float *Ms = smem;
    const int frow = tid >> 5;                 // 0..7: filter row of the piece handled in the gather
    const int ot = tid & 31;                   // tile of the gather (same tile as in the transform phase)
    for (int q = 0; q < 4; ++q) {
        // accumulator register r of lane (li, lh) is filter 8 * (r / 4) + 4 * lh + r % 4, tile li
#pragma unroll
        for (int e = 0; e < 9; ++e)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) Ms[((cg * 9 + e) * 8 + 4 * lh + rr) * FL_P + li] = acc[e][4 * q + rr];
        __syncthreads();
        const int k = k0 + 8 * q + frow;
        if (tile_ok && k < g.K) {
            float m[6][6], tt[4][6], y[4][4];
#pragma unroll
            for (int xi = 0; xi < 6; ++xi)
#pragma unroll
                for (int nu = 0; nu < 6; ++nu) m[xi][nu] = Ms[((xi * 6 + nu) * 8 + frow) * FL_P + ot];
#pragma unroll
            for (int nu = 0; nu < 6; ++nu) {
                const float col[6] = {m[0][nu], m[1][nu], m[2][nu], m[3][nu], m[4][nu], m[5][nu]};
                float o[4];
                at_mul<4>(col, o);
#pragma unroll
                for (int p = 0; p < 4; ++p) tt[p][nu] = o[p];
            }
#pragma unroll
            for (int p = 0; p < 4; ++p) at_mul<4>(tt[p], y[p]);
            float *dst = ybase + (size_t)k * g.Ho * g.Wo;
#pragma unroll
            for (int p = 0; p < 4; ++p)
                if (orow + p < g.Ho)
                    __builtin_nontemporal_store(floatx4_l{y[p][0], y[p][1], y[p][2], y[p][3]},
                                                reinterpret_cast<floatx4_l *>(dst + (size_t)p * g.Wo));
        }
        __syncthreads();
    }
    }   // items
}

bool fused_lds_eligible(const Geo &g)
{
    // the tiles of one workgroup span at most `span` images; their byte offsets from the first must stay below 2^30
    const unsigned long long tiles = (unsigned long long)g.Th * g.Tw;
    const unsigned long long span = (FL_P + tiles - 2) / tiles + 1;
    const unsigned long long image_bytes = (unsigned long long)g.C * g.H * g.W * 4ull;
    return g.dt == WINO_F32 && g.m == 4 && g.pad == 1 && g.W % 4 == 0 && span * image_bytes + 65536 < FL_MAX_BYTES &&
           (unsigned long long)36 * g.Cp * g.Kp * 4ull < (1ull << 31);   // 32-bit byte offsets into U
}

hipError_t launch_fused_lds(const Geo &g, const float *D, const float *U, float *Y, hipStream_t s)
{
    const int n_kb = g.Kp / FL_K;
    const long long items = (long long)((g.P + FL_P - 1) / FL_P) * n_kb;
    if (items > 0x7fffffffLL) return hipErrorInvalidValue;
    // two workgroups per CU (what registers and LDS allow) on 256 CUs, in multiples of the 8 XCDs
    const unsigned grid = (unsigned)(items >= 512 ? 512 : (items + 7) / 8 * 8);
    if (g.C % FL_C != 0)
        fused_lds_kernel<true><<<dim3(grid), dim3(FL_T), 0, s>>>(D, U, Y, g, n_kb, (int)items);
    else
        fused_lds_kernel<false><<<dim3(grid), dim3(FL_T), 0, s>>>(D, U, Y, g, n_kb, (int)items);
    return hipGetLastError();
}

}  // namespace wino

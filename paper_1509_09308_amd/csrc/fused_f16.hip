// Loops 2-4 of Algorithm 1 (Lavin & Gray) in one kernel for fp16 storage: F(4x4,3x3), V and M never
// reach memory (Section 6 describes such a fused kernel for F(2x2,3x3)).  With fp16 operands the
// multiply is 16 times cheaper than in fp32 while M stays fp32, so the four-stage path of a layer
// with few filters spends its time writing and re-reading V and above all M; here a workgroup keeps
// all 36 components of a 64-filter x 32-tile block in registers and the layer costs one read of D
// and one write of Y.
//
// Workgroup = 4 KH wavefronts owning 32 KH filters x 32 tiles.  KH = 1 is small enough in registers and
// LDS for two workgroups per CU.  KH = 2 (one workgroup per CU, used when the layer has more than 32
// filters) lets a second set of four wavefronts multiply the same transformed tiles with 32 more filters:
// the input transform, which costs a wavefront four times what its share of the multiply does, is then
// done once per 64 filters instead of once per 32.  Per step of 8 channels:
//   1. transform phase: every thread of the first four wavefronts unpacks the 6 x 6 fp16 tile of one (tile, channel) pair (per row
//      one aligned 8-byte load and the two outer columns, requested one step ahead; zeros outside
//      the image), computes v = B^T (d B) in fp32, rounds once to fp16 and writes the 36 values to
//      LDS in the operand order of the MFMA, [e][c / 4][tile][c % 4]; the 36 x 32 x 8 transformed filters
//      of the step are copied from U (same order, [e][c / 8][k][c % 8]) with 16-byte loads;
//   2. multiply phase: wavefront cg owns components 9 cg .. 9 cg + 8: one v_mfma_f32_32x32x8_f16
//      per component, both operands one 8-byte LDS read per lane, fp32 accumulation.
// After the last step the accumulators go through LDS in four pieces of 8 KH filters, every thread
// gathers the 36 components of one (filter, tile) pair, applies Y = A^T m A and writes the 4 x 4
// outputs that are inside the image as 16-byte rows.
// Needs m = 4, pad = 1, W % 4 == 0 (aligned 8-byte loads, 16- or 8-byte stores); Y in fp32 or fp16.
#include "wino_internal.h"
#include "transforms.h"
#include <mutex>

namespace wino {

typedef float floatx16_h __attribute__((ext_vector_type(16)));
typedef float floatx4_h __attribute__((ext_vector_type(4)));
typedef _Float16 halfx4_h __attribute__((ext_vector_type(4)));

constexpr int HF_P = 32, HF_C = 8;                                // tiles per workgroup, channels per step
constexpr int HF_V_WORDS = 36 * HF_P;                             // 16-byte words of V per step
constexpr int hf_u_words(int KH) { return 36 * 32 * KH; }         // 16-byte words of U per step
constexpr int hf_lds_words(int KH) { return 2 * hf_u_words(KH) + HF_V_WORDS; }   // two filter buffers and one for V
constexpr int hf_m_floats(int KH) { return 36 * 8 * KH * HF_P; }  // one piece of M in the epilogue
static_assert(hf_m_floats(1) * 4 <= hf_lds_words(1) * 16 && hf_m_floats(2) * 4 <= hf_lds_words(2) * 16,
              "the epilogue reuses the operand area");

#define WINO_H_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define WINO_H_GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

// Barrier that orders LDS traffic only (global loads requested earlier stay in flight across it).
__device__ __forceinline__ void hf_lds_barrier()
{
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
}

// 16 bytes per lane from a buffer straight into LDS: lane l of the wavefront fills lds + 16 l.  (Kept out of the
// kernel template: the host pass of the compiler cannot check this builtin in a context that depends on a
// template parameter and would drop the kernel without a diagnostic.)
__device__ __forceinline__ void hf_copy16_to_lds(__amdgpu_buffer_rsrc_t rsrc, uint4 *lds, unsigned voffset, unsigned soffset)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, WINO_H_LDS_PTR(lds), 16, voffset, soffset, 0, 0);
}

constexpr unsigned HF_MAX_BYTES = 0x40000000u;                     // longest stretch of D one workgroup's buffer covers
constexpr unsigned HF_ROW_OOB = 0x80000000u, HF_COL_OOB = 0x40000000u;   // offset markers of taps outside the image

// CPAD: the channel loop (over the padded count Cp) holds channel slots past the last channel.
// four neighbouring outputs of a row, not kept in the caches; fp32 or rounded once to fp16
__device__ __forceinline__ void hf_store4(float *p, floatx4_h v)
{
    __builtin_nontemporal_store(v, reinterpret_cast<floatx4_h *>(p));
}
__device__ __forceinline__ void hf_store4(__half *p, floatx4_h v)
{
    typedef unsigned uintx2_s __attribute__((ext_vector_type(2)));
    const __half2 a = __floats2half2_rn(v[0], v[1]), b = __floats2half2_rn(v[2], v[3]);
    __builtin_nontemporal_store(uintx2_s{__builtin_bit_cast(unsigned, a), __builtin_bit_cast(unsigned, b)},
                                reinterpret_cast<uintx2_s *>(p));
}

template <bool CPAD, int KH, typename YT>
__global__ __launch_bounds__(256 * KH, 3 - KH) void fused_f16_kernel(const __half *__restrict__ D, const uint4 *__restrict__ U,
                                                                     YT *__restrict__ Y, Geo g, int n_kb, int n_items)
{
    constexpr int HF_K = 32 * KH, HF_U_WORDS = hf_u_words(KH), WAVES = 4 * KH;
    extern __shared__ uint4 smem[];                                 // hf_lds_words(KH) words
    uint4 *Us = smem;                                               // buffer b at + b * HF_U_WORDS
    __half *Vs = reinterpret_cast<__half *>(smem + 2 * HF_U_WORDS);
    const uint4 *Vw = smem + 2 * HF_U_WORDS;
    const int tid = threadIdx.x;

    // A workgroup stays on its CU and walks a list of (tile block, filter block) items: the output stores of one
    // item drain while the next one is computed.  Each XCD takes one contiguous eighth of the items and its
    // resident workgroups stride through it together, so the filter blocks of one tile block meet in one L2.
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8, slots = gridDim.x / 8;
    const int per_xcd = (n_items + 7) / 8;
    const int item_end = min((xcd + 1) * per_xcd, n_items);
    for (int item = xcd * per_xcd + slot; item < item_end; item += slots) {
    const int kb = item % n_kb, tb = item / n_kb;
    const int k0 = kb * HF_K, b0 = tb * HF_P;

    // ---- transform-phase role: (tile, channel of the step) ------------------------------------
    const int tl = tid & 31, cl = (tid >> 5) & 7;
    const int b = b0 + tl;
    const bool tile_ok = b < g.P;
    // The taps are loaded through a buffer that starts at the first image this workgroup touches.  A row outside the
    // image gets the offset HF_ROW_OOB, a column outside gets HF_COL_OOB added instead of its distance from the
    // middle piece: with the offsets of valid taps below 2^30 (see fused_f16_eligible) every sum with a marker in
    // it lies beyond the buffer, where a load returns 0 -- the implicit zero padding of Section 6 without a compare.
    const int tiles_per_image = g.Th * g.Tw;
    const int img0 = b0 / tiles_per_image;                     // uniform
    unsigned vo_m[6];                                          // byte offset of columns 1..4 of row p, channel slot cl, step 0
    // The outer columns (0 and 5) of a tile are column 4 of the tile to its left and column 1 of the tile to its
    // right, and neighbouring tiles sit in neighbouring lanes: a lane takes them from its neighbours' registers
    // (DPP, within rows of 16 lanes) instead of from memory -- requests of 2 bytes per lane at a stride of 8 bytes
    // cost the vector memory path as much as the 8-byte ones next to them.  Only the first lane of a row of 16 has
    // to fetch its left column and the last lane its right column: one 4-byte request per tile row (`edge_adj` =
    // where, or a marker for the lanes in between) for the word that the missing neighbour would hold, columns
    // 3 and 4 of the tile to the left resp. 1 and 2 of the tile to the right.  A tile at the image's left or right
    // border has zeros there (`left_in`, `right_in`), whatever its neighbour lane holds.
    unsigned edge_adj;
    bool left_in, right_in;
    {
        const int bb = tile_ok ? b : b0;
        const int ty = bb % g.Tw;
        const int t2 = bb / g.Tw;
        const int tx = t2 % g.Th;
        const int i = t2 / g.Th;
        const int x0 = 4 * tx - 1, y0 = 4 * ty - 1;
        left_in = y0 >= 0;
        right_in = y0 + 5 < g.W;
        edge_adj = ((tl & 15) == 0 && left_in) ? 0xfffffffcu /* -4 bytes */ : ((tl & 15) == 15 && right_in) ? 8u : HF_COL_OOB;
        const unsigned plane0 = (unsigned)((i - img0) * g.C + cl) * (unsigned)(g.H * g.W);
#pragma unroll
        for (int p = 0; p < 6; ++p) {
            const int x = x0 + p;
            const bool rok = tile_ok && x >= 0 && x < g.H;
            vo_m[p] = rok ? (plane0 + (unsigned)(x * g.W + y0 + 1)) * 2u : HF_ROW_OOB;   // column y0 + 1 = 4 ty
        }
    }
    const unsigned step_bytes = (unsigned)(HF_C * g.H * g.W) * 2u;
    const size_t image_halves = (size_t)g.C * g.H * g.W;
    const size_t left = ((size_t)g.N - img0) * image_halves * 2;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(D + (size_t)img0 * image_halves), 0, (unsigned)(left < HF_MAX_BYTES ? left : HF_MAX_BYTES), 0x00020000);

    // ---- multiply-phase role -------------------------------------------------------------------
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int cg = wave & 3, kh = wave >> 2;                   // nine components, 32 filters
    const bool xf = KH == 1 || wave < 4;                       // takes part in the transform phase
    const int li = lane & 31, lg = lane >> 5;
    floatx16_h acc[9];
#pragma unroll
    for (int e = 0; e < 9; ++e)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[e][r] = 0.0f;

    const int nsteps = g.Cp / HF_C;

    // raw fp16 taps of one tile: per row the four middle columns (8 bytes) and, in the lanes at the ends of a row
    // of 16, the word with the outer column.  They are requested one step ahead, at the start of the multiply
    // phase of the step before.
    typedef unsigned uintx2_h __attribute__((ext_vector_type(2)));
    uintx2_h rmid[6];
    unsigned red[6];
    auto load_raw = [&](int step) {
        const unsigned so = (unsigned)step * step_bytes;
        const bool ch_ok = !CPAD || (step * HF_C + cl < g.C);
#pragma unroll
        for (int p = 0; p < 6; ++p) {
            const unsigned om = ch_ok ? vo_m[p] : HF_ROW_OOB;
            rmid[p] = __builtin_amdgcn_raw_buffer_load_b64(rsrc, om, so, 0);
            red[p] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, om + edge_adj, so, 0);
        }
    };
    // Transformed filters of a step, [e][c8 = step][k] -> Us[e * 32 + k]: direct global -> LDS loads of
    // 16 bytes per lane (no registers), one step ahead into the other buffer; a step waits for all of its own
    // requests (vmcnt(0)) before the barrier that precedes its multiply phase.
    constexpr int NCH = (HF_U_WORDS / 64 + WAVES - 1) / WAVES;   // chunks of 64 words per wavefront
    // chunk wave + WAVES j holds components (64 / HF_K)(wave + WAVES j) ..: the lane's word of chunk j lies a fixed
    // number of bytes behind its word of chunk 0
    const int w0 = wave * 64 + lane;
    const unsigned uoff = ((unsigned)((w0 / HF_K) * nsteps) * g.Kp + min(k0 + w0 % HF_K, g.Kp - 1)) * 16u;   // step 0
    const unsigned uj_bytes = (unsigned)(WAVES * 64 / HF_K) * (unsigned)nsteps * (unsigned)g.Kp * 16u;
    const __amdgpu_buffer_rsrc_t rsrc_u =
        __builtin_amdgcn_make_buffer_rsrc((void *)U, 0, (unsigned)((size_t)36 * nsteps * g.Kp * 16), 0x00020000);
    auto load_u = [&](int buf, int step) {
        const unsigned so = (unsigned)step * (unsigned)g.Kp * 16u;
#pragma unroll
        for (int j = 0; j < NCH; ++j) {
            const int chunk = wave + WAVES * j;
            if (chunk < HF_U_WORDS / 64)
                hf_copy16_to_lds(rsrc_u, Us + buf * HF_U_WORDS + chunk * 64, uoff, so + j * uj_bytes);
        }
    };
    if (xf) load_raw(0);
    load_u(0, 0);
    for (int step = 0; step < nsteps; ++step) {
        const uint4 *Ub = Us + (step & 1) * HF_U_WORDS;
        const bool more = step + 1 < nsteps;
        // the filters of the next step, into the buffer the previous multiply phase has finished with
        if (more) load_u((step + 1) & 1, step + 1);
        // 1. one input tile: unpack, transform rows then columns (v = B^T (d B)), round, scatter
        if (xf) {
            float t[6][6];
#pragma unroll
            for (int p = 0; p < 6; ++p) {
                const unsigned w01 = rmid[p][0], w23 = rmid[p][1];      // (a bit cast wants a scalar object, not a vector element)
                const __half2 h01 = __builtin_bit_cast(__half2, w01);
                const __half2 h23 = __builtin_bit_cast(__half2, w23);
                // columns (3, 4) of the lane below (row_shr:1), columns (1, 2) of the lane above (row_shl:1); the
                // first and the last lane of a row of 16, which have no such neighbour, keep the word they fetched
                const unsigned wl = (unsigned)__builtin_amdgcn_update_dpp((int)red[p], (int)w23, 0x111, 0xf, 0xf, false);
                const unsigned wr = (unsigned)__builtin_amdgcn_update_dpp((int)red[p], (int)w01, 0x101, 0xf, 0xf, false);
                const float lv = left_in ? __high2float(__builtin_bit_cast(__half2, wl)) : 0.0f;
                const float rv = right_in ? __low2float(__builtin_bit_cast(__half2, wr)) : 0.0f;
                const float d[6] = {lv, __low2float(h01), __high2float(h01), __low2float(h23), __high2float(h23), rv};
                bt_mul<4>(d, t[p]);
            }
            __half *dst = Vs + ((size_t)(cl >> 2) * HF_P + tl) * 4 + (cl & 3);   // [e][c / 4][tile][c % 4]
#pragma unroll
            for (int q = 0; q < 6; ++q) {
                const float col[6] = {t[0][q], t[1][q], t[2][q], t[3][q], t[4][q], t[5][q]};
                float o[6];
                bt_mul<4>(col, o);
#pragma unroll
                for (int p = 0; p < 6; ++p) dst[(size_t)(p * 6 + q) * (HF_P * 8)] = __float2half_rn(o[p]);
            }
        }
        // this step's filters (requested a step ago) and the LDS stores above must have landed; the next step's
        // filters, requested at the top of this step, are waited for as well (they had the transform to arrive)
        __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        // the taps of the next step: in flight during the multiply phase below
        if (xf && more) load_raw(step + 1);
        // 2. nine components x (32 filters x 32 tiles x 8 channels); lane (li, lg) feeds channels 4 lg .. 4 lg + 3
#pragma unroll
        for (int e = 0; e < 9; ++e) {
            const int ee = cg * 9 + e;
            const uint2 ua = reinterpret_cast<const uint2 *>(Ub)[(ee * HF_K + kh * 32 + li) * 2 + lg];
            const uint2 vb = reinterpret_cast<const uint2 *>(Vw)[(ee * 2 + lg) * HF_P + li];
            acc[e] = __builtin_amdgcn_mfma_f32_32x32x8f16(*reinterpret_cast<const halfx4_h *>(&ua),
                                                          *reinterpret_cast<const halfx4_h *>(&vb), acc[e], 0, 0, 0);
        }
        hf_lds_barrier();
    }
    __syncthreads();

    // ---- inverse transform: four pieces of 8 filters of every 32 ---------------------------------
    float *Ms = reinterpret_cast<float *>(smem);
    const int frow = tid >> 5;                 // 0 .. 8 KH - 1: filter row of the piece handled in the gather
    const int ot = tid & 31;                   // tile of the gather (same tile as in the transform phase)
    YT *ybase = Y;
    int orow = 0;
    {
        const int bb = tile_ok ? b : 0;
        const int ty = bb % g.Tw;
        const int t2 = bb / g.Tw;
        orow = 4 * (t2 % g.Th);
        ybase = Y + ((size_t)(t2 / g.Th) * g.K * g.Ho + orow) * g.Wo + 4 * ty;
    }
    for (int q = 0; q < 4; ++q) {
        // accumulator register r of lane (li, lg) is filter 8 * (r / 4) + 4 * lg + r % 4, tile li
#pragma unroll
        for (int e = 0; e < 9; ++e)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr)
                Ms[((cg * 9 + e) * (8 * KH) + 8 * kh + 4 * lg + rr) * HF_P + li] = acc[e][4 * q + rr];
        __syncthreads();
        const int k = k0 + 32 * (frow >> 3) + 8 * q + (frow & 7);
        if (tile_ok && k < g.K) {
            float m[6][6], tt[4][6], y[4][4];
#pragma unroll
            for (int xi = 0; xi < 6; ++xi)
#pragma unroll
                for (int nu = 0; nu < 6; ++nu) m[xi][nu] = Ms[((xi * 6 + nu) * (8 * KH) + frow) * HF_P + ot];
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
            YT *dst = ybase + (size_t)k * g.Ho * g.Wo;
#pragma unroll
            for (int p = 0; p < 4; ++p)
                if (orow + p < g.Ho) hf_store4(dst + (size_t)p * g.Wo, floatx4_h{y[p][0], y[p][1], y[p][2], y[p][3]});
        }
        __syncthreads();
    }
    }   // items
}

bool fused_f16_eligible(const Geo &g)
{
    // the tiles of one workgroup span at most `span` images; their byte offsets from the first must stay below 2^30
    const unsigned long long tiles = (unsigned long long)g.Th * g.Tw;
    const unsigned long long span = (HF_P + tiles - 2) / tiles + 1;
    const unsigned long long image_bytes = (unsigned long long)g.C * g.H * g.W * 2ull;
    return g.dt == WINO_F16 && g.m == 4 && g.pad == 1 && g.W % 4 == 0 && span * image_bytes + 65536 < HF_MAX_BYTES;
}

template <bool CPAD, int KH, typename YT>
static hipError_t launch_one(const Geo &g, const void *D, const void *U, YT *Y, hipStream_t s)
{
    constexpr int HF_K = 32 * KH;
    constexpr size_t lds = (size_t)hf_lds_words(KH) * 16;
    const int n_kb = (g.Kp + HF_K - 1) / HF_K;
    const long long items = (long long)((g.P + HF_P - 1) / HF_P) * n_kb;
    if (items > 0x7fffffffLL) return hipErrorInvalidValue;
    if (lds > 65536) {   // beyond the default limit of a launch: raised once per device
        static std::mutex mu;
        static bool done[64] = {};
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
        std::lock_guard<std::mutex> lock(mu);
        if (!done[dev]) {
            e = hipFuncSetAttribute((const void *)fused_f16_kernel<CPAD, KH, YT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            done[dev] = true;
        }
    }
    // as many workgroups as stay resident on 256 CUs (registers and LDS allow 3 - KH per CU), in multiples of the 8 XCDs
    const long long resident = 256 * (3 - KH);
    const unsigned grid = (unsigned)(items >= resident ? resident : (items + 7) / 8 * 8);
    fused_f16_kernel<CPAD, KH, YT><<<dim3(grid), dim3(256 * KH), lds, s>>>((const __half *)D, (const uint4 *)U, Y, g, n_kb, (int)items);
    return hipGetLastError();
}

template <typename YT>
static hipError_t launch_typed(const Geo &g, const void *D, const void *U, YT *Y, hipStream_t s)
{
    const bool cpad = g.Cp != g.C;   // the channel loop runs over Cp: slots past C must be fetched as zeros
    if (g.Kp > 32) return cpad ? launch_one<true, 2>(g, D, U, Y, s) : launch_one<false, 2>(g, D, U, Y, s);
    return cpad ? launch_one<true, 1>(g, D, U, Y, s) : launch_one<false, 1>(g, D, U, Y, s);
}

// Y is fp32 or fp16 (y_dt)
hipError_t launch_fused_f16(const Geo &g, const void *D, const void *U, void *Y, int y_dt, hipStream_t s)
{
    return y_dt == WINO_F16 ? launch_typed(g, D, U, (__half *)Y, s) : launch_typed(g, D, U, (float *)Y, s);
}

}  // namespace wino

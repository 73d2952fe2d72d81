// All four loops of Algorithm 1 (Lavin & Gray) in ONE launch for F(2x2,3x3), fp32: the filter
// transform u = G g G^T is computed inside the kernel from the untransformed filters (the variant
// Section 6 of the paper describes next to the one with pre-transformed filters), so neither U, V
// nor M ever exist in memory.  Meant for small batches, where a layer is a few microseconds of
// arithmetic and every extra launch costs as much as the arithmetic itself.
//
// Workgroup = 4 wavefronts owning 32 filters x an 8 x 8 block of tiles of one image (two MFMA
// column blocks of 4 x 8 tiles) x 16 components, and a slice of the channels.  Per step of 8 channels:
//   1. the 18 x 18 input patch under the tile block is loaded ONCE per channel (11 coalesced
//      4-byte loads per thread instead of 32 overlapping ones, zeros written for taps outside the
//      image) into a double-buffered LDS area, one step ahead; every thread reads the 4 x 4 taps
//      of one tile in two channels from there, computes v = B^T d B (32 additions each) and stores
//      it as [e][c / 2][tile][c % 2]; every thread also transforms one filter (k, c) -- 9 loads
//      requested a step ahead, 28 flops -- into LDS as [e][c / 2][k][c % 2];
//   2. wavefront w owns row xi = w of the transform domain (components 4w .. 4w + 3); lane (i, h)
//      reads channels 4j + 2h, 4j + 2h + 1 of its filter row and of its two tile columns with one
//      8-byte read each and feeds v_mfma_f32_32x32x2_f32.
// A last step that would run past the channels is moved back to end at the last channel; the
// filters of the channels it sees a second time are zeroed, so nothing is added twice.
// After the last step each wavefront applies the row half of Y = A^T m A to its own accumulators
// (t = m_row A), the four wavefronts exchange t through LDS and every thread finishes the column
// half for (filter, tile) pairs.
//
// Small layers do not have enough (filter block, tile block) pairs to fill the chip, so the channel
// loop is split over `splits` workgroups.  The inverse transform is linear, so each of them
// transforms its partial sums and stores 2 x 2 partial outputs to the workspace; the workgroup that
// arrives last (an atomic ticket per output block) adds the partial outputs in the order of the
// shares and writes Y, which keeps the result independent of the arrival order.  Nobody waits for
// anybody: every workgroup stores, takes a ticket and leaves, or finds it is last and finishes.
#include <mutex>

#include "wino_internal.h"
#include "transforms.h"

namespace wino {

typedef float floatx16_t __attribute__((ext_vector_type(16)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));

constexpr int F2_K = 32, F2_P = 64, F2_C = 8, F2_T = 256;     // filters, tiles, channels per step, threads
constexpr int F2_U_FLOATS = 16 * (F2_C / 2) * F2_K * 2;       // transformed filters of a step
constexpr int F2_V_FLOATS = 16 * (F2_C / 2) * F2_P * 2;       // transformed tiles of a step
constexpr int F2_BT = 8;                                      // the 64 tiles are an 8 x 8 block of one image
constexpr int F2_PR = 2 * F2_BT + 2;                          // rows and columns of the input patch under it
constexpr int F2_RS = 20;                                     // LDS row stride of the patch (even: 8-byte tap reads)
constexpr int F2_PATCH = F2_C * F2_PR * F2_PR;                // patch elements of a step (2592)
constexpr int F2_R_FLOATS = F2_C * F2_PR * F2_RS;             // one patch buffer in LDS
constexpr int F2_NLD = (F2_PATCH + F2_T - 1) / F2_T;          // patch elements per thread (11, the last for 32 threads)
constexpr int F2_T_FLOATS = 4 * 2 * F2_K * 32;                // epilogue exchange of one tile block
constexpr int F2_MAX_BLOCKS = 4096;                           // output blocks a split launch may have
static_assert(F2_T_FLOATS <= F2_U_FLOATS + F2_V_FLOATS, "the epilogue reuses the operand area");

constexpr int F2_SLOTS = 8;                                   // streams that may run split launches

// Arrival counters of the output blocks of a split launch.  Zero when the library is loaded; the
// workgroup that finishes a block sets its counter back to zero, so every launch starts from zero.
// Launches on one stream run one after the other and share a set of counters; every stream that
// asks for a split launch is given a set of its own (f2_ticket_slot), so launches that overlap on
// one GPU never meet in a counter.  A ninth stream gets none and its layers run unsplit.
static __device__ unsigned int f2_tickets[F2_SLOTS * F2_MAX_BLOCKS];

// Partial outputs travel between workgroups, which may sit on different XCDs with separate L2
// caches.  They are written and read with agent-scope atomic accesses (relaxed, 8 bytes): such a
// store goes through to the level all XCDs share and such a load reads from there, so the
// hand-over needs no write-back or invalidation of a whole L2, which an agent-scope fence costs
// on this chip (several hundred nanoseconds per workgroup, serialised).  Order comes from the
// memory counter of each wavefront: a store counts in vmcnt until the level that serves its scope
// has acknowledged it -- for an sc1 store, the memory side all XCDs share -- so every wavefront
// waits for vmcnt(0) (f2_wait_stores) before the barrier that precedes the ticket: when the
// ticket is taken, every partial output of this workgroup is where any other XCD's sc1 load will
// find it.  The loads of the finishing workgroup are issued after the barrier that follows its
// ticket, which it can only see as last after all other shares have taken theirs.
__device__ __forceinline__ void f2_st_agent(float *p, float a, float b)
{
    const floatx2_t v = {a, b};
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), __builtin_bit_cast(unsigned long long, v),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ floatx2_t f2_ld_agent(const float *p)
{
    const unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
    return __builtin_bit_cast(floatx2_t, u);
}

// Waits until every vector-memory access of this wavefront, stores included, has been acknowledged.
__device__ __forceinline__ void f2_wait_stores()
{
    __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0); expcnt and lgkmcnt left alone
}

// Writes the rows and columns of the 2 x 2 output of tile (tx, ty) that are inside the image.
__device__ __forceinline__ void f2_store(const Geo &g, float *Y, int k, int img, int tx, int ty, floatx4_t y)
{
    float *dst = Y + (((size_t)img * g.K + k) * g.Ho + 2 * tx) * g.Wo + 2 * ty;
    const bool row1 = 2 * tx + 1 < g.Ho, col1 = 2 * ty + 1 < g.Wo;
    if (col1 && (g.Wo & 1) == 0) {
        *reinterpret_cast<floatx2_t *>(dst) = floatx2_t{y[0], y[1]};
        if (row1) *reinterpret_cast<floatx2_t *>(dst + g.Wo) = floatx2_t{y[2], y[3]};
    } else {
        dst[0] = y[0];
        if (col1) dst[1] = y[1];
        if (row1) {
            dst[g.Wo] = y[2];
            if (col1) dst[g.Wo + 1] = y[3];
        }
    }
}

// Barrier that orders LDS traffic only: global loads requested earlier stay in flight across it
// (__syncthreads() would wait for them too and undo the prefetch).
__device__ __forceinline__ void f2_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// BWD: the layer is the input gradient (Section 4.2 of the paper): its filter (k, c) is filter
// (c, k) of the stored G[C][K][3][3], rotated by 180 degrees.
// Two workgroups per CU (at most 256 registers per lane), so that one can multiply while the other
// waits for memory or for its barrier.
template <bool BWD>
__global__ __launch_bounds__(F2_T, 2) void fused_f2_kernel(const float *__restrict__ D, const float *__restrict__ G,
                                                           float *Y, float *part, Geo g, int n_kb, int n_tb,
                                                           int splits, int steps_per_split, int slot)
{
    __shared__ float smem[F2_U_FLOATS + F2_V_FLOATS + 2 * F2_R_FLOATS];
    __shared__ int s_last;
    float *Us = smem;
    float *Vs = smem + F2_U_FLOATS;
    float *Rs = smem + F2_U_FLOATS + F2_V_FLOATS;

    const int bid = blockIdx.x;
    const int kb = bid % n_kb;
    const int rest = bid / n_kb;
    const int sp = rest % splits, tb = rest / splits;
    const int k0 = kb * F2_K;
    const int nby = (g.Tw + F2_BT - 1) / F2_BT, nbx = (g.Th + F2_BT - 1) / F2_BT;
    const int by = tb % nby, bx = (tb / nby) % nbx, img = tb / (nby * nbx);
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int nsteps = (g.C + F2_C - 1) / F2_C;
    const int step_lo = sp * steps_per_split;
    const int step_hi = min(step_lo + steps_per_split, nsteps);
    const int nblk = (F2_BT * bx + F2_BT / 2 < g.Th) ? 2 : 1;       // MFMA column blocks that hold tiles
    // first channel the LDS slots of a step hold: the last step ends at the last channel
    auto first_channel = [&](int step) { return step == nsteps - 1 ? max(g.C - F2_C, 0) : step * F2_C; };

    // ---- loader role: patch elements tid, tid + 256, ... of [channel slot][row][column] ------------
    const size_t plane = (size_t)g.H * g.W;
    unsigned loff[F2_NLD];          // element offset from the first channel of the step, clamped into the image
    int lidx[F2_NLD];               // LDS index inside a patch buffer
    unsigned lmask = 0;             // bit n: element n is inside the image
    {
        const int x0 = 2 * F2_BT * bx - g.pad, y0 = 2 * F2_BT * by - g.pad;
#pragma unroll
        for (int n = 0; n < F2_NLD; ++n) {
            const int e = tid + n * F2_T;
            const bool e_ok = e < F2_PATCH;
            const int ee = e_ok ? e : 0;
            const int c = ee / (F2_PR * F2_PR), rem = ee % (F2_PR * F2_PR);
            const int r = rem / F2_PR, q = rem % F2_PR;
            const int x = x0 + r, y = y0 + q;
            if (e_ok && x >= 0 && x < g.H && y >= 0 && y < g.W) lmask |= 1u << n;
            loff[n] = (unsigned)min(c, g.C - 1) * (unsigned)(g.H * g.W) +
                      (unsigned)(min(max(x, 0), g.H - 1) * g.W + min(max(y, 0), g.W - 1));
            lidx[n] = (c * F2_PR + r) * F2_RS + q;
        }
    }
    const float *Dimg = D + (size_t)img * g.C * plane;
    // ---- filter role: filter kk of the block, channel slot cc of the step ---------------------------
    const int kk = tid >> 3, cc = tid & 7;
    const bool k_ok = k0 + kk < g.K;
    const int kc = min(k0 + kk, g.K - 1), ccl = min(cc, g.C - 1);
    const unsigned goff = BWD ? (unsigned)(ccl * g.K + kc) * 9u : (unsigned)(kc * g.C + ccl) * 9u;
    const size_t gchan = BWD ? (size_t)g.K * 9 : (size_t)9;        // elements from one channel to the next
    // ---- tile role of the data transform: tile (ti, tj) of the block, channel slots 2 wave, 2 wave + 1
    const int ti = lane >> 3, tj = lane & 7;

    float raw[F2_NLD], rg[9];
    auto load_patch = [&](int step) {
        const float *pc = Dimg + (size_t)first_channel(step) * plane;
#pragma unroll
        for (int n = 0; n < F2_NLD; ++n) raw[n] = pc[loff[n]];
    };
    auto store_patch = [&](float *Rb) {
#pragma unroll
        for (int n = 0; n < F2_NLD; ++n)
            if (n + 1 < F2_NLD || tid < F2_PATCH - (F2_NLD - 1) * F2_T) Rb[lidx[n]] = ((lmask >> n) & 1u) ? raw[n] : 0.0f;
    };
    auto load_filter = [&](int step) {
        const float *pg = G + (size_t)first_channel(step) * gchan;
#pragma unroll
        for (int j = 0; j < 9; ++j) rg[j] = pg[goff + (BWD ? 8 - j : j)];
    };
    auto transform = [&](const float *Rb, int step) {
        // v = B^T d B of one tile in two channels, stored as a channel pair
        float v[2][16];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const float *src = Rb + ((2 * wave + h) * F2_PR + 2 * ti) * F2_RS + 2 * tj;
            float d[4][4], t[4][4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const floatx2_t lo = *reinterpret_cast<const floatx2_t *>(src + p * F2_RS);
                const floatx2_t hi = *reinterpret_cast<const floatx2_t *>(src + p * F2_RS + 2);
                d[p][0] = lo[0], d[p][1] = lo[1], d[p][2] = hi[0], d[p][3] = hi[1];
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float col[4] = {d[0][j], d[1][j], d[2][j], d[3][j]};
                float o[4];
                bt_mul<2>(col, o);
#pragma unroll
                for (int p = 0; p < 4; ++p) t[p][j] = o[p];
            }
#pragma unroll
            for (int p = 0; p < 4; ++p) bt_mul<2>(t[p], &v[h][4 * p]);
        }
        float *vd = Vs + ((size_t)wave * F2_P + lane) * 2;
#pragma unroll
        for (int e = 0; e < 16; ++e)
            *reinterpret_cast<floatx2_t *>(vd + (size_t)e * (4 * F2_P * 2)) = floatx2_t{v[0][e], v[1][e]};
        // u = G g G^T of one filter; zero for filters past K, channels past C and channels an
        // earlier step has already added
        const int c = first_channel(step) + cc;
        const bool f_ok = k_ok && c >= step * F2_C && c < g.C;
        float t[4][3], u[4][4];
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            const float col[3] = {f_ok ? rg[j] : 0.0f, f_ok ? rg[3 + j] : 0.0f, f_ok ? rg[6 + j] : 0.0f};
            float o[4];
            g_mul<2>(col, o);
#pragma unroll
            for (int p = 0; p < 4; ++p) t[p][j] = o[p];
        }
#pragma unroll
        for (int p = 0; p < 4; ++p) g_mul<2>(t[p], u[p]);
        float *ud = Us + ((size_t)(cc >> 1) * F2_K + kk) * 2 + (cc & 1);
#pragma unroll
        for (int e = 0; e < 16; ++e) ud[(size_t)e * (4 * F2_K * 2)] = u[e >> 2][e & 3];
    };

    // ---- multiply-phase role ---------------------------------------------------------------------
    const int li = lane & 31, lh = lane >> 5;
    floatx16_t acc[4][2];
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[e][q][r] = 0.0f;

    // Operands of one component: filter pairs a[j], tile pairs of the two blocks bl[j], bh[j].
    struct Ops {
        floatx2_t a[2], bl[2], bh[2];
    };
    auto read_ops = [&](Ops &o, int e) {
        const int comp = wave * 4 + e;
        const float *ua = Us + (size_t)comp * (4 * F2_K * 2) + (lh * F2_K + li) * 2;
        const float *va = Vs + (size_t)comp * (4 * F2_P * 2) + (lh * F2_P + li) * 2;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            o.a[j] = *reinterpret_cast<const floatx2_t *>(ua + j * (2 * F2_K * 2));
            o.bl[j] = *reinterpret_cast<const floatx2_t *>(va + j * (2 * F2_P * 2));
            o.bh[j] = *reinterpret_cast<const floatx2_t *>(va + j * (2 * F2_P * 2) + 32 * 2);
        }
    };
    auto multiply = [&]() {
        // Both tile blocks always: a block without tiles holds zeros and costs no extra time, since
        // other workgroups of the launch multiply two blocks anyway.  The operands of the next
        // component are requested before the MFMAs of the current one, so that the LDS latency
        // is paid once per step and not once per component.
        Ops o[2];
        read_ops(o[0], 0);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (e + 1 < 4) read_ops(o[(e + 1) & 1], e + 1);
            __builtin_amdgcn_sched_barrier(0);      // keep the reads ahead of the MFMAs below
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    acc[e][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(o[e & 1].a[j][h], o[e & 1].bl[j][h], acc[e][0], 0, 0, 0);
                    acc[e][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(o[e & 1].a[j][h], o[e & 1].bh[j][h], acc[e][1], 0, 0, 0);
                }
        }
    };
    load_patch(step_lo);
    load_filter(step_lo);
    store_patch(Rs);
    if (step_lo + 1 < step_hi) load_patch(step_lo + 1);
    f2_lds_barrier();
    for (int step = step_lo; step < step_hi; ++step) {
        float *Rcur = Rs + ((step - step_lo) & 1) * F2_R_FLOATS, *Rnext = Rs + ((step - step_lo + 1) & 1) * F2_R_FLOATS;
        transform(Rcur, step);
        if (step + 1 < step_hi) store_patch(Rnext);          // requested during the previous multiply phase
        f2_lds_barrier();
        if (step + 2 < step_hi) load_patch(step + 2);          // both arrive while the MFMAs run
        if (step + 1 < step_hi) load_filter(step + 1);
        multiply();
        f2_lds_barrier();
    }

    // ---- inverse transform -----------------------------------------------------------------------
    // Accumulator register r of lane (li, lh) is filter 8 (r / 4) + 4 lh + r % 4, tile li of the block.
    float *Ts = smem;                           // [xi][q][filter 32][tile 32]
    const int ot = tid & 31, okq = tid >> 5;
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
        if (blk == nblk) break;               // the same for the whole workgroup
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float mrow[4] = {acc[0][blk][r], acc[1][blk][r], acc[2][blk][r], acc[3][blk][r]};
            float t[2];
            at_mul<2>(mrow, t);
            const int kr = 8 * (r >> 2) + 4 * lh + (r & 3);
            Ts[((wave * 2 + 0) * F2_K + kr) * 32 + li] = t[0];
            Ts[((wave * 2 + 1) * F2_K + kr) * 32 + li] = t[1];
        }
        __syncthreads();
        const int tx = F2_BT * bx + blk * 4 + (ot >> 3), ty = F2_BT * by + (ot & 7);
        const bool t_ok = tx < g.Th && ty < g.Tw;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int kr = okq + 8 * i;
            floatx4_t y;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const float col[4] = {Ts[((0 * 2 + q) * F2_K + kr) * 32 + ot], Ts[((1 * 2 + q) * F2_K + kr) * 32 + ot],
                                      Ts[((2 * 2 + q) * F2_K + kr) * 32 + ot], Ts[((3 * 2 + q) * F2_K + kr) * 32 + ot]};
                float o[2];
                at_mul<2>(col, o);
                y[q] = o[0];
                y[2 + q] = o[1];
            }
            if (splits == 1) {
                if (t_ok && k0 + kr < g.K) f2_store(g, Y, k0 + kr, img, tx, ty, y);
            } else if (t_ok && k0 + kr < g.K) {
                const size_t blockno = ((size_t)sp * n_tb + tb) * n_kb + kb;
                float *dst = part + ((blockno * F2_K + kr) * F2_P + blk * 32 + ot) * 4;
                f2_st_agent(dst, y[0], y[1]);
                f2_st_agent(dst + 2, y[2], y[3]);
            }
        }
        __syncthreads();
    }
    if (splits == 1) return;

    // ---- the last share to arrive adds the partial outputs ---------------------------------------
    unsigned int *const ticket = &f2_tickets[slot * F2_MAX_BLOCKS + tb * n_kb + kb];
    f2_wait_stores();                         // this wavefront's partial outputs have been acknowledged ...
    __syncthreads();                          // ... and so have those of the other three
    if (tid == 0)
        s_last = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (unsigned)(splits - 1);
    __syncthreads();
    if (!s_last) return;
    for (int idx = tid; idx < F2_K * 32 * nblk; idx += F2_T) {
        const int tile = idx % (32 * nblk), kr = idx / (32 * nblk);
        const int tx = F2_BT * bx + (tile >> 3), ty = F2_BT * by + (tile & 7);
        if (tx >= g.Th || ty >= g.Tw || k0 + kr >= g.K) continue;
        const size_t sstride = (size_t)n_tb * n_kb * F2_K * F2_P * 4;
        const float *ps = part + ((((size_t)tb * n_kb + kb) * F2_K + kr) * F2_P + tile) * 4;
        floatx4_t y = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int s0 = 0; s0 < splits; s0 += 8) {          // eight shares in flight, added in order
            floatx2_t lo[8], hi[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (s0 + u < splits) {
                    lo[u] = f2_ld_agent(ps + (size_t)(s0 + u) * sstride);
                    hi[u] = f2_ld_agent(ps + (size_t)(s0 + u) * sstride + 2);
                }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (s0 + u < splits) y += floatx4_t{lo[u][0], lo[u][1], hi[u][0], hi[u][1]};
        }
        f2_store(g, Y, k0 + kr, img, tx, ty, y);
    }
    if (tid == 0) __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Tile blocks of the layer: 8 x 8 tiles of one image each.
static long long f2_tile_blocks(const Geo &g)
{
    return (long long)g.N * ((g.Th + F2_BT - 1) / F2_BT) * ((g.Tw + F2_BT - 1) / F2_BT);
}

bool fused_f2_eligible(const Geo &g)
{
    // 32-bit element offsets inside an image and into G; the grid holds at most 2^31 - 1 workgroups
    return g.dt == WINO_F32 && g.m == 2 && (long long)g.C * g.H * g.W < (1LL << 31) &&
           (long long)g.K * g.C * 9 < (1LL << 31) && (long long)(g.Kp / F2_K) * f2_tile_blocks(g) <= 0x3fffffffLL;
}

// Channel shares: enough workgroups for two per CU where the channel loop allows it, every share at
// least one step, output blocks within the ticket array, partial outputs within the workspace.
static void f2_plan(const Geo &g, size_t workspace_bytes, bool may_split, int *splits, int *per)
{
    const long long base = (long long)(g.Kp / F2_K) * f2_tile_blocks(g);
    const int nsteps = (g.C + F2_C - 1) / F2_C;
    long long s = 1;
    if (base < 192) s = (512 + base - 1) / base < 16 ? (512 + base - 1) / base : 16;
    const long long fit = (long long)(workspace_bytes / ((size_t)base * F2_K * F2_P * 4 * sizeof(float)));
    if (s > fit) s = fit;
    if (s > nsteps) s = nsteps;
    if (s < 2 || base > F2_MAX_BLOCKS || !may_split) s = 1;
    *per = (int)((nsteps + s - 1) / s);
    *splits = (nsteps + *per - 1) / *per;
}

// The set of arrival counters of stream `s`: the first F2_SLOTS streams that ask get one each, for as long as
// the library is loaded; -1 for any further stream.
static int f2_ticket_slot(hipStream_t s)
{
    static std::mutex mu;
    static hipStream_t owner[F2_SLOTS];
    static int used = 0;
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < used; ++i)
        if (owner[i] == s) return i;
    if (used == F2_SLOTS) return -1;
    owner[used] = s;
    return used++;
}

hipError_t launch_fused_f2(const Geo &g, const float *D, const float *G, float *Y, void *workspace,
                           size_t workspace_bytes, bool bwd, hipStream_t s)
{
    const int n_kb = g.Kp / F2_K, n_tb = (int)f2_tile_blocks(g);
    int splits, per;
    f2_plan(g, workspace_bytes, true, &splits, &per);
    int slot = 0;
    if (splits > 1 && (slot = f2_ticket_slot(s)) < 0) {
        f2_plan(g, workspace_bytes, false, &splits, &per);
        slot = 0;
    }
    const long long blocks = (long long)n_kb * n_tb * splits;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (bwd)
        fused_f2_kernel<true><<<dim3((unsigned)blocks), dim3(F2_T), 0, s>>>(D, G, Y, (float *)workspace, g, n_kb, n_tb,
                                                                            splits, per, slot);
    else
        fused_f2_kernel<false><<<dim3((unsigned)blocks), dim3(F2_T), 0, s>>>(D, G, Y, (float *)workspace, g, n_kb, n_tb,
                                                                             splits, per, slot);
    return hipGetLastError();
}

}  // namespace wino

// All of Algorithm 1 after the filter transform in one kernel (Lavin & Gray, Section 6 describes
// the same fusion for F(2x2,3x3) on Maxwell): tile gather and data transform, the alpha^2
// products of Eq. (13) reduced over channels, and the inverse transform of Eq. (10), with
// neither V nor M ever written to memory.  F(4x4,3x3), fp32.  This is a gfx950 design:
//
//  * MFMA shape v_mfma_f32_16x16x4_f32.  Its B operand wants, in lane l, element
//    [channel l/16][tile l%16]: one (channel, tile) pair per lane.  So a lane transforms the
//    6 x 6 input tile of ITS channel and ITS tile in registers (v = B^T d B) and the results are
//    at once the B operands of the MFMAs of this step: V exists only in registers.
//  * Its accumulator puts rows 4*(l/16)..+3 of column l%16 in lane l, so after the channel loop
//    a lane holds the components m_{k,b} of 4 filters x 1 tile per 16 x 16 block and the inverse
//    transform Y = A^T m A runs in registers.
//  * 36 components x (32 filters x 16 tiles) is 288 accumulator registers, more than the 256
//    AccVGPRs.  So two wavefronts share a block and split the components by row: one takes
//    xi = 0..2, the other xi = 3..5 (18 components, 144 accumulators each).  Each computes only
//    its three rows of B^T d (half the transform) and, at the end, its part of A^T m A; the two
//    partial 4 x 4 outputs are added through LDS.  That leaves room for two wavefronts per SIMD,
//    so one wavefront's transform arithmetic overlaps the other's MFMAs.
//  * Raw input taps and transformed filters reach LDS by direct global->LDS loads (no registers),
//    one channel step ahead (filters) and three ahead (taps).  Zero padding is implicit: a tap
//    outside the image is fetched with a buffer offset beyond the buffer, for which the
//    hardware delivers 0.
//
// A workgroup of 8 wavefronts owns FK = 64 filters x FP = 32 tiles:
// wave = (k half wm) * 4 + (tile group wn) * 2 + (component half h).
#include <stdlib.h>

#include <mutex>

#include "wino_internal.h"
#include "transforms.h"

namespace wino {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int FK = 64;  // filters per workgroup
constexpr int FP = 32;  // tiles per workgroup
constexpr int FC = 4;   // channels per step (the depth of one MFMA)
constexpr unsigned OOB = 0x80000000u;  // byte offset beyond any admissible input tensor

#define WINO_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define WINO_GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

__device__ __forceinline__ int xcd_remap_f(int bid, int nblocks)
{
    constexpr int XCDS = 8;
    const int per = nblocks / XCDS;
    if (bid >= per * XCDS) return bid;
    return (bid % XCDS) * per + bid / XCDS;
}

// three rows of B^T (Eq. (15)) applied to a column of 6: rows 0..2 (HALF 0) or 3..5 (HALF 1)
template <int HALF> __device__ __forceinline__ void bt_half(const float *d, float *o)
{
    if constexpr (HALF == 0) {
        const float s42 = d[4] - 4.0f * d[2], s31 = d[3] - 4.0f * d[1];
        o[0] = 4.0f * d[0] - 5.0f * d[2] + d[4];
        o[1] = s42 + s31;
        o[2] = s42 - s31;
    } else {
        const float t42 = d[4] - d[2], t31 = 2.0f * (d[3] - d[1]);
        o[0] = t42 + t31;
        o[1] = t42 - t31;
        o[2] = 4.0f * d[1] - 5.0f * d[3] + d[5];
    }
}

// the columns 0..2 (HALF 0) or 3..5 (HALF 1) of A^T (Eq. (15)) applied to three values
template <int HALF> __device__ __forceinline__ void at_half(float t0, float t1, float t2, float *o)
{
    if constexpr (HALF == 0) {
        o[0] = t0 + t1 + t2;
        o[1] = t1 - t2;
        o[2] = t1 + t2;
        o[3] = t1 - t2;
    } else {
        const float p = t0 + t1, m = t0 - t1;
        o[0] = p;
        o[1] = 2.0f * m;
        o[2] = 4.0f * p;
        o[3] = 8.0f * m + t2;
    }
}

struct FusedLane {
    int wave, lane, h, wn, wm, t16, cs;
    int kb, img, tx, ty;
    bool tile_ok;
};

template <int HALF, int PHASE, bool RAGGED, bool CPAD>
__device__ __forceinline__ void fused_body(const float *__restrict__ D, const float *__restrict__ U,
                                           float *__restrict__ Y, const Geo &g, unsigned d_bytes,
                                           const FusedLane &L, float *lds)
{
    constexpr int M = 4, A = 6, A2 = 36, HC = 18;
    constexpr int SLAB = A2 * FC * FK;   // floats of transformed filters per step
    constexpr int RROW = 64 * A;         // one tile row of a raw stage: [q=0: 64][q=1..4: 64 x 4][q=5: 64]
    constexpr int RSTAGE = A * RROW;     // floats per (tile group, stage)
    float *const ulds = lds;                                   // [2][SLAB]
    float *const rlds = lds + 2 * SLAB + L.wn * (3 * RSTAGE);  // this tile group: [3][RSTAGE]

    const int lane = L.lane, cs = L.cs, t16 = L.t16;
    const int x0 = M * L.tx - g.pad, y0 = M * L.ty - g.pad;
    const int HW = g.H * g.W;
    const int S = g.Cp / FC;  // channel steps; channels >= C have zero filters in U
    const unsigned step_bytes = (unsigned)(FC * HW) * 4u;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)D, 0, d_bytes, 0x00020000);

    // ---- raw taps: a tile row is fetched as {q=0 (4 B), q=1..4 (16 B), q=5 (4 B)} per lane.  The
    //      four wavefronts of a tile group each fetch two rows: rows 0-1, 2-3, 4-4, 5-5 (the last
    //      two fetch their row twice, which keeps the loop free of wave-dependent branches). ------
    const int idx4 = L.wm * 2 + L.h;
    const int rrow[2] = {(idx4 < 2) ? 2 * idx4 : idx4 + 2, (idx4 < 2) ? 2 * idx4 + 1 : idx4 + 2};
    unsigned rvoff[2][3];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int part = 0; part < 3; ++part) {
            const int x = x0 + rrow[i];
            const int y = (part == 0) ? y0 : (part == 1) ? y0 + 1 : y0 + 5;
            const bool ok = L.tile_ok && x >= 0 && x < g.H && y >= 0 && y < g.W;
            rvoff[i][part] = ok ? (unsigned)((L.img * g.C + cs) * HW + x * g.W + y) * 4u : OOB;
        }
    auto load_raw = [&](int st, int s) {
        const unsigned so = (unsigned)s * step_bytes;
        const bool ch_ok = !CPAD || (s * FC + cs < g.C);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            float *dst = rlds + st * RSTAGE + rrow[i] * RROW;
#pragma unroll
            for (int part = 0; part < 3; ++part) {
                unsigned vo = rvoff[i][part];
                if (CPAD) vo = (ch_ok && vo != OOB) ? vo + so : OOB;  // bounds check sees the whole address
                if (part == 0)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, WINO_LDS_PTR(dst), 4, vo, CPAD ? 0u : so, 0, 0);
                else if (part == 1)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, WINO_LDS_PTR(dst + 64), 16, vo, CPAD ? 0u : so, 0, 0);
                else
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, WINO_LDS_PTR(dst + 64 + 256), 4, vo, CPAD ? 0u : so, 0,
                                                             0);
            }
        }
    };
    // columns that may lie outside the image when the 4-wide run overhangs the row (RAGGED only)
    bool cv[A];
#pragma unroll
    for (int q = 0; q < A; ++q) cv[q] = (y0 + q >= 0) && (y0 + q < g.W);

    // LDS stage -> registers (the 36 raw taps of this lane's tile and channel)
    auto load_taps = [&](float (&d)[A2], int st) {
        const float *src = rlds + st * RSTAGE;
#pragma unroll
        for (int p = 0; p < A; ++p) {
            const floatx4 mid = *reinterpret_cast<const floatx4 *>(src + p * RROW + 64 + lane * 4);
            d[p * A + 0] = src[p * RROW + lane];
            d[p * A + 1] = mid[0];
            d[p * A + 2] = mid[1];
            d[p * A + 3] = mid[2];
            d[p * A + 4] = mid[3];
            d[p * A + 5] = src[p * RROW + 64 + 256 + lane];
        }
    };
    // this wavefront's three rows of v = B^T d B
    auto transform = [&](float (&v)[HC], float (&d)[A2]) {
        float t[3][A];
        if (RAGGED) {
#pragma unroll
            for (int p = 0; p < A; ++p)
#pragma unroll
                for (int q = 1; q < 5; ++q) d[p * A + q] = cv[q] ? d[p * A + q] : 0.0f;
        }
#pragma unroll
        for (int q = 0; q < A; ++q) {
            float col[A], o[3];
#pragma unroll
            for (int p = 0; p < A; ++p) col[p] = d[p * A + q];
            bt_half<HALF>(col, o);
            t[0][q] = o[0];
            t[1][q] = o[1];
            t[2][q] = o[2];
        }
#pragma unroll
        for (int i = 0; i < 3; ++i) bt_mul<M>(t[i], &v[i * A]);
    };

    // ---- transformed filters: direct global -> LDS; load n of this wavefront is component
    //      wave + 8n.  LDS slab: [e][channel 0..3][64 filters], the four 16-filter groups of odd
    //      channel rows pairwise swapped so that the A-operand reads spread over all banks. ------
    const int f4 = lane & 15;
    const int ucol = min(L.kb * FK + (((f4 >> 2) ^ (cs & 1)) << 4) + ((f4 & 3) << 2), g.Kp - 4);
    const size_t e_stride = (size_t)g.Cp * g.Kp;
    const size_t s_stride = (size_t)FC * g.Kp;
    // component of load n: wave + 8n, the last one clamped to 35 (waves 4..7 fetch it redundantly)
    const int e_last = min(L.wave + 32, A2 - 1);
    const float *usrc = U + (size_t)cs * g.Kp + ucol + (size_t)L.wave * e_stride;
    const float *usrc_last = U + (size_t)cs * g.Kp + ucol + (size_t)e_last * e_stride;
    float *const udst = ulds + L.wave * (FC * FK);
    float *const udst_last = ulds + e_last * (FC * FK);
    auto load_u = [&](int buf, int s) {
        const float *src = usrc + (size_t)s * s_stride;
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            __builtin_amdgcn_global_load_lds(WINO_GLB_PTR(src), WINO_LDS_PTR(udst + buf * SLAB + n * 8 * (FC * FK)), 16, 0,
                                             0);
            src += 8 * e_stride;
        }
        __builtin_amdgcn_global_load_lds(WINO_GLB_PTR(usrc_last + (size_t)s * s_stride),
                                         WINO_LDS_PTR(udst_last + buf * SLAB), 16, 0, 0);
    };
    // A operand of lane (cs, t16): filter row t16 of 16-filter group wm*2 + j, channel cs
    const int a_lane0 = HALF * HC * (FC * FK) + cs * FK + (((L.wm * 2 + 0) ^ (cs & 1)) << 4) + t16;
    const int a_lane1 = HALF * HC * (FC * FK) + cs * FK + (((L.wm * 2 + 1) ^ (cs & 1)) << 4) + t16;

    floatx4 acc[HC][2];
#pragma unroll
    for (int e = 0; e < HC; ++e) {
        acc[e][0] = floatx4{0.f, 0.f, 0.f, 0.f};
        acc[e][1] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
    auto load_a = [&](float (&a0)[HC], float (&a1)[HC], int buf) {
        const float *as = ulds + buf * SLAB;
#pragma unroll
        for (int e = 0; e < HC; ++e) {
            a0[e] = as[e * (FC * FK) + a_lane0];
            a1[e] = as[e * (FC * FK) + a_lane1];
        }
    };
    auto mma_step = [&](const float (&v)[HC], const float (&a0)[HC], const float (&a1)[HC]) {
#pragma unroll
        for (int e = 0; e < HC; ++e) {
            acc[e][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0[e], v[e], acc[e][0], 0, 0, 0);
            acc[e][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1[e], v[e], acc[e][1], 0, 0, 0);
        }
    };

    // ---- channel loop.  During step s: MFMAs on v(s); v(s+1) is made from raw stage (s+1)%3;
    //      the filters of step s+1 and the taps of step s+3 stream into LDS.  At the end of a
    //      step everything but the taps issued in that step must have landed.  The two wavefronts
    //      that share a SIMD (same wn and h, different wm) run the MFMA block and the transform
    //      block in opposite order, so that one's MFMAs overlap the other's VALU work. -----------
    auto wait_all_but_new_taps = [&]() { __builtin_amdgcn_s_waitcnt(0x0f76); };  // vmcnt(6)
    float va[HC], vb[HC];
    load_u(0, 0);
    load_raw(0, 0);
    load_raw(1, min(1, S - 1));
    load_raw(2, min(2, S - 1));
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wavefront's loads have landed in LDS
    __syncthreads();
    {
        float d[A2];
        load_taps(d, 0);
        transform(va, d);
    }
    __syncthreads();  // stage 0 is free for the loads of step 0
    int st_w = 0, st_r = 1;  // raw stage written (s % 3) and read ((s + 1) % 3) in step s

    // All LDS reads of a block are issued before its arithmetic (the scheduling barriers keep
    // the compiler from sinking them next to their uses, which would expose the LDS latency
    // once per group of MFMAs instead of once per step).
#define WINO_FUSED_STEP(CUR, NXT, s)                                \
    {                                                               \
        float d[A2], a0[HC], a1[HC];                                \
        load_u(((s) + 1) & 1, min((s) + 1, S - 1));                 \
        load_raw(st_w, min((s) + 3, S - 1));                        \
        if constexpr (PHASE == 0) {                                 \
            load_a(a0, a1, (s) & 1);                                \
            load_taps(d, st_r);                                     \
            __builtin_amdgcn_sched_barrier(0);                      \
            mma_step(CUR, a0, a1);                                  \
            __builtin_amdgcn_sched_barrier(0);                      \
            transform(NXT, d);                                      \
        } else {                                                    \
            load_taps(d, st_r);                                     \
            __builtin_amdgcn_sched_barrier(0);                      \
            transform(NXT, d);                                      \
            load_a(a0, a1, (s) & 1);                                \
            __builtin_amdgcn_sched_barrier(0);                      \
            mma_step(CUR, a0, a1);                                  \
        }                                                           \
        wait_all_but_new_taps();                                    \
        __syncthreads();                                            \
        st_w = st_r;                                                \
        st_r = (st_r == 2) ? 0 : st_r + 1;                          \
    }
    for (int s = 0; s < S; s += 2) {  // S is a multiple of 4
        WINO_FUSED_STEP(va, vb, s)
        WINO_FUSED_STEP(vb, va, s + 1)
    }
#undef WINO_FUSED_STEP
    __builtin_amdgcn_s_waitcnt(0x0f70);  // the (redundant) last tap loads must not land in the exchange area
    __syncthreads();

    // ---- inverse transform: each wavefront turns its 18 components into a partial 4 x 4 output
    //      (rows xi of its half), the pair exchanges one 16-filter block each through LDS. --------
    auto partial_y = [&](int j, int r, float (&y)[16]) {
        float tt[3][M];
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            float row[A];
#pragma unroll
            for (int nu = 0; nu < A; ++nu) row[nu] = acc[i * A + nu][j][r];
            at_mul<M>(row, tt[i]);
        }
#pragma unroll
        for (int q = 0; q < M; ++q) {
            float o[M];
            at_half<HALF>(tt[0][q], tt[1][q], tt[2][q], o);
#pragma unroll
            for (int p = 0; p < M; ++p) y[p * M + q] = o[p];
        }
    };
    float *const xsend = lds + L.wave * (64 * 64);
    const float *const xrecv = lds + (L.wave ^ 1) * (64 * 64);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        float y[16];
        partial_y(1 - HALF, r, y);
#pragma unroll
        for (int i = 0; i < 16; ++i) xsend[(r * 16 + i) * 64 + lane] = y[i];
    }
    __syncthreads();
    if (!L.tile_ok) return;
    const int xo = M * L.tx, yo = M * L.ty;
    const bool vec_row = (g.Wo % M == 0);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int k = L.kb * FK + L.wm * 32 + HALF * 16 + cs * 4 + r;
        float y[16];
        partial_y(HALF, r, y);
#pragma unroll
        for (int i = 0; i < 16; ++i) y[i] += xrecv[(r * 16 + i) * 64 + lane];
        if (k >= g.K) continue;
        float *dst = Y + ((size_t)L.img * g.K + k) * g.Ho * g.Wo;
#pragma unroll
        for (int p = 0; p < M; ++p) {
            if (xo + p >= g.Ho) break;
            float *row = dst + (size_t)(xo + p) * g.Wo + yo;
            if (vec_row) {
                *reinterpret_cast<floatx4 *>(row) = floatx4{y[p * M], y[p * M + 1], y[p * M + 2], y[p * M + 3]};
            } else {
#pragma unroll
                for (int q = 0; q < M; ++q)
                    if (yo + q < g.Wo) row[q] = y[p * M + q];
            }
        }
    }
}

template <bool RAGGED, bool CPAD>
__global__ __launch_bounds__(512) void fused_f4_kernel(const float *__restrict__ D, const float *__restrict__ U,
                                                       float *__restrict__ Y, Geo g, int n_pt, unsigned d_bytes)
{
    extern __shared__ float lds[];
    FusedLane L;
    const int tid = threadIdx.x;
    L.wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform by construction: keep it scalar
    L.lane = tid & 63;
    L.h = L.wave & 1;
    L.wn = (L.wave >> 1) & 1;
    L.wm = L.wave >> 2;
    L.t16 = L.lane & 15;
    L.cs = L.lane >> 4;
    const int bid = xcd_remap_f(blockIdx.x, gridDim.x);
    const int pt = bid % n_pt;
    L.kb = bid / n_pt;
    const int b = pt * FP + L.wn * 16 + L.t16;
    L.tile_ok = b < g.P;
    const int bb = L.tile_ok ? b : 0;
    L.ty = bb % g.Tw;
    const int t2 = bb / g.Tw;
    L.tx = t2 % g.Th;
    L.img = t2 / g.Th;
    // four straight-line instances: component half x order of the MFMA and transform blocks
    if (L.h == 0) {
        if (L.wm == 0)
            fused_body<0, 0, RAGGED, CPAD>(D, U, Y, g, d_bytes, L, lds);
        else
            fused_body<0, 1, RAGGED, CPAD>(D, U, Y, g, d_bytes, L, lds);
    } else {
        if (L.wm == 0)
            fused_body<1, 0, RAGGED, CPAD>(D, U, Y, g, d_bytes, L, lds);
        else
            fused_body<1, 1, RAGGED, CPAD>(D, U, Y, g, d_bytes, L, lds);
    }
}

bool fused_eligible(const Geo &g)
{
    if (g.dt == WINO_F16) return fused_f16_eligible(g);
    if (g.dt != WINO_F32) return false;
    if (g.m == 2) return fused_wide_eligible(g);      // F(2x2): only the 64-filter design
    if (g.m != 4) return false;
    // 32-bit byte offsets into D below the out-of-bounds marker
    const unsigned long long bytes = (unsigned long long)g.N * g.C * g.H * g.W * 4ull;
    return bytes < (1ull << 31) - 65536;
}

// Where the one-kernel path beats the four-stage path (measured on MI355X at N = 64).  The one-kernel path
// repeats the data transform for every 32 filters, the four-stage path writes and re-reads V (C rows per tile) and
// M (K rows per tile): the first wins while K C / (K + C) is small -- 43 to 85 for the VGG layers with 64 to 128
// channels (1.15x to 2x faster), a tie at 128 (256 -> 256 channels), a loss from 170 up (256 -> 512) -- and there
// are enough workgroups to fill the 256 CUs.
bool fused_preferred(const Geo &g)
{
    if (!fused_eligible(g)) return false;
    const long long blocks = (long long)((g.P + FP - 1) / FP) * ((g.K + FK - 1) / FK);
    if (g.dt == WINO_F16)   // same crossover as in fp32 (N = 32: 128 -> 256 channels 0.139 vs 0.155 ms, 256 -> 256 0.249 vs 0.197)
        return (long long)g.K * g.C <= 100LL * (g.K + g.C) && (long long)((g.P + 31) / 32) * ((g.K + 63) / 64) >= 256;
    if (g.m == 2) {
        // F(2x2,3x3) in one kernel (fused_wide.hip) against its four stages, whose V and M are 4 values per output:
        // -58 % for 64 -> 64 channels at 224 x 224 (N = 32), -39 % for 128 -> 128 at 112 x 112, -22 % for 256 -> 256
        // at 56 x 56, -6 % for 512 -> 512 at 28 x 28 (all N = 64); 512 -> 512 at 14 x 14: -5 % at N = 64, -2 % at
        // N = 32, -11 % at N = 16 (392 items); 512 -> 512 at 28 x 28, N = 8 (784 items): -3 %.  Below some hundred
        // items the launch does not fill the GPU.
        const long long items = (long long)((g.P + 15) / 16) * ((g.Kp + 63) / 64);
        return (long long)g.K * g.C <= 256LL * (g.K + g.C) && items >= 384;
    }
    if (!fused_lds_eligible(g)) return g.K <= 128 && blocks >= 512;
    if ((long long)g.K * g.C <= 100LL * (g.K + g.C) && blocks >= 512) return true;
    // with 64 filters per workgroup (fused_wide.hip) the crossover moves up past 256 -> 256 channels (56 x 56: 0.59
    // against 0.73 ms at N = 64, 0.38 against 0.41 at N = 32, 0.21 against 0.22 at N = 16) and 256 -> 512 (28 x 28,
    // K C / (K + C) = 171: 0.32 against 0.36 ms at N = 64, 0.19 against 0.21 at N = 32, a tie at N = 16); 512 -> 512
    // (256) was a loss (0.71 against 0.65 ms) until the items of a partly filled last round were shared between
    // workgroups.  Since then it depends on how well the rounds are filled (fused_wide_fill): at 28 x 28, 512 -> 512
    // channels, -6 % at N = 64 (fill 0.93), -9 % at N = 40 (0.96), -3 % at N = 48 and 96 (0.88, 0.92), -6 % at
    // N = 128, but +9 % at N = 32 (0.77) and +3 % at N = 24 (0.80); 384 -> 384: -7 % at N = 64 (0.88), -2 % at
    // N = 32 (0.79); 512 -> 512 at 56 x 56: -1 to -6 % (0.92 to 0.97).
    const long long wide_items = (long long)((g.P + 15) / 16) * ((g.Kp + 63) / 64);
    // Three quarters of the resident workgroups suffice up to 175 (320 -> 320 at 28 x 28: -26 % with 490 items,
    // -12 % with 368; 384 -> 384: -8 % with 444; 512 -> 256: a tie with 392, +23 % with 296).
    if (fused_wide_eligible(g)) {
        // Up to 256 items every workgroup has a CU to itself: with 196 of them 64 -> 128 and 128 -> 128 channels at
        // 112 x 112 (N = 2), 128 -> 128 at 56 x 56 (N = 8) and 128 -> 256 (N = 4) run 20-23 % faster in one kernel
        // (104 items: 19 % slower; 296, where CUs begin to hold two: a tie).
        if ((long long)g.K * g.C <= 100LL * (g.K + g.C) && wide_items >= 192 && wide_items <= 256) return true;
        if ((long long)g.K * g.C <= 175LL * (g.K + g.C) && wide_items >= 384) return true;
        if ((long long)g.K * g.C <= 256LL * (g.K + g.C) && wide_items >= 512 && fused_wide_fill(g) >= 0.85) return true;
    }
    // small batches: with very few filters and channels (64 -> 64) one launch that does everything still beats
    // three launches as soon as it has a workgroup for every other CU (batch 1, 224 x 224: 32 vs 37 us)
    const long long items = (long long)((g.P + 31) / 32) * (g.Kp / 32);
    return (long long)g.K * g.C <= 32LL * (g.K + g.C) && items >= 128;
}

hipError_t launch_fused(const Geo &g, const void *Dv, const void *Uv, void *Yv, int y_dt, hipStream_t s)
{
    if (g.dt == WINO_F16) return launch_fused_f16(g, Dv, Uv, Yv, y_dt, s);
    if (y_dt != WINO_F32) return hipErrorNotSupported;
    float *Y = (float *)Yv;
    const float *D = (const float *)Dv, *U = (const float *)Uv;
    const int n_pt = (g.P + FP - 1) / FP, n_kb = (g.K + FK - 1) / FK;
    const long long blocks = (long long)n_pt * n_kb;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    // main loop: 2 filter slabs + 2 tile groups x 3 raw stages; epilogue: 8 x (64 x 64) exchange
    const size_t lds_bytes = 8ull * 64 * 64 * sizeof(float);
    static_assert(2 * 36 * FC * FK + 2 * 3 * 6 * 64 * 6 <= 8 * 64 * 64, "main-loop LDS fits the exchange area");
    const unsigned d_bytes = (unsigned)((size_t)g.N * g.C * g.H * g.W * 4);
    const bool ragged = !(g.pad == 1 && g.W % 4 == 0);
    // the channel loop runs over Cp (a multiple of 16): every step beyond C must be fetched as zeros, not
    // from whatever follows the channel planes of this image (the next image, or the end of the tensor)
    const bool cpad = g.Cp != g.C;
    static std::mutex attr_mutex;
    static bool attr_set = false;
    std::lock_guard<std::mutex> attr_lock(attr_mutex);
    if (!attr_set) {
        const void *fns[4] = {(const void *)fused_f4_kernel<false, false>, (const void *)fused_f4_kernel<false, true>,
                              (const void *)fused_f4_kernel<true, false>, (const void *)fused_f4_kernel<true, true>};
        for (const void *fn : fns) {
            hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
            if (e != hipSuccess) return e;
        }
        attr_set = true;
    }
    const dim3 grid((unsigned)blocks), block(512);
    if (!ragged && !cpad)
        fused_f4_kernel<false, false><<<grid, block, lds_bytes, s>>>(D, U, Y, g, n_pt, d_bytes);
    else if (!ragged)
        fused_f4_kernel<false, true><<<grid, block, lds_bytes, s>>>(D, U, Y, g, n_pt, d_bytes);
    else if (!cpad)
        fused_f4_kernel<true, false><<<grid, block, lds_bytes, s>>>(D, U, Y, g, n_pt, d_bytes);
    else
        fused_f4_kernel<true, true><<<grid, block, lds_bytes, s>>>(D, U, Y, g, n_pt, d_bytes);
    return hipGetLastError();
}

}  // namespace wino

// Loop 3 of Algorithm 1 (Lavin & Gray): the alpha^2 independent products
// M^(xi,nu) = U^(xi,nu) V^(xi,nu) (Eq. (13)), K x C by C x P each, on the MFMA units.
#include <stdlib.h>

#include "wino_internal.h"

namespace wino {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Maps the hardware workgroup id to a logical block id so that logically consecutive blocks run
// on the same XCD.  Workgroups are dealt to the 8 XCDs round-robin (id % 8) and each XCD has
// its own L2; consecutive logical blocks share an operand panel, so they should share an L2.
__device__ __forceinline__ int xcd_remap(int bid, int nblocks)
{
    constexpr int XCDS = 8;
    const int per = nblocks / XCDS;            // blocks in the evenly divisible part
    if (bid >= per * XCDS) return bid;         // ragged remainder keeps its id
    return (bid % XCDS) * per + bid / XCDS;
}

// 16 bytes per lane from a buffer straight into LDS: lane l of the wavefront fills LDS bytes lds + 16 l ..
// (lds the same in all lanes).  Written as assembly on purpose: while a copy into LDS that the compiler knows of
// may be in flight, it puts a wait for ALL outstanding memory requests in front of every LDS read, which would
// serialise the copy of the next slab with the multiply of the current one.  The kernel waits for its copies itself.
typedef int intx4_g __attribute__((ext_vector_type(4)));
#define WINO_G_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
__device__ __forceinline__ intx4_g gemm_buffer(const void *base, unsigned bytes)
{
    const unsigned long long a = (unsigned long long)base;
    return intx4_g{__builtin_amdgcn_readfirstlane((int)(unsigned)a),
                   __builtin_amdgcn_readfirstlane((int)((unsigned)(a >> 32) & 0xffffu)),
                   __builtin_amdgcn_readfirstlane((int)bytes), 0x00020000};
}
__device__ __forceinline__ void gemm_copy16_to_lds(intx4_g rsrc, unsigned lds, unsigned voffset, unsigned soffset)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds), "v"(voffset), "s"(rsrc), "s"(soffset)
                 : "memory");   // (m0 is not a register the compiler keeps values in)
}

// fp32 operands, v_mfma_f32_32x32x2_f32.  A workgroup of WM x WN wavefronts owns a BM x BN
// block of one M^(e); every wavefront owns TM x TN MFMA tiles of 32 x 32.  Both operands are
// stored reduction-index-major (U[e][c][k], V[e][c][b]), so a BK-deep slab is BK contiguous row
// segments: loaded with 16-byte accesses, kept in LDS as [c][k] / [c][b], and read by the MFMA
// lanes (lane = column + 32 * (c & 1)) without bank conflicts.
//
// Pipeline: two LDS slabs (slab t+1 is copied from memory straight into LDS while slab t is
// multiplied) and two register sets per wavefront holding half a slab of MFMA operands each,
// so LDS reads for the next half overlap the MFMAs of the current one; one barrier per slab.
//
// Blocks that overhang Kp or Pp load from clamped (valid) addresses: rows/columns of a product
// are independent, so whatever is loaded there only reaches outputs that are never stored.
template <int BM, int BN, int WM, int WN, int BK>
__global__ __launch_bounds__(64 * WM * WN) void gemm_f32_kernel(const float *__restrict__ U,
                                                                 const float *__restrict__ V,
                                                                 float *__restrict__ Mo, int Kp, int Cp, int Pp,
                                                                 int tiles_m, int tiles_n, int a2, int nk_split)
{
    constexpr int NT = 64 * WM * WN;
    constexpr int TM = BM / (32 * WM), TN = BN / (32 * WN);
    constexpr int A4 = BK * BM / 4, B4 = BK * BN / 4;  // float4s per slab
    static_assert(A4 % NT == 0 && B4 % NT == 0, "slab must divide evenly among the threads");
    static_assert(BK % 8 == 0, "two half-slabs of whole MFMA steps");
    constexpr int AL = A4 / NT, BL = B4 / NT;
    constexpr int HS = BK / 4;                          // MFMA steps (2 channels each) per half slab
    __shared__ float As[2][BK * BM];
    __shared__ float Bs[2][BK * BN];

    int bid = xcd_remap(blockIdx.x, gridDim.x);
    const int tm_i = bid % tiles_m;
    bid /= tiles_m;
    const int tn_i = bid % tiles_n;
    bid /= tiles_n;
    const int e = bid % a2;
    const int z = bid / a2;   // which share of the channel loop (layers with few blocks split it)
    const int k0 = tm_i * BM, p0 = tn_i * BN;
    const int c_first = z * nk_split * BK;

    const float *Ue = U + ((size_t)e * Cp + c_first) * Kp;
    const float *Ve = V + ((size_t)e * Cp + c_first) * Pp;
    float *Me = Mo + ((size_t)z * a2 + e) * Kp * Pp;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lg = lane >> 5;

    // Operands are fetched through buffers that start at this block's first channel row of U^(e) and V^(e): the
    // per-thread byte offsets are fixed for the kernel and the slab advances in a scalar register, so the loop holds
    // no 64-bit address arithmetic (one component's Cp x Kp or Cp x Pp floats stay below 4 GB: see the launcher).
    unsigned oa[AL], ob[BL];
#pragma unroll
    for (int j = 0; j < AL; ++j) {
        const int idx = tid + j * NT;
        const int row = idx / (BM / 4), col = min(k0 + (idx % (BM / 4)) * 4, Kp - 4);
        oa[j] = (unsigned)(row * Kp + col) * 4u;
    }
#pragma unroll
    for (int j = 0; j < BL; ++j) {
        const int idx = tid + j * NT;
        const int row = idx / (BN / 4), col = min(p0 + (idx % (BN / 4)) * 4, Pp - 4);
        ob[j] = (unsigned)(row * Pp + col) * 4u;
    }
    const int c_rows = Cp - c_first;
    const intx4_g rsrc_a = gemm_buffer(Ue, (unsigned)((size_t)c_rows * Kp * 4));
    const intx4_g rsrc_b = gemm_buffer(Ve, (unsigned)((size_t)c_rows * Pp * 4));
    unsigned sa = 0, sb = 0;                            // byte offset of the next slab
    // A slab goes from memory straight into LDS (16 bytes per lane, 1 KB contiguous per wavefront and request: the
    // order of the slab in LDS is the order of the threads' words).  No registers are involved, so the requests are
    // made a whole slab of MFMAs ahead of the barrier that publishes them.
    const unsigned wave_bytes = (unsigned)__builtin_amdgcn_readfirstlane(wave) * 1024u;   // (in a scalar register)
    const unsigned lds_a = (unsigned)(size_t)WINO_G_LDS_PTR(&As[0][0]) + wave_bytes;
    const unsigned lds_b = (unsigned)(size_t)WINO_G_LDS_PTR(&Bs[0][0]) + wave_bytes;
    auto request_slab = [&](int buf) {
#pragma unroll
        for (int j = 0; j < AL; ++j) gemm_copy16_to_lds(rsrc_a, lds_a + (unsigned)(buf * BK * BM + j * NT * 4) * 4u, oa[j], sa);
#pragma unroll
        for (int j = 0; j < BL; ++j) gemm_copy16_to_lds(rsrc_b, lds_b + (unsigned)(buf * BK * BN + j * NT * 4) * 4u, ob[j], sb);
        sa += (unsigned)(BK * Kp) * 4u;
        sb += (unsigned)(BK * Pp) * 4u;
    };
    // every copy this wavefront has requested has landed (the multiply makes no other vector-memory request)
    auto slab_landed = [&]() { __builtin_amdgcn_s_waitcnt(0x0f70); };   // vmcnt(0)
    const int a_off = wm * (TM * 32) + li, b_off = wn * (TN * 32) + li;
    auto lds_load = [&](int buf, int half, float (&a)[HS][TM], float (&b)[HS][TN]) {
#pragma unroll
        for (int s = 0; s < HS; ++s) {
            const int c = 2 * (half * HS + s) + lg;
#pragma unroll
            for (int i = 0; i < TM; ++i) a[s][i] = As[buf][c * BM + a_off + i * 32];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[s][j] = Bs[buf][c * BN + b_off + j * 32];
        }
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    auto mma = [&](const float (&a)[HS][TM], const float (&b)[HS][TN]) {
#pragma unroll
        for (int s = 0; s < HS; ++s)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s][i], b[s][j], acc[i][j], 0, 0, 0);
    };

    float a0[HS][TM], b0[HS][TN], a1[HS][TM], b1[HS][TN];
    const int nk = min(nk_split, Cp / BK - z * nk_split);   // >= 1 by construction of the launch
    request_slab(0);
    slab_landed();
    __syncthreads();
    lds_load(0, 0, a0, b0);
    // all slabs but the last: fetch the next slab while multiplying the current one.  Two slabs per trip, so that
    // the LDS buffer of every access is known at compile time and its address is a per-lane base plus a constant
    // (with a buffer index computed in the loop, every LDS read cost a vector add in the MFMA issue slot).
    auto slab = [&](int cur) {
        request_slab(cur ^ 1);               // (the other buffer: everybody left it before the last barrier)
        lds_load(cur, 1, a1, b1);
        mma(a0, b0);
        slab_landed();
        __syncthreads();
        lds_load(cur ^ 1, 0, a0, b0);
        mma(a1, b1);
    };
    int kt = 0;
    for (; kt + 2 < nk; kt += 2) {
        slab(0);
        slab(1);
    }
    if (kt + 1 < nk) {   // one more full iteration: the last slab then sits in buffer 1
        slab(0);
        lds_load(1, 1, a1, b1);
    } else {
        lds_load(0, 1, a1, b1);
    }
    mma(a0, b0);
    mma(a1, b1);

    // accumulator register r of lane (li, lg) is row 8*(r/4) + 4*lg + r%4, column li of its tile;
    // Kp and Pp are multiples of 32, so a 32 x 32 tile is entirely inside or entirely outside
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int ct = p0 + wn * (TN * 32) + j * 32, rt = k0 + wm * (TM * 32) + i * 32;
            if (ct < Pp && rt < Kp) {
                float *dst = Me + (size_t)(rt + 4 * lg) * Pp + ct + li;
#pragma unroll
                for (int r = 0; r < 16; ++r) dst[(size_t)(8 * (r / 4) + (r % 4)) * Pp] = acc[i][j][r];
            }
        }
}

template <int BM, int BN, int WM, int WN, int BK>
static hipError_t launch_f32(const Geo &g, const float *U, const float *V, float *M, int splits, hipStream_t s)
{
    const int tiles_m = (g.Kp + BM - 1) / BM, tiles_n = (g.Pp + BN - 1) / BN;
    const int nk = g.Cp / BK;
    const int nk_split = (nk + splits - 1) / splits;
    const int used = (nk + nk_split - 1) / nk_split;   // every share gets at least one slab
    if (used != splits) return hipErrorInvalidValue;
    const long long blocks = (long long)tiles_m * tiles_n * g.a2 * splits;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    // 32-bit byte offsets inside one component of U and of V
    if ((unsigned long long)g.Cp * g.Pp * 4ull >= (1ull << 32) || (unsigned long long)g.Cp * g.Kp * 4ull >= (1ull << 32))
        return hipErrorNotSupported;
    gemm_f32_kernel<BM, BN, WM, WN, BK><<<dim3((unsigned)blocks), dim3(64 * WM * WN), 0, s>>>(
        U, V, M, g.Kp, g.Cp, g.Pp, tiles_m, tiles_n, g.a2, nk_split);
    return hipGetLastError();
}

// fp16 operands, fp32 accumulation, v_mfma_f32_32x32x16_f16.  Operands are stored as
// [e][c/8][row][c%8]: the 8 reduction values a lane feeds to one MFMA are one 16-byte word, a
// BK=32 slab is 4 contiguous runs of 16-byte words per operand, and LDS keeps the same order.
// Lanes 0-31 take the even 8-channel group of a 16-deep MFMA step, lanes 32-63 the odd one,
// for both operands alike, so every product pairs equal channels.
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));

template <int BM, int BN>
__global__ __launch_bounds__(256) void gemm_f16_kernel(const uint4 *__restrict__ U, const uint4 *__restrict__ V,
                                                       float *__restrict__ Mo, int Kp, int Cp, int Pp, int tiles_m,
                                                       int tiles_n)
{
    constexpr int BK = 32, G8 = BK / 8;
    constexpr int TM = BM / 64, TN = BN / 64;
    constexpr int A4 = G8 * BM, B4 = G8 * BN;                  // 16-byte words per slab
    constexpr int AL = (A4 + 255) / 256, BL = (B4 + 255) / 256;
    __shared__ uint4 As[2][A4];
    __shared__ uint4 Bs[2][B4];

    int bid = xcd_remap(blockIdx.x, gridDim.x);   // the filter blocks that share a run of V meet in one L2
    const int tm_i = bid % tiles_m;
    bid /= tiles_m;
    const int tn_i = bid % tiles_n;
    const int e = bid / tiles_n;
    const int k0 = tm_i * BM, p0 = tn_i * BN;
    const int C8 = Cp / 8;

    const uint4 *Ue = U + (size_t)e * C8 * Kp;
    const uint4 *Ve = V + (size_t)e * C8 * Pp;
    float *Me = Mo + (size_t)e * Kp * Pp;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, lg = lane >> 5;

    uint4 ra[AL], rb[BL];
    auto load_global = [&](int g0) {
#pragma unroll
        for (int j = 0; j < AL; ++j) {
            const int idx = tid + j * 256;
            const int grp = idx / BM, col = idx % BM;
            ra[j] = make_uint4(0, 0, 0, 0);
            if (idx < A4 && k0 + col < Kp) ra[j] = Ue[(size_t)(g0 + grp) * Kp + k0 + col];
        }
#pragma unroll
        for (int j = 0; j < BL; ++j) {
            const int idx = tid + j * 256;
            const int grp = idx / BN, col = idx % BN;
            rb[j] = make_uint4(0, 0, 0, 0);
            if (idx < B4 && p0 + col < Pp) rb[j] = Ve[(size_t)(g0 + grp) * Pp + p0 + col];
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int j = 0; j < AL; ++j) {
            const int idx = tid + j * 256;
            if (idx < A4) As[buf][idx] = ra[j];
        }
#pragma unroll
        for (int j = 0; j < BL; ++j) {
            const int idx = tid + j * 256;
            if (idx < B4) Bs[buf][idx] = rb[j];
        }
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int nk = Cp / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) load_global((kt + 1) * G8);
        const uint4 *as = &As[cur][wm * (BM / 2) + li];
        const uint4 *bs = &Bs[cur][wn * (BN / 2) + li];
#pragma unroll
        for (int kk = 0; kk < G8 / 2; ++kk) {
            halfx8 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const uint4 t = as[(2 * kk + lg) * BM + i * 32];
                a[i] = *reinterpret_cast<const halfx8 *>(&t);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const uint4 t = bs[(2 * kk + lg) * BN + j * 32];
                b[j] = *reinterpret_cast<const halfx8 *>(&t);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_lds(cur ^ 1);
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = p0 + wn * (BN / 2) + j * 32 + li;
            const int rbase = k0 + wm * (BM / 2) + i * 32 + 4 * lg;
            if (col < Pp) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = rbase + 8 * (r / 4) + (r % 4);
                    if (row < Kp) Me[(size_t)row * Pp + col] = acc[i][j][r];
                }
            }
        }
}

template <int BM, int BN>
static hipError_t launch_f16(const Geo &g, const void *U, const void *V, float *M, hipStream_t s)
{
    const int tiles_m = (g.Kp + BM - 1) / BM, tiles_n = (g.Pp + BN - 1) / BN;
    const long long blocks = (long long)tiles_m * tiles_n * g.a2;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    gemm_f16_kernel<BM, BN><<<dim3((unsigned)blocks), dim3(256), 0, s>>>((const uint4 *)U, (const uint4 *)V, M, g.Kp,
                                                                         g.Cp, g.Pp, tiles_m, tiles_n);
    return hipGetLastError();
}

// Launch shape of the fp32 multiply: block tile and number of shares of the channel loop.
// Large problems use 128 x 128 blocks and no split.  A problem with few blocks (small batch,
// small images) would leave most of the 256 CUs idle while each block runs a long serial loop,
// so it gets 64-wide blocks and, if that is still short of one block per CU, its reduction over
// C is spread over 2, 4 or 8 groups of blocks, each writing its own partial M (the inverse
// transform adds the partials while gathering).  More than one round of blocks per CU does not
// pay: every block has a fixed prologue and epilogue.
struct GemmShape { int bm, bn, splits; };

static GemmShape gemm_shape(const Geo &g)
{
    GemmShape sh;
    sh.bm = g.Kp >= 128 ? 128 : 64;
    sh.bn = g.Pp >= 128 ? 128 : 64;
    sh.splits = 1;
    if (g.dt != WINO_F32) return sh;
    auto blocks = [&](int bm, int bn) {
        return (long long)((g.Kp + bm - 1) / bm) * ((g.Pp + bn - 1) / bn) * g.a2;
    };
    {
        // Every CU works through blocks / 256 blocks; when that is a small number with a large fractional part, the
        // CUs that get one block more set the time (conv5.x at N = 64: 1600 blocks, 6.25 per CU, 7 rounds).  Halving
        // the block along the tiles doubles the count and brings the loss under 6 % (measured at N = 64: 28 x 28
        // layers 0.621 -> 0.604 ms, 14 x 14 layers 0.272 -> 0.260 ms); U, the operand that is then read twice as
        // often, is the small one.
        auto loss = [&](long long b) { return (double)((b + 255) / 256) / ((double)b / 256.0); };
        if (sh.bm == 128 && sh.bn == 128 && blocks(128, 128) >= 1024 && loss(blocks(128, 128)) > 1.06 &&
            loss(blocks(128, 64)) < loss(blocks(128, 128)) - 0.02)
            sh.bn = 64;
    }
    // Fewer than three 128 x 128 blocks per CU leave the fourth slot of most CUs empty and, with few tiles, pad the
    // last block column heavily (512 -> 512 channels at 28 x 28, batch 8, F(4x4,3x3): 576 blocks for 416 tile
    // columns; 128 x 64 blocks: 1008 blocks, 0.136 -> 0.122 ms for the layer).  From about 900 blocks on the wide
    // block is as fast or faster.
    if (blocks(sh.bm, sh.bn) < 768 && sh.bn == 128) sh.bn = 64;
    if (blocks(sh.bm, sh.bn) < 512 && sh.bm == 128) sh.bm = 64;
    const int nk = g.Cp / 16;
    const long long b = blocks(sh.bm, sh.bn);
    while (sh.splits < 8 && b * sh.splits * 2 <= 256 && nk % (sh.splits * 2) == 0 && nk / (sh.splits * 2) >= 2)
        sh.splits *= 2;
    return sh;
}

int gemm_splits(const Geo &g) { return gemm_shape(g).splits; }

void gemm_launch_shape(const Geo &g, int *bm, int *bn, int *splits)
{
    const GemmShape sh = gemm_shape(g);
    *bm = sh.bm, *bn = sh.bn, *splits = sh.splits;
}

hipError_t launch_batched_gemm(const Geo &g, const void *U, const void *V, float *M, int splits, hipStream_t s)
{
    if (g.dt == WINO_F16) {
        const bool wide_m = g.Kp >= 128, wide_n = g.Pp >= 128;
        if (splits != 1) return hipErrorInvalidValue;
        if (wide_m && wide_n) return launch_f16<128, 128>(g, U, V, M, s);
        if (wide_m) return launch_f16<128, 64>(g, U, V, M, s);
        if (wide_n) return launch_f16<64, 128>(g, U, V, M, s);
        return launch_f16<64, 64>(g, U, V, M, s);
    }
    const float *u = (const float *)U, *v = (const float *)V;
    const GemmShape sh = gemm_shape(g);
    if (sh.bm == 128 && sh.bn == 128) return launch_f32<128, 128, 2, 2, 16>(g, u, v, M, splits, s);
    // The narrower blocks serve small problems, where a workgroup is alone on its CU and its loop over the
    // channels is a chain of memory latencies: slabs of 32 channels halve the links of that chain (measured at
    // batch 1: 3-8 % per layer; 64 gains nothing more).
    if (g.Cp % (32 * splits) == 0) {
        if (sh.bm == 128) return launch_f32<128, 64, 2, 2, 32>(g, u, v, M, splits, s);
        if (sh.bn == 128) return launch_f32<64, 128, 2, 2, 32>(g, u, v, M, splits, s);
        return launch_f32<64, 64, 2, 2, 32>(g, u, v, M, splits, s);
    }
    if (sh.bm == 128) return launch_f32<128, 64, 2, 2, 16>(g, u, v, M, splits, s);
    if (sh.bn == 128) return launch_f32<64, 128, 2, 2, 16>(g, u, v, M, splits, s);
    return launch_f32<64, 64, 2, 2, 16>(g, u, v, M, splits, s);
}

}  // namespace wino

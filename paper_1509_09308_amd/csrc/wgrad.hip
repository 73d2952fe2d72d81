// Gradient with respect to the filters with F(3x3, 2x2) (Lavin & Gray, Section 4.2, Eq. (14)):
// the error tensor is cut into 2 x 2 blocks, each paired with the 4 x 4 input tile around it
// (tiles overlap by 2); in transform space  w = G e G^T,  v = B^T d B,  M = sum over all blocks and
// images of w . v,  dG = A^T M A.  The sum over blocks is 16 matrix products
// M^(e)[K x C] = W^(e)[K x Pb] V^(e)[C x Pb]^T whose reduction index is the block index b.
//
// Stages, each its own kernel: error transform (E -> W[e][k][b]), data transform (D -> V[e][c][b]),
// the 16 products on fp32 MFMAs with the reduction split over workgroups, and the inverse
// transform that also adds the partial products.  fp32, stride 1, pad 1.
#include <stdlib.h>

#include "wino_internal.h"

namespace wino {

typedef float floatx16_w __attribute__((ext_vector_type(16)));
typedef float floatx4_w __attribute__((ext_vector_type(4)));
typedef float floatx2_w __attribute__((ext_vector_type(2)));

// rows of B^T of F(3,2): (1,0,-1,0) (0,1,1,0) (0,-1,1,0) (0,-1,0,1)
__device__ __forceinline__ void bt32_mul(const float *d, float *o)
{
    o[0] = d[0] - d[2];
    o[1] = d[1] + d[2];
    o[2] = d[2] - d[1];
    o[3] = d[3] - d[1];
}
// rows of G of F(3,2): (1,0) (1/2,1/2) (1/2,-1/2) (0,1)
__device__ __forceinline__ void g32_mul(const float *e, float *o)
{
    o[0] = e[0];
    o[1] = 0.5f * (e[0] + e[1]);
    o[2] = 0.5f * (e[0] - e[1]);
    o[3] = e[1];
}
// rows of A^T of F(3,2): (1,1,1,0) (0,1,-1,0) (0,1,1,1)
__device__ __forceinline__ void at32_mul(const float *x, float *o)
{
    o[0] = x[0] + x[1] + x[2];
    o[1] = x[1] - x[2];
    o[2] = x[1] + x[2] + x[3];
}

struct WgradGeo {
    int N, C, H, W, K;
    int Bh, Bw;       // 2 x 2 error blocks per image
    int Pb, Pbp;      // blocks in all, padded to the reduction slab
    int Kp, Cq;       // padded rows of W and V (and extents of M)
};

// One thread per (row, b), b fastest: row is a filter k (IS_ERR) or a channel c.  Rows and blocks
// in the padding are written as zeros.
template <bool IS_ERR>
__global__ __launch_bounds__(256) void wgrad_transform_kernel(const float *__restrict__ X, float *__restrict__ T,
                                                              WgradGeo g)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    const int r = blockIdx.y;
    const int rows = IS_ERR ? g.K : g.C, rows_p = IS_ERR ? g.Kp : g.Cq;
    if (b >= g.Pbp) return;
    float out[4][4];
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int q = 0; q < 4; ++q) out[p][q] = 0.0f;
    if (r < rows && b < g.Pb) {
        const int by = b % g.Bw;
        const int t2 = b / g.Bw;
        const int bx = t2 % g.Bh;
        const int i = t2 / g.Bh;
        const float *src = X + ((size_t)i * rows + r) * g.H * g.W;
        if (IS_ERR) {
            float e[2][2], t[4][2];
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int x = 2 * bx + p, y = 2 * by + q;
                    e[p][q] = (x < g.H && y < g.W) ? src[(size_t)x * g.W + y] : 0.0f;
                }
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                float col[2] = {e[0][q], e[1][q]}, o[4];
                g32_mul(col, o);
#pragma unroll
                for (int p = 0; p < 4; ++p) t[p][q] = o[p];
            }
#pragma unroll
            for (int p = 0; p < 4; ++p) g32_mul(t[p], out[p]);
        } else {
            float d[4][4], t[4][4];
#pragma unroll
            for (int p = 0; p < 4; ++p)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int x = 2 * bx - 1 + p, y = 2 * by - 1 + q;
                    d[p][q] = (x >= 0 && x < g.H && y >= 0 && y < g.W) ? src[(size_t)x * g.W + y] : 0.0f;
                }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float col[4] = {d[0][q], d[1][q], d[2][q], d[3][q]}, o[4];
                bt32_mul(col, o);
#pragma unroll
                for (int p = 0; p < 4; ++p) t[p][q] = o[p];
            }
#pragma unroll
            for (int p = 0; p < 4; ++p) bt32_mul(t[p], out[p]);
        }
    }
#pragma unroll
    for (int xi = 0; xi < 4; ++xi)
#pragma unroll
        for (int nu = 0; nu < 4; ++nu) T[((size_t)(xi * 4 + nu) * rows_p + r) * g.Pbp + b] = out[xi][nu];
    (void)rows_p;
}

// M^(e) = W^(e) V^(e)^T on v_mfma_f32_32x32x2_f32.  Both operands are stored with the reduction
// index b contiguous.  A BK-deep slab is kept in LDS as [row][BK + 2]; lane (i, h) of an MFMA
// reads rows i of its tiles at columns 4t + 2h, 4t + 2h + 1 with one 8-byte read and uses them in
// two consecutive MFMAs (the order of the reduction is free as long as both operands agree).
// The row stride of 18 floats makes those reads conflict-free.  Two LDS slabs: the next slab's
// global loads are in flight during the MFMAs of the current one.  The reduction is split over
// `gridDim` shares z, each writing its own partial M.
template <int BM, int BN>
__global__ __launch_bounds__(256) void wgrad_gemm_kernel(const float *__restrict__ Wt, const float *__restrict__ Vt,
                                                         float *__restrict__ Mo, int Kp, int Cq, int Pbp, int tiles_m,
                                                         int tiles_n, int nk_split)
{
    constexpr int BK = 16, LS = BK + 2;
    constexpr int TM = BM / 64, TN = BN / 64;
    constexpr int A4 = BM * BK / 4, B4 = BN * BK / 4;
    static_assert(A4 % 256 == 0 && B4 % 256 == 0, "slab must divide evenly among the threads");
    constexpr int AL = A4 / 256, BL = B4 / 256;
    __shared__ float As[2][BM * LS];
    __shared__ float Bs[2][BN * LS];

    int bid = blockIdx.x;
    const int tm_i = bid % tiles_m;
    bid /= tiles_m;
    const int tn_i = bid % tiles_n;
    bid /= tiles_n;
    const int e = bid % 16;
    const int z = bid / 16;
    const int k0 = tm_i * BM, c0 = tn_i * BN;
    const int b_first = z * nk_split * BK;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, lh = lane >> 5;

    const float *pa[AL], *pb[BL];
    int sa[AL], sb[BL];
#pragma unroll
    for (int j = 0; j < AL; ++j) {
        const int idx = tid + j * 256;
        const int row = idx / (BK / 4), q = idx % (BK / 4);
        pa[j] = Wt + ((size_t)e * Kp + min(k0 + row, Kp - 1)) * Pbp + b_first + 4 * q;
        sa[j] = row * LS + 4 * q;
    }
#pragma unroll
    for (int j = 0; j < BL; ++j) {
        const int idx = tid + j * 256;
        const int row = idx / (BK / 4), q = idx % (BK / 4);
        pb[j] = Vt + ((size_t)e * Cq + min(c0 + row, Cq - 1)) * Pbp + b_first + 4 * q;
        sb[j] = row * LS + 4 * q;
    }
    floatx4_w ra[AL], rb[BL];
    auto load_global = [&]() {
#pragma unroll
        for (int j = 0; j < AL; ++j) {
            ra[j] = *reinterpret_cast<const floatx4_w *>(pa[j]);
            pa[j] += BK;
        }
#pragma unroll
        for (int j = 0; j < BL; ++j) {
            rb[j] = *reinterpret_cast<const floatx4_w *>(pb[j]);
            pb[j] += BK;
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int j = 0; j < AL; ++j) {
            *reinterpret_cast<floatx2_w *>(&As[buf][sa[j]]) = floatx2_w{ra[j][0], ra[j][1]};
            *reinterpret_cast<floatx2_w *>(&As[buf][sa[j] + 2]) = floatx2_w{ra[j][2], ra[j][3]};
        }
#pragma unroll
        for (int j = 0; j < BL; ++j) {
            *reinterpret_cast<floatx2_w *>(&Bs[buf][sb[j]]) = floatx2_w{rb[j][0], rb[j][1]};
            *reinterpret_cast<floatx2_w *>(&Bs[buf][sb[j] + 2]) = floatx2_w{rb[j][2], rb[j][3]};
        }
    };

    floatx16_w acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int a_off = (wm * (TM * 32) + li) * LS + 2 * lh, b_off = (wn * (TN * 32) + li) * LS + 2 * lh;
    auto compute = [&](int buf) {
#pragma unroll
        for (int t = 0; t < BK / 4; ++t) {
            floatx2_w a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const floatx2_w *>(&As[buf][a_off + i * 32 * LS + 4 * t]);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const floatx2_w *>(&Bs[buf][b_off + j * 32 * LS + 4 * t]);
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][s], b[j][s], acc[i][j], 0, 0, 0);
        }
    };

    const int nk = min(nk_split, Pbp / BK - z * nk_split);   // >= 1 by construction of the launch
    load_global();
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt + 1 < nk; ++kt) {
        const int cur = kt & 1;
        load_global();
        compute(cur);
        store_lds(cur ^ 1);
        __syncthreads();
    }
    compute((nk - 1) & 1);

    float *Me = Mo + ((size_t)z * 16 + e) * Kp * Cq;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int ct = c0 + wn * (TN * 32) + j * 32, rt = k0 + wm * (TM * 32) + i * 32;
            if (ct < Cq && rt < Kp) {
                float *dst = Me + (size_t)(rt + 4 * lh) * Cq + ct + li;
#pragma unroll
                for (int r = 0; r < 16; ++r) dst[(size_t)(8 * (r / 4) + (r % 4)) * Cq] = acc[i][j][r];
            }
        }
}

// The same products with both transforms inside the multiply: W and V never reach memory.  For
// layers with few filters and channels the stand-alone transforms and the multiply above are all
// bound by the 4x expansion of E and D into W and V; here a workgroup of 8 wavefronts owns a
// 64 x 64 block of all 16 M^(e) and walks its share of the error blocks 16 at a time:
//   1. every thread transforms two horizontally adjacent 2 x 2 error blocks (filter r) and the two
//      4 x 4 input tiles around them (channel r) from registers loaded during the previous step
//      -- per row one aligned 16-byte load plus the two outer columns -- and writes the results
//      to LDS as [e][r][b] (b contiguous, row stride 18: conflict-free 8-byte accesses);
//   2. after a barrier the raw data of the next 16 blocks is requested, then each wavefront
//      multiplies: 8 of the 16 components x one 32 x 32 quarter of the block, 64 MFMAs, operands
//      read as in wgrad_gemm_kernel (one 8-byte read feeds two MFMAs), the 8 accumulators
//      interleaved so that consecutive MFMAs are independent.
// Transform and multiply phases alternate rather than overlap; on this chip MFMA and ordinary
// vector instructions do not overlap anyway, and the global loads (about 3 us of latency for this
// access pattern: 64 planes x 128 bytes per step) are in flight during phase 2.  Loads are
// unconditional from clamped (valid) addresses; what falls outside the image, past the last block
// or past K / C is zeroed afterwards, so the loop has no branches and no divisions.
// Needs W % 4 == 0 (block pairs never straddle a row; 16-byte loads) and tensors of fewer than
// 2^31 elements (32-bit offsets).  Partial M per share as above.
constexpr int WF_BK = 16, WF_LS = WF_BK + 2;

__global__ __launch_bounds__(512) void wgrad_fused_kernel(const float *__restrict__ D, const float *__restrict__ E,
                                                          float *__restrict__ Mo, WgradGeo g, int tiles_k, int tiles_c,
                                                          int slabs_per_share)
{
    __shared__ float Ws[16 * 64 * WF_LS];
    __shared__ float Vs[16 * 64 * WF_LS];

    int bid = blockIdx.x;
    const int kt = bid % tiles_k;
    bid /= tiles_k;
    const int ct = bid % tiles_c;
    const int z = bid / tiles_c;
    const int tid = threadIdx.x;
    const int r = tid >> 3, pl = tid & 7;        // row of the block (filter / channel), pair of blocks
    const int k = kt * 64 + r, c = ct * 64 + r;
    const int slab_lo = z * slabs_per_share;
    const int slab_hi = min(slab_lo + slabs_per_share, (g.Pb + WF_BK - 1) / WF_BK);

    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int st = wave & 3, ch = wave >> 2;
    const int wm = st >> 1, wn = st & 1;
    const int li = lane & 31, lh = lane >> 5;

    floatx16_w acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[e][q] = 0.0f;

    // position of this thread's pair of blocks (b, b + 1; b even, so is by)
    const int kc = min(k, g.K - 1), cc = min(c, g.C - 1);
    int b_cur = slab_lo * WF_BK + 2 * pl;
    int by, bx, im;
    {
        const int b = min(b_cur, g.Pb - 2);
        by = b % g.Bw;
        const int t2 = b / g.Bw;
        bx = t2 % g.Bh;
        im = t2 / g.Bh;
    }
    floatx4_w er[2], dm[4];    // error rows 2bx, 2bx+1 and input rows 2bx-1 .. 2bx+2, columns 2by .. 2by+3
    float dl[4], dr[4];        // input columns 2by-1 and 2by+4
    bool okb, ok1, okl, okr, okx[4];
    auto load_raw = [&]() {
        okb = b_cur < g.Pb;
        ok1 = 2 * bx + 1 < g.H;
        okl = by > 0;
        okr = by + 2 < g.Bw;
        const unsigned eo = (((unsigned)im * g.K + kc) * g.H + 2 * bx) * g.W + 2 * by;
        er[0] = *reinterpret_cast<const floatx4_w *>(E + eo);
        er[1] = *reinterpret_cast<const floatx4_w *>(E + eo + (ok1 ? g.W : 0));
        const unsigned dbase = ((unsigned)im * g.C + cc) * g.H * g.W + 2 * by;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int x = 2 * bx - 1 + p;
            okx[p] = x >= 0 && x < g.H;
            const float *row = D + dbase + (unsigned)min(max(x, 0), g.H - 1) * g.W;
            dm[p] = *reinterpret_cast<const floatx4_w *>(row);
            dl[p] = *(row - (okl ? 1 : 0));
            dr[p] = *(row + (okr ? 4 : 3));
        }
    };
    auto advance = [&]() {
        b_cur += WF_BK;
        if (b_cur < g.Pb) {          // past the end the position stays on the last valid pair
            by += WF_BK;
            while (by >= g.Bw) {
                by -= g.Bw;
                if (++bx == g.Bh) {
                    bx = 0;
                    ++im;
                }
            }
        }
    };
    auto transform_to_lds = [&]() {
        const bool ke = okb && k < g.K, kd = okb && c < g.C;
        float t[4][4], o[4], wa[16], wb[16];
        // w = G e G^T of the two error blocks
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            float *dst = blk ? wb : wa;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const float col[2] = {ke ? er[0][2 * blk + q] : 0.0f, (ke && ok1) ? er[1][2 * blk + q] : 0.0f};
                g32_mul(col, o);
#pragma unroll
                for (int p = 0; p < 4; ++p) t[p][q] = o[p];
            }
#pragma unroll
            for (int p = 0; p < 4; ++p) g32_mul(t[p], dst + 4 * p);
        }
#pragma unroll
        for (int e = 0; e < 16; ++e)
            *reinterpret_cast<floatx2_w *>(&Ws[(e * 64 + r) * WF_LS + 2 * pl]) = floatx2_w{wa[e], wb[e]};
        // v = B^T d B of the two input tiles: columns 2by-1 .. 2by+2 and 2by+1 .. 2by+4
        float d[4][6];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const bool v = kd && okx[p];
            d[p][0] = (v && okl) ? dl[p] : 0.0f;
            d[p][1] = v ? dm[p][0] : 0.0f;
            d[p][2] = v ? dm[p][1] : 0.0f;
            d[p][3] = v ? dm[p][2] : 0.0f;
            d[p][4] = v ? dm[p][3] : 0.0f;
            d[p][5] = (v && okr) ? dr[p] : 0.0f;
        }
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            float *dst = blk ? wb : wa;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float col[4] = {d[0][2 * blk + q], d[1][2 * blk + q], d[2][2 * blk + q], d[3][2 * blk + q]};
                bt32_mul(col, o);
#pragma unroll
                for (int p = 0; p < 4; ++p) t[p][q] = o[p];
            }
#pragma unroll
            for (int p = 0; p < 4; ++p) bt32_mul(t[p], dst + 4 * p);
        }
#pragma unroll
        for (int e = 0; e < 16; ++e)
            *reinterpret_cast<floatx2_w *>(&Vs[(e * 64 + r) * WF_LS + 2 * pl]) = floatx2_w{wa[e], wb[e]};
    };
    const int a_off = (wm * 32 + li) * WF_LS + 2 * lh, b_off = (wn * 32 + li) * WF_LS + 2 * lh;
    auto multiply = [&]() {
#pragma unroll
        for (int t = 0; t < WF_BK / 4; ++t) {
            floatx2_w a[8], b[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int eo = (ch * 8 + e) * 64 * WF_LS;
                a[e] = *reinterpret_cast<const floatx2_w *>(&Ws[eo + a_off + 4 * t]);
                b[e] = *reinterpret_cast<const floatx2_w *>(&Vs[eo + b_off + 4 * t]);
            }
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    acc[e] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e][h], b[e][h], acc[e], 0, 0, 0);
        }
    };

    load_raw();
    for (int slab = slab_lo; slab < slab_hi; ++slab) {
        transform_to_lds();
        __syncthreads();
        advance();
        load_raw();          // after the last slab this re-reads a valid position and is discarded
        multiply();
        __syncthreads();
    }

    // a share past the end of the blocks still writes its (zero) partial M
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int rt = kt * 64 + wm * 32, ctile = ct * 64 + wn * 32;
        if (rt < g.Kp && ctile < g.Cq) {
            float *dst = Mo + (((size_t)z * 16 + ch * 8 + e) * g.Kp + rt + 4 * lh) * g.Cq + ctile + li;
#pragma unroll
            for (int q = 0; q < 16; ++q) dst[(size_t)(8 * (q / 4) + (q % 4)) * g.Cq] = acc[e][q];
        }
    }
}

// First level of the sum over shares when there are many of them: out[zg][i] = sum of in[z][i] over
// the WR_GROUP shares z of group zg, in share order.  One thread per element and group, so the
// partial results (up to 134 MB for a 64 x 64 layer with 512 shares) are read by thousands of
// wavefronts instead of the few that own an output.
constexpr int WR_GROUP = 16, WR_MIN_SHARES = 33;

__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float *__restrict__ in, float *__restrict__ out,
                                                           int nelem4, int shares)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    const int zg = blockIdx.y;
    if (i >= nelem4) return;
    const int z0 = zg * WR_GROUP, z1 = min(z0 + WR_GROUP, shares);
    const floatx4_w *src = reinterpret_cast<const floatx4_w *>(in);
    floatx4_w a = src[(size_t)z0 * nelem4 + i];
    for (int z = z0 + 1; z < z1; ++z) a += src[(size_t)z * nelem4 + i];
    reinterpret_cast<floatx4_w *>(out)[(size_t)zg * nelem4 + i] = a;
}

// Reduces `shares` partial arrays of nelem floats at `part` to fewer (when there are more than 32 and
// nelem % 4 == 0; otherwise nothing is done), using `tmp`
// (room for ceil(shares / WR_GROUP) arrays).  Returns where the remaining partials are and how many.
static const float *wgrad_pre_reduce(const float *part, float *tmp, size_t nelem, int *shares, hipStream_t s)
{
    if (*shares < WR_MIN_SHARES || nelem % 4 != 0) return part;
    const int groups = (*shares + WR_GROUP - 1) / WR_GROUP;
    const int n4 = (int)(nelem / 4);
    wgrad_reduce_kernel<<<dim3((n4 + 255) / 256, groups), dim3(256), 0, s>>>(part, tmp, n4, *shares);
    *shares = groups;
    return tmp;
}

static size_t wgrad_pre_reduce_bytes(size_t nelem, int shares)
{
    if (shares < WR_MIN_SHARES || nelem % 4 != 0) return 0;
    return (((size_t)((shares + WR_GROUP - 1) / WR_GROUP) * nelem * 4) + 255) & ~(size_t)255;
}

// dG[k][c] = A^T (sum over shares of M[e][k][c]) A; one thread per (k, c), c fastest.
__global__ __launch_bounds__(256) void wgrad_output_kernel(const float *__restrict__ Mi, float *__restrict__ dG,
                                                           WgradGeo g, int shares)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    const int k = blockIdx.y;
    if (c >= g.C) return;
    float m[4][4];
#pragma unroll
    for (int xi = 0; xi < 4; ++xi)
#pragma unroll
        for (int nu = 0; nu < 4; ++nu) m[xi][nu] = 0.0f;
    const size_t plane = (size_t)g.Kp * g.Cq;
    for (int z = 0; z < shares; ++z)
#pragma unroll
        for (int xi = 0; xi < 4; ++xi)
#pragma unroll
            for (int nu = 0; nu < 4; ++nu) m[xi][nu] += Mi[((size_t)z * 16 + xi * 4 + nu) * plane + (size_t)k * g.Cq + c];
    float t[3][4], y[3][3];
#pragma unroll
    for (int nu = 0; nu < 4; ++nu) {
        float col[4] = {m[0][nu], m[1][nu], m[2][nu], m[3][nu]}, o[3];
        at32_mul(col, o);
#pragma unroll
        for (int p = 0; p < 3; ++p) t[p][nu] = o[p];
    }
#pragma unroll
    for (int p = 0; p < 3; ++p) at32_mul(t[p], y[p]);
    float *dst = dG + ((size_t)k * g.C + c) * 9;
#pragma unroll
    for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int q = 0; q < 3; ++q) dst[p * 3 + q] = y[p][q];
}

// Layers with very few channels (the 3-channel first layer): the transforms above would spend
// almost all their time on the error tensor (16 values written and read back per 4 read) for a
// handful of products, so the gradient is evaluated directly from its definition instead.  One
// wavefront takes KB = 4 filters of one image and one of RS row bands; lanes run along 4-pixel
// segments of the error rows (16-byte loads); the 3 x 6 input window of a segment is loaded once
// per channel and used for all 4 filters; 4 * 9 * CH running sums per lane are reduced across the
// wavefront at the end.  The per-(image, band) partial sums are added by
// wgrad_direct_reduce_kernel in a fixed order.  Needs W % 4 == 0.
constexpr int WD_KB = 4, WD_RS = 4;

template <int CH>
__global__ __launch_bounds__(256) void wgrad_direct_kernel(const float *__restrict__ D, const float *__restrict__ E,
                                                           float *__restrict__ part, int N, int H, int W, int K)
{
    const int KG = (K + WD_KB - 1) / WD_KB;
    int task = blockIdx.x * 4 + (threadIdx.x >> 6);   // ((i * RS + band) * KG + kg)
    const int lane = threadIdx.x & 63;
    if (task >= N * WD_RS * KG) return;
    const int kg = task % KG;
    task /= KG;
    const int band = task % WD_RS, i = task / WD_RS;
    const int rows = (H + WD_RS - 1) / WD_RS;
    const int x_lo = band * rows, x_hi = min(H, x_lo + rows);
    const float *Di = D + (size_t)i * CH * H * W;
    const int W4 = W >> 2, nq = max(0, x_hi - x_lo) * W4;
    float acc[WD_KB][CH][3][3];
#pragma unroll
    for (int f = 0; f < WD_KB; ++f)
#pragma unroll
        for (int c = 0; c < CH; ++c)
#pragma unroll
            for (int u = 0; u < 3; ++u)
#pragma unroll
                for (int v = 0; v < 3; ++v) acc[f][c][u][v] = 0.0f;
    for (int q = lane; q < nq; q += 64) {
        const int xr = q / W4, x = x_lo + xr, y = (q - xr * W4) * 4;
        floatx4_w e[WD_KB];
#pragma unroll
        for (int f = 0; f < WD_KB; ++f) {
            const int k = min(kg * WD_KB + f, K - 1);   // filters past K are computed and dropped
            e[f] = *reinterpret_cast<const floatx4_w *>(E + (((size_t)i * K + k) * H + x) * W + y);
        }
#pragma unroll
        for (int c = 0; c < CH; ++c)
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                const int xx = x + u - 1;
                if (xx < 0 || xx >= H) continue;
                const float *row = Di + ((size_t)c * H + xx) * W + y;
                const floatx4_w mid = *reinterpret_cast<const floatx4_w *>(row);
                const float d[6] = {y > 0 ? row[-1] : 0.0f, mid[0], mid[1], mid[2], mid[3], y + 4 < W ? row[4] : 0.0f};
#pragma unroll
                for (int f = 0; f < WD_KB; ++f)
#pragma unroll
                    for (int v = 0; v < 3; ++v)
                        acc[f][c][u][v] += e[f][0] * d[v] + e[f][1] * d[v + 1] + e[f][2] * d[v + 2] + e[f][3] * d[v + 3];
            }
    }
    float *dst = part + (size_t)(i * WD_RS + band) * K * CH * 9;
#pragma unroll
    for (int f = 0; f < WD_KB; ++f)
#pragma unroll
        for (int c = 0; c < CH; ++c)
#pragma unroll
            for (int u = 0; u < 3; ++u)
#pragma unroll
                for (int v = 0; v < 3; ++v) {
                    float a = acc[f][c][u][v];
#pragma unroll
                    for (int off = 32; off >= 1; off >>= 1) a += __shfl_xor(a, off, 64);
                    const int k = kg * WD_KB + f;
                    if (lane == 0 && k < K) dst[((size_t)k * CH + c) * 9 + u * 3 + v] = a;
                }
}

// dG[k][c][uv] = sum over images and row bands of part[.][k][c][uv]; one thread per output.
__global__ __launch_bounds__(256) void wgrad_direct_reduce_kernel(const float *__restrict__ part, float *__restrict__ dG,
                                                                  int nparts, int KC9)
{
    const int o = blockIdx.x * 256 + threadIdx.x;
    if (o >= KC9) return;
    float a = 0.0f;
    for (int i = 0; i < nparts; ++i) a += part[(size_t)i * KC9 + o];
    dG[o] = a;
}

static bool wgrad_direct_ok(int C, int W) { return C <= 4 && W % 4 == 0; }

static WgradGeo make_wgeo(int N, int C, int H, int W, int K)
{
    WgradGeo g;
    g.N = N; g.C = C; g.H = H; g.W = W; g.K = K;
    g.Bh = (H + 1) / 2; g.Bw = (W + 1) / 2;
    g.Pb = N * g.Bh * g.Bw;
    g.Pbp = round_up(g.Pb, 16);
    g.Kp = round_up(K, 32);
    g.Cq = round_up(C, 32);
    return g;
}

static void wgrad_shape(const WgradGeo &g, int *bm, int *bn, int *shares, int *nk_split)
{
    *bm = g.Kp >= 128 ? 128 : 64;
    *bn = g.Cq >= 128 ? 128 : 64;
    const long long blocks = (long long)((g.Kp + *bm - 1) / *bm) * ((g.Cq + *bn - 1) / *bn) * 16;
    const int nk = g.Pbp / 16;
    int want = (int)((768 + blocks - 1) / blocks);   // about three blocks per CU in all
    if (want > 256) want = 256;
    if (want > nk / 8) want = nk / 8 > 0 ? nk / 8 : 1;   // at least 8 slabs per share
    if (want < 1) want = 1;
    *nk_split = (nk + want - 1) / want;
    *shares = (nk + *nk_split - 1) / *nk_split;
}

// The fused kernel is chosen where the stand-alone transforms dominate: few filters and channels
// (every 64 x 64 block of M repeats both transforms, so their cost grows with K * C).
static bool wgrad_fused_ok(const WgradGeo &g)
{
    if (g.W % 4 != 0) return false;
    if ((long long)g.N * (g.K > g.C ? g.K : g.C) * g.H * g.W >= (1LL << 31)) return false;   // 32-bit offsets
    return g.K <= 256 && g.C <= 256;   // measured at N=64: faster up to 256 x 256, slower at 512 x 512
}

static void wgrad_fused_shape(const WgradGeo &g, int *tiles_k, int *tiles_c, int *shares, int *slabs_per_share)
{
    *tiles_k = (g.Kp + 63) / 64;
    *tiles_c = (g.Cq + 63) / 64;
    const int slabs = (g.Pb + WF_BK - 1) / WF_BK;
    int want = 512 / (*tiles_k * *tiles_c);   // one workgroup fits a CU at a time: two rounds of 256
    if (want > slabs / 4) want = slabs / 4;   // at least 4 slabs per share
    if (want < 1) want = 1;
    *slabs_per_share = (slabs + want - 1) / want;
    *shares = (slabs + *slabs_per_share - 1) / *slabs_per_share;
}

bool wgrad_supported(long long N, long long C, long long H, long long W, long long K)
{
    const long long Pb = N * ((H + 1) / 2) * ((W + 1) / 2);
    return Pb < (1LL << 30) && C <= 65000 && K <= 65000;
}

size_t wgrad_workspace_bytes(int N, int C, int H, int W, int K)
{
    if (wgrad_direct_ok(C, W))
        return (((size_t)N * WD_RS * K * C * 9 * 4 + 255) & ~(size_t)255) + wgrad_pre_reduce_bytes((size_t)K * C * 9, N * WD_RS);
    const WgradGeo g = make_wgeo(N, C, H, W, K);
    int bm, bn, shares, nk_split;
    auto al = [](size_t x) { return (x + 255) & ~(size_t)255; };
    if (wgrad_fused_ok(g)) {
        int tk, tc, sps;
        wgrad_fused_shape(g, &tk, &tc, &shares, &sps);
        return al((size_t)shares * 16 * g.Kp * g.Cq * 4) + wgrad_pre_reduce_bytes((size_t)16 * g.Kp * g.Cq, shares);
    }
    wgrad_shape(g, &bm, &bn, &shares, &nk_split);
    return al((size_t)16 * g.Kp * g.Pbp * 4) + al((size_t)16 * g.Cq * g.Pbp * 4) + al((size_t)shares * 16 * g.Kp * g.Cq * 4) +
           wgrad_pre_reduce_bytes((size_t)16 * g.Kp * g.Cq, shares);
}

hipError_t launch_wgrad(int N, int C, int H, int W, int K, const float *D, const float *E, float *dG, void *workspace,
                        hipStream_t s)
{
    if (wgrad_direct_ok(C, W)) {
        float *part = (float *)workspace;
        const dim3 grid((N * WD_RS * ((K + WD_KB - 1) / WD_KB) + 3) / 4), blk(256);
        if (C == 1) wgrad_direct_kernel<1><<<grid, blk, 0, s>>>(D, E, part, N, H, W, K);
        else if (C == 2) wgrad_direct_kernel<2><<<grid, blk, 0, s>>>(D, E, part, N, H, W, K);
        else if (C == 3) wgrad_direct_kernel<3><<<grid, blk, 0, s>>>(D, E, part, N, H, W, K);
        else wgrad_direct_kernel<4><<<grid, blk, 0, s>>>(D, E, part, N, H, W, K);
        int nparts = N * WD_RS;
        float *tmp = (float *)((char *)workspace + (((size_t)nparts * K * C * 9 * 4 + 255) & ~(size_t)255));
        const float *ps = wgrad_pre_reduce(part, tmp, (size_t)K * C * 9, &nparts, s);
        wgrad_direct_reduce_kernel<<<dim3((K * C * 9 + 255) / 256), blk, 0, s>>>(ps, dG, nparts, K * C * 9);
        return hipGetLastError();
    }
    const WgradGeo g = make_wgeo(N, C, H, W, K);
    int bm, bn, shares, nk_split;
    if (wgrad_fused_ok(g)) {
        int tk, tc, sps;
        wgrad_fused_shape(g, &tk, &tc, &shares, &sps);
        float *Mw = (float *)workspace;
        float *tmp = (float *)((char *)workspace + (((size_t)shares * 16 * g.Kp * g.Cq * 4 + 255) & ~(size_t)255));
        wgrad_fused_kernel<<<dim3((unsigned)(tk * tc * shares)), dim3(512), 0, s>>>(D, E, Mw, g, tk, tc, sps);
        const float *Ms = wgrad_pre_reduce(Mw, tmp, (size_t)16 * g.Kp * g.Cq, &shares, s);
        wgrad_output_kernel<<<dim3((C + 255) / 256, K), dim3(256), 0, s>>>(Ms, dG, g, shares);
        return hipGetLastError();
    }
    wgrad_shape(g, &bm, &bn, &shares, &nk_split);
    auto al = [](size_t x) { return (x + 255) & ~(size_t)255; };
    char *ws = (char *)workspace;
    float *Wt = (float *)ws;
    float *Vt = (float *)(ws + al((size_t)16 * g.Kp * g.Pbp * 4));
    float *Mw = (float *)(ws + al((size_t)16 * g.Kp * g.Pbp * 4) + al((size_t)16 * g.Cq * g.Pbp * 4));
    dim3 block(256);
    wgrad_transform_kernel<true><<<dim3((g.Pbp + 255) / 256, g.Kp), block, 0, s>>>(E, Wt, g);
    wgrad_transform_kernel<false><<<dim3((g.Pbp + 255) / 256, g.Cq), block, 0, s>>>(D, Vt, g);
    const int tiles_m = (g.Kp + bm - 1) / bm, tiles_n = (g.Cq + bn - 1) / bn;
    const long long blocks = (long long)tiles_m * tiles_n * 16 * shares;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks);
    if (bm == 128 && bn == 128)
        wgrad_gemm_kernel<128, 128><<<grid, block, 0, s>>>(Wt, Vt, Mw, g.Kp, g.Cq, g.Pbp, tiles_m, tiles_n, nk_split);
    else if (bm == 128)
        wgrad_gemm_kernel<128, 64><<<grid, block, 0, s>>>(Wt, Vt, Mw, g.Kp, g.Cq, g.Pbp, tiles_m, tiles_n, nk_split);
    else if (bn == 128)
        wgrad_gemm_kernel<64, 128><<<grid, block, 0, s>>>(Wt, Vt, Mw, g.Kp, g.Cq, g.Pbp, tiles_m, tiles_n, nk_split);
    else
        wgrad_gemm_kernel<64, 64><<<grid, block, 0, s>>>(Wt, Vt, Mw, g.Kp, g.Cq, g.Pbp, tiles_m, tiles_n, nk_split);
    float *tmp = (float *)((char *)Mw + al((size_t)shares * 16 * g.Kp * g.Cq * 4));
    const float *Ms = wgrad_pre_reduce(Mw, tmp, (size_t)16 * g.Kp * g.Cq, &shares, s);
    wgrad_output_kernel<<<dim3((C + 255) / 256, K), block, 0, s>>>(Ms, dG, g, shares);
    return hipGetLastError();
}

}  // namespace wino

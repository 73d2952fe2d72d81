// Bodies of the filter transform (loop 1 of Algorithm 1) and of the input transform (loop 2)
// as device functions of a block index, so that they can run as kernels of their own or side by
// side in one launch (the two loops are independent of each other).
#pragma once
#include "wino_internal.h"
#include "transforms.h"

namespace wino {

template <typename T> __device__ __forceinline__ float ld_f(const T *p);
template <> __device__ __forceinline__ float ld_f<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float ld_f<__half>(const __half *p) { return __half2float(*p); }

template <typename T> __device__ __forceinline__ float ld_in(const T *p);
template <> __device__ __forceinline__ float ld_in<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float ld_in<__half>(const __half *p) { return __half2float(*p); }

// One thread per (k, c) of the padded Kp x Cp grid, k fastest: a wavefront is 64 consecutive
// filters of one channel, so each of its alpha^2 stores is 256 contiguous bytes.  A workgroup
// covers KT filters x CT channels; the 9*CT source values of one filter are contiguous in G and
// are staged through LDS with coalesced loads.
constexpr int FT_KT = 64, FT_CT = 4, FT_ROW = FT_CT * 9 + 1, FT_LDS = FT_KT * FT_ROW;   // floats of LDS per block

template <int M, typename T>
__device__ __forceinline__ void filter_transform_block(const T *__restrict__ G, T *__restrict__ U, int K, int C,
                                                       int Kp, int Cp, int bx, int by, float *gs)
{
    constexpr int A = M + 2, KT = FT_KT, CT = FT_CT, ROW = FT_ROW;
    const int k0 = bx * KT, c0 = by * CT;
    for (int idx = threadIdx.x; idx < KT * CT * 9; idx += 256) {
        const int kl = idx / (CT * 9), j = idx % (CT * 9);
        const int k = k0 + kl, c = c0 + j / 9;
        float v = 0.0f;
        if (k < K && c < C) v = ld_f<T>(G + ((size_t)k * C + c0) * 9 + j);
        gs[kl * ROW + j] = v;
    }
    __syncthreads();
    const int kl = threadIdx.x % KT, cl = threadIdx.x / KT;
    const int k = k0 + kl, c = c0 + cl;
    if (k >= Kp || c >= Cp) return;
    float g[3][3], t[A][3], u[A][A];
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int j = 0; j < 3; ++j) g[i][j] = gs[kl * ROW + cl * 9 + i * 3 + j];
    // t = G g : transform the columns of g
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        float col[3] = {g[0][j], g[1][j], g[2][j]}, o[A];
        g_mul<M>(col, o);
#pragma unroll
        for (int i = 0; i < A; ++i) t[i][j] = o[i];
    }
    // u = t G^T : transform the rows of t
#pragma unroll
    for (int i = 0; i < A; ++i) g_mul<M>(t[i], u[i]);
#pragma unroll
    for (int xi = 0; xi < A; ++xi)
#pragma unroll
        for (int nu = 0; nu < A; ++nu) {
            const int e = xi * A + nu;
            if constexpr (sizeof(T) == 4) {
                U[((size_t)e * Cp + c) * Kp + k] = u[xi][nu];
            } else {
                // fp16 layout [e][c/8][k][c%8]
                U[(((size_t)e * (Cp / 8) + c / 8) * Kp + k) * 8 + (c % 8)] = __float2half_rn(u[xi][nu]);
            }
        }
}

// One thread per (c, b); b is the fastest index of a workgroup so the stores to every
// V^(xi,nu) row are contiguous across a wavefront.  Channels c >= C and tiles b >= P are
// padding and are written as zeros.
typedef float floatx4_v __attribute__((ext_vector_type(4)));

template <int M, typename T, bool VEC>
__device__ __forceinline__ void input_transform_block(const T *__restrict__ D, T *__restrict__ V, const Geo &g, int bx,
                                                      int by)
{
    constexpr int A = M + 2;
    const int b = bx * 256 + threadIdx.x;
    const int c = by;
    if (b >= g.Pp) return;
    float d[A][A];
#pragma unroll
    for (int p = 0; p < A; ++p)
#pragma unroll
        for (int q = 0; q < A; ++q) d[p][q] = 0.0f;
    if (c < g.C && b < g.P) {
        const int ty = b % g.Tw;
        const int t2 = b / g.Tw;
        const int tx = t2 % g.Th;
        const int i = t2 / g.Th;
        const int x0 = M * tx - g.pad, y0 = M * ty - g.pad;
        const T *src = D + ((size_t)i * g.C + c) * g.H * g.W;
#pragma unroll
        for (int p = 0; p < A; ++p) {
            const int x = x0 + p;
            if (x >= 0 && x < g.H) {
                if constexpr (VEC) {
                    // pad 1 and W a multiple of 4: columns 1..4 are one aligned 16-byte load
                    const float *row = reinterpret_cast<const float *>(src) + (size_t)x * g.W + y0;
                    const floatx4_v mid = *reinterpret_cast<const floatx4_v *>(row + 1);
                    d[p][1] = mid[0]; d[p][2] = mid[1]; d[p][3] = mid[2]; d[p][4] = mid[3];
                    if (y0 >= 0) d[p][0] = row[0];
                    if (y0 + 5 < g.W) d[p][5] = row[5];
                } else {
#pragma unroll
                    for (int q = 0; q < A; ++q) {
                        const int y = y0 + q;
                        if (y >= 0 && y < g.W) d[p][q] = ld_in<T>(src + (size_t)x * g.W + y);
                    }
                }
            }
        }
    }
    // t = B^T d (columns), v = t B (rows)
    float t[A][A], v[A][A];
#pragma unroll
    for (int q = 0; q < A; ++q) {
        float col[A], o[A];
#pragma unroll
        for (int p = 0; p < A; ++p) col[p] = d[p][q];
        bt_mul<M>(col, o);
#pragma unroll
        for (int p = 0; p < A; ++p) t[p][q] = o[p];
    }
#pragma unroll
    for (int p = 0; p < A; ++p) bt_mul<M>(t[p], v[p]);
#pragma unroll
    for (int xi = 0; xi < A; ++xi)
#pragma unroll
        for (int nu = 0; nu < A; ++nu) {
            const int e = xi * A + nu;
            if constexpr (sizeof(T) == 4) {
                V[((size_t)e * g.Cp + c) * g.Pp + b] = v[xi][nu];
            } else {
                V[(((size_t)e * (g.Cp / 8) + c / 8) * g.Pp + b) * 8 + (c % 8)] = __float2half_rn(v[xi][nu]);
            }
        }
}

// fp32, pad 1, W a multiple of 8 (an even number of tiles per row): two horizontally adjacent
// tiles per thread.  Their 10 input columns are fetched per row as two aligned 16-byte loads
// (32 contiguous bytes per lane, so a wavefront requests whole cache lines) plus the two outer
// columns, which are absent on the image border; the two results go out as one 8-byte store per
// component, 512 contiguous bytes per wavefront and store instruction.
typedef float floatx4_it __attribute__((ext_vector_type(4)));
typedef float floatx2_it __attribute__((ext_vector_type(2)));

template <int M>
__device__ __forceinline__ void input_transform_pair_block(const float *__restrict__ D, float *__restrict__ V,
                                                           const Geo &g, int bx, int by)
{
    constexpr int A = M + 2;
    static_assert(M == 4, "two 6-wide tiles share 10 columns: 1 + 4 + 4 + 1");
    const int b0 = (bx * 256 + threadIdx.x) * 2;   // even; Tw is even, so b0 and b0+1 share a tile row
    const int c = by;
    if (b0 >= g.Pp) return;
    float d[A][10];
#pragma unroll
    for (int p = 0; p < A; ++p)
#pragma unroll
        for (int q = 0; q < 10; ++q) d[p][q] = 0.0f;
    if (c < g.C && b0 < g.P) {   // P is even as well, so both tiles exist
        const int ty = b0 % g.Tw;
        const int t2 = b0 / g.Tw;
        const int tx = t2 % g.Th;
        const int i = t2 / g.Th;
        const int x0 = M * tx - 1, y0 = M * ty - 1;
        const float *src = D + ((size_t)i * g.C + c) * g.H * g.W;
#pragma unroll
        for (int p = 0; p < A; ++p) {
            const int x = x0 + p;
            if (x >= 0 && x < g.H) {
                const float *row = src + (size_t)x * g.W + y0;
                const floatx4_it m0 = *reinterpret_cast<const floatx4_it *>(row + 1);
                const floatx4_it m1 = *reinterpret_cast<const floatx4_it *>(row + 5);
                d[p][1] = m0[0]; d[p][2] = m0[1]; d[p][3] = m0[2]; d[p][4] = m0[3];
                d[p][5] = m1[0]; d[p][6] = m1[1]; d[p][7] = m1[2]; d[p][8] = m1[3];
                if (y0 >= 0) d[p][0] = row[0];
                if (y0 + 9 < g.W) d[p][9] = row[9];
            }
        }
    }
    float v[2][A][A];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        float tt[A][A];
#pragma unroll
        for (int q = 0; q < A; ++q) {
            float col[A], o[A];
#pragma unroll
            for (int p = 0; p < A; ++p) col[p] = d[p][4 * t + q];
            bt_mul<M>(col, o);
#pragma unroll
            for (int p = 0; p < A; ++p) tt[p][q] = o[p];
        }
#pragma unroll
        for (int p = 0; p < A; ++p) bt_mul<M>(tt[p], v[t][p]);
    }
#pragma unroll
    for (int xi = 0; xi < A; ++xi)
#pragma unroll
        for (int nu = 0; nu < A; ++nu) {
            const int e = xi * A + nu;
            *reinterpret_cast<floatx2_it *>(V + ((size_t)e * g.Cp + c) * g.Pp + b0) =
                floatx2_it{v[0][xi][nu], v[1][xi][nu]};
        }
}

// ---- fp16 storage ------------------------------------------------------------------------------
// Both bodies transform in fp32, round once to fp16, collect the results of a block in LDS and write 16-byte units
// (one of them is the 8 channels a lane feeds to the fp16 MFMA); `smem` must hold f16_stage_bytes(M) bytes.
constexpr int F16_KT = 64, F16_CT = 8, F16_ROW = F16_CT * 9 + 1, F16_TB = 64;
constexpr int f16_stage_bytes(int M)
{
    const int collect = (M + 2) * (M + 2) * 64 * 8 * 2, taps = F16_KT * F16_ROW * 4;
    return collect > taps ? collect : taps;
}

// Filter transform.  U is laid out [e][c/8][k][c%8], so a (k, c) thread owns isolated 2-byte elements of U.  A block
// therefore takes 64 filters x 8 channels (their 72 source values per filter are contiguous in G) and writes U as
// 1 KB contiguous per component and wavefront instead of 64 scattered 2-byte stores.  NT threads (256 or 512).
template <int M, int NT>
__device__ __forceinline__ void filter_transform_f16_block(const __half *__restrict__ G, __half *__restrict__ U, int K,
                                                           int C, int Kp, int Cp, int bx, int by, void *smem)
{
    constexpr int A = M + 2, A2 = A * A, KT = F16_KT, CT = F16_CT, ROW = F16_ROW, PAIRS = KT * CT / NT;
    float *gs = reinterpret_cast<float *>(smem);       // the taps of the block ...
    __half *us = reinterpret_cast<__half *>(smem);     // ... and, once every thread holds its taps, the results
    const int tid = threadIdx.x;
    const int k0 = bx * KT, c0 = by * CT;
    for (int idx = tid; idx < KT * CT * 9; idx += NT) {
        const int kl = idx / (CT * 9), j = idx % (CT * 9);
        const int k = k0 + kl, c = c0 + j / 9;
        gs[kl * ROW + j] = (k < K && c < C) ? __half2float(G[((size_t)k * C + c0) * 9 + j]) : 0.0f;
    }
    __syncthreads();
    const int kl = tid % KT;
    float g[PAIRS][3][3];
#pragma unroll
    for (int h = 0; h < PAIRS; ++h) {
        const int cl = tid / KT + (NT / KT) * h;
#pragma unroll
        for (int i = 0; i < 3; ++i)
#pragma unroll
            for (int j = 0; j < 3; ++j) g[h][i][j] = gs[kl * ROW + cl * 9 + i * 3 + j];
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < PAIRS; ++h) {
        const int cl = tid / KT + (NT / KT) * h;
        float t[A][3], u[A][A];
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            float col[3] = {g[h][0][j], g[h][1][j], g[h][2][j]}, o[A];
            g_mul<M>(col, o);
#pragma unroll
            for (int i = 0; i < A; ++i) t[i][j] = o[i];
        }
#pragma unroll
        for (int i = 0; i < A; ++i) g_mul<M>(t[i], u[i]);
#pragma unroll
        for (int xi = 0; xi < A; ++xi)
#pragma unroll
            for (int nu = 0; nu < A; ++nu) us[((xi * A + nu) * KT + kl) * CT + cl] = __float2half_rn(u[xi][nu]);
    }
    __syncthreads();
    const uint4 *in = reinterpret_cast<const uint4 *>(us);
    uint4 *out = reinterpret_cast<uint4 *>(U);
    for (int w = tid; w < A2 * KT; w += NT) {
        const int e = w / KT, k = k0 + w % KT;
        if (k < Kp) out[((size_t)e * (Cp / 8) + by) * Kp + k] = in[w];
    }
}

// Input transform.  V is laid out [e][c/8][b][c%8]; a block takes 8 channels x 64 tiles (512 threads) and writes V as
// 1 KB contiguous per component and wavefront.  VEC: pad 1, W a multiple of 4, M = 4 (columns 1..4 of a tile row are
// one aligned 8-byte load).
template <int M, bool VEC>
__device__ __forceinline__ void input_transform_f16_block(const __half *__restrict__ D, __half *__restrict__ V,
                                                          const Geo &g, int bx, int by, void *smem)
{
    constexpr int A = M + 2, A2 = A * A, TB = F16_TB;
    __half *stage = reinterpret_cast<__half *>(smem);
    const int bl = threadIdx.x % TB, cl = threadIdx.x / TB;
    const int b = bx * TB + bl;
    const int c = by * 8 + cl;
    float d[A][A];
#pragma unroll
    for (int p = 0; p < A; ++p)
#pragma unroll
        for (int q = 0; q < A; ++q) d[p][q] = 0.0f;
    if (c < g.C && b < g.P) {
        const int ty = b % g.Tw;
        const int t2 = b / g.Tw;
        const int tx = t2 % g.Th;
        const int i = t2 / g.Th;
        const int x0 = M * tx - g.pad, y0 = M * ty - g.pad;
        const __half *src = D + ((size_t)i * g.C + c) * g.H * g.W;
#pragma unroll
        for (int p = 0; p < A; ++p) {
            const int x = x0 + p;
            if (x >= 0 && x < g.H) {
                const __half *row = src + (size_t)x * g.W + y0;
                if constexpr (VEC) {
                    const uint2 mid = *reinterpret_cast<const uint2 *>(row + 1);
                    const __half2 h01 = *reinterpret_cast<const __half2 *>(&mid.x);
                    const __half2 h23 = *reinterpret_cast<const __half2 *>(&mid.y);
                    d[p][1] = __low2float(h01);
                    d[p][2] = __high2float(h01);
                    d[p][3] = __low2float(h23);
                    d[p][4] = __high2float(h23);
                    if (y0 >= 0) d[p][0] = __half2float(row[0]);
                    if (y0 + 5 < g.W) d[p][5] = __half2float(row[5]);
                } else {
#pragma unroll
                    for (int q = 0; q < A; ++q) {
                        const int y = y0 + q;
                        if (y >= 0 && y < g.W) d[p][q] = __half2float(row[q]);
                    }
                }
            }
        }
    }
    float t[A][A], v[A][A];
#pragma unroll
    for (int q = 0; q < A; ++q) {
        float col[A], o[A];
#pragma unroll
        for (int p = 0; p < A; ++p) col[p] = d[p][q];
        bt_mul<M>(col, o);
#pragma unroll
        for (int p = 0; p < A; ++p) t[p][q] = o[p];
    }
#pragma unroll
    for (int p = 0; p < A; ++p) bt_mul<M>(t[p], v[p]);
#pragma unroll
    for (int xi = 0; xi < A; ++xi)
#pragma unroll
        for (int nu = 0; nu < A; ++nu) stage[((xi * A + nu) * TB + bl) * 8 + cl] = __float2half_rn(v[xi][nu]);
    __syncthreads();
    uint4 *out = reinterpret_cast<uint4 *>(V);
    const uint4 *in = reinterpret_cast<const uint4 *>(stage);
    for (int u = threadIdx.x; u < A2 * TB; u += 512) {
        const int e = u / TB, ub = bx * TB + u % TB;
        if (ub < g.Pp) out[((size_t)e * (g.Cp / 8) + by) * g.Pp + ub] = in[u];
    }
}

}  // namespace wino

// Loop 1 of Algorithm 1 (Lavin & Gray): u = G g G^T for every filter/channel pair, scattered
// to the alpha^2 matrices U^(xi,nu).  Run once per set of weights (the "FX" variant of
// Section 6); bound by memory traffic: 9 values in, alpha^2 values out per (k, c).
#include "wino_internal.h"
#include "stage_bodies.h"

namespace wino {

// Side job of the first block: 1024 words set to zero for the kernel that follows on the stream (the arrival
// counters of the one-kernel layer, which would otherwise need a launch of their own); null: nothing.
__device__ __forceinline__ void ft_zero1024(unsigned int *zero1024)
{
    if (zero1024 != nullptr && blockIdx.x == 0 && blockIdx.y == 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) zero1024[threadIdx.x + 256 * i] = 0u;
    }
}

template <int M, typename T>
__global__ __launch_bounds__(256) void filter_transform_kernel(const T *__restrict__ G, T *__restrict__ U, int K,
                                                               int C, int Kp, int Cp, unsigned int *zero1024)
{
    __shared__ float gs[FT_LDS];
    ft_zero1024(zero1024);
    filter_transform_block<M, T>(G, U, K, C, Kp, Cp, blockIdx.x, blockIdx.y, gs);
}

// fp16 storage: see filter_transform_f16_block.
template <int M>
__global__ __launch_bounds__(256) void filter_transform_f16_kernel(const __half *__restrict__ G, __half *__restrict__ U,
                                                                   int K, int C, int Kp, int Cp)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[f16_stage_bytes(M)];
    filter_transform_f16_block<M, 256>(G, U, K, C, Kp, Cp, blockIdx.x, blockIdx.y, smem);
}

// Filter transform for the gradient with respect to the input (Section 4.2 of the paper): that
// gradient is the forward algorithm applied to the error tensor with every filter rotated by
// 180 degrees and the roles of filters and channels exchanged.  So the output is a U for a layer
// with K' = C "filters" and C' = K "channels": U'[e][c' = k][k' = c] = (G g~ G^T)[e] with
// g~[u][v] = g_{k,c}[2-u][2-v].  One thread per (k', c'), k' fastest.
template <int M, typename T>
__global__ __launch_bounds__(256) void filter_transform_bwd_kernel(const T *__restrict__ G, T *__restrict__ U, int K,
                                                                   int C, int Kp2, int Cp2, unsigned int *zero1024)
{
    constexpr int A = M + 2;
    ft_zero1024(zero1024);
    const int k2 = blockIdx.x * 64 + threadIdx.x % 64;   // = c of G
    const int c2 = blockIdx.y * 4 + threadIdx.x / 64;    // = k of G
    if (k2 >= Kp2 || c2 >= Cp2) return;
    float g[3][3], t[A][3], u[A][A];
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int j = 0; j < 3; ++j)
            g[i][j] = (k2 < C && c2 < K) ? ld_f<T>(G + ((size_t)c2 * C + k2) * 9 + (2 - i) * 3 + (2 - j)) : 0.0f;
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        float col[3] = {g[0][j], g[1][j], g[2][j]}, o[A];
        g_mul<M>(col, o);
#pragma unroll
        for (int i = 0; i < A; ++i) t[i][j] = o[i];
    }
#pragma unroll
    for (int i = 0; i < A; ++i) g_mul<M>(t[i], u[i]);
#pragma unroll
    for (int xi = 0; xi < A; ++xi)
#pragma unroll
        for (int nu = 0; nu < A; ++nu) {
            const int e = xi * A + nu;
            if constexpr (sizeof(T) == 4) {
                U[((size_t)e * Cp2 + c2) * Kp2 + k2] = u[xi][nu];
            } else {
                U[(((size_t)e * (Cp2 / 8) + c2 / 8) * Kp2 + k2) * 8 + (c2 % 8)] = __float2half_rn(u[xi][nu]);
            }
        }
}

// `g` describes the swapped layer (g.K = channels of the forward layer, g.C = its filters).
hipError_t launch_filter_transform_bwd(const Geo &g, const void *G, void *U, hipStream_t s, unsigned int *zero1024)
{
    dim3 grid((g.Kp + 63) / 64, (g.Cp + 3) / 4), block(256);
    const int K = g.C, C = g.K;   // extents of G[K][C][3][3]
    if (g.dt == WINO_F32) {
        if (g.m == 2)
            filter_transform_bwd_kernel<2, float><<<grid, block, 0, s>>>((const float *)G, (float *)U, K, C, g.Kp, g.Cp, zero1024);
        else if (g.m == 4)
            filter_transform_bwd_kernel<4, float><<<grid, block, 0, s>>>((const float *)G, (float *)U, K, C, g.Kp, g.Cp, zero1024);
        else
            filter_transform_bwd_kernel<6, float><<<grid, block, 0, s>>>((const float *)G, (float *)U, K, C, g.Kp, g.Cp, zero1024);
    } else {
        if (g.m == 2)
            filter_transform_bwd_kernel<2, __half><<<grid, block, 0, s>>>((const __half *)G, (__half *)U, K, C, g.Kp, g.Cp, zero1024);
        else
            filter_transform_bwd_kernel<4, __half><<<grid, block, 0, s>>>((const __half *)G, (__half *)U, K, C, g.Kp, g.Cp, zero1024);
    }
    return hipGetLastError();
}

hipError_t launch_filter_transform(const Geo &g, const void *G, void *U, hipStream_t s, unsigned int *zero1024)
{
    if (g.dt != WINO_F32 && zero1024 != nullptr) return hipErrorInvalidValue;
    dim3 grid((g.Kp + 63) / 64, (g.Cp + 3) / 4), block(256);
    if (g.dt == WINO_F32) {
        if (g.m == 2)
            filter_transform_kernel<2, float><<<grid, block, 0, s>>>((const float *)G, (float *)U, g.K, g.C, g.Kp, g.Cp, zero1024);
        else if (g.m == 4)
            filter_transform_kernel<4, float><<<grid, block, 0, s>>>((const float *)G, (float *)U, g.K, g.C, g.Kp, g.Cp, zero1024);
        else
            filter_transform_kernel<6, float><<<grid, block, 0, s>>>((const float *)G, (float *)U, g.K, g.C, g.Kp, g.Cp, zero1024);
    } else {
        dim3 gridh((g.Kp + 63) / 64, g.Cp / 8);
        if (g.m == 2)
            filter_transform_f16_kernel<2><<<gridh, block, 0, s>>>((const __half *)G, (__half *)U, g.K, g.C, g.Kp, g.Cp);
        else
            filter_transform_f16_kernel<4><<<gridh, block, 0, s>>>((const __half *)G, (__half *)U, g.K, g.C, g.Kp, g.Cp);
    }
    return hipGetLastError();
}

}  // namespace wino

// Loop 4 of Algorithm 1 (Lavin & Gray): gather m_{k,b} from the alpha^2 matrices M^(xi,nu),
// Y_{k,b} = A^T m A (Eq. (10)), and write the m x m outputs that fall inside the image.
// Bound by memory traffic: alpha^2 values in, m^2 values out per (k, b).
#include "wino_internal.h"
#include "transforms.h"

namespace wino {

template <typename T> __device__ __forceinline__ void st_out(T *p, float v);
template <> __device__ __forceinline__ void st_out<float>(float *p, float v) { *p = v; }
template <> __device__ __forceinline__ void st_out<__half>(__half *p, float v) { *p = __float2half_rn(v); }

// One thread per (k, b), b fastest: loads from every M^(xi,nu) row are contiguous across a
// wavefront, and neighbouring threads write neighbouring m-wide output segments.  M is read exactly
// once, so its loads are marked non-temporal (streamed past the caches): 13-20 % more bandwidth on
// the layers whose M does not fit the last-level cache anyway.
template <int M, typename T>
__global__ __launch_bounds__(256) void output_transform_kernel(const float *__restrict__ Min, T *__restrict__ Y, Geo g,
                                                               int splits)
{
    constexpr int A = M + 2;
    const int b = blockIdx.x * 256 + threadIdx.x;
    const int k = blockIdx.y;
    if (b >= g.P) return;
    float mm[A][A];
#pragma unroll
    for (int xi = 0; xi < A; ++xi)
#pragma unroll
        for (int nu = 0; nu < A; ++nu)
            mm[xi][nu] = __builtin_nontemporal_load(Min + ((size_t)(xi * A + nu) * g.Kp + k) * g.Pp + b);
    // partial products of a split channel loop are added here, in the order of the shares
    const size_t zstride = (size_t)A * A * g.Kp * g.Pp;
    for (int z = 1; z < splits; ++z)
#pragma unroll
        for (int xi = 0; xi < A; ++xi)
#pragma unroll
            for (int nu = 0; nu < A; ++nu)
                mm[xi][nu] += Min[z * zstride + ((size_t)(xi * A + nu) * g.Kp + k) * g.Pp + b];
    // t = A^T m (columns), y = t A (rows)
    float t[M][A], y[M][M];
#pragma unroll
    for (int nu = 0; nu < A; ++nu) {
        float col[A], o[M];
#pragma unroll
        for (int xi = 0; xi < A; ++xi) col[xi] = mm[xi][nu];
        at_mul<M>(col, o);
#pragma unroll
        for (int p = 0; p < M; ++p) t[p][nu] = o[p];
    }
#pragma unroll
    for (int p = 0; p < M; ++p) at_mul<M>(t[p], y[p]);

    const int ty = b % g.Tw;
    const int t2 = b / g.Tw;
    const int tx = t2 % g.Th;
    const int i = t2 / g.Th;
    T *dst = Y + ((size_t)i * g.K + k) * g.Ho * g.Wo;
    const int xo = M * tx, yo = M * ty;
    const bool full_row = (yo + M <= g.Wo) && (g.Wo % M == 0) && sizeof(T) == 4;
#pragma unroll
    for (int p = 0; p < M; ++p) {
        if (xo + p >= g.Ho) break;
        T *row = dst + (size_t)(xo + p) * g.Wo + yo;
        if (full_row) {
            if constexpr (M == 4) {
                *reinterpret_cast<float4 *>(row) = make_float4(y[p][0], y[p][1], y[p][2], y[p][3]);
            } else if constexpr (M == 6) {
                // 6-wide segments are 8-byte aligned when Wo is a multiple of 6
                *reinterpret_cast<float2 *>(row) = make_float2(y[p][0], y[p][1]);
                *reinterpret_cast<float2 *>(row + 2) = make_float2(y[p][2], y[p][3]);
                *reinterpret_cast<float2 *>(row + 4) = make_float2(y[p][4], y[p][5]);
            } else {
                *reinterpret_cast<float2 *>(row) = make_float2(y[p][0], y[p][1]);
            }
        } else {
#pragma unroll
            for (int q = 0; q < M; ++q)
                if (yo + q < g.Wo) st_out<T>(row + q, y[p][q]);
        }
    }
}

hipError_t launch_output_transform(const Geo &g, int y_dt, const float *M, void *Y, int splits, hipStream_t s)
{
    dim3 grid((g.P + 255) / 256, g.K), block(256);
    if (y_dt == WINO_F32) {
        if (g.m == 2)
            output_transform_kernel<2, float><<<grid, block, 0, s>>>(M, (float *)Y, g, splits);
        else if (g.m == 4)
            output_transform_kernel<4, float><<<grid, block, 0, s>>>(M, (float *)Y, g, splits);
        else
            output_transform_kernel<6, float><<<grid, block, 0, s>>>(M, (float *)Y, g, splits);
    } else {
        if (g.m == 2)
            output_transform_kernel<2, __half><<<grid, block, 0, s>>>(M, (__half *)Y, g, splits);
        else if (g.m == 4)
            output_transform_kernel<4, __half><<<grid, block, 0, s>>>(M, (__half *)Y, g, splits);
        else
            output_transform_kernel<6, __half><<<grid, block, 0, s>>>(M, (__half *)Y, g, splits);
    }
    return hipGetLastError();
}

}  // namespace wino

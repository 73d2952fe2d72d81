// Loop 2 of Algorithm 1 (Lavin & Gray): gather each alpha x alpha input tile d_{c,b} (tiles
// overlap by r-1 = 2, zeros outside the image -- the implicit zero padding of Section 6),
// v = B^T d B (Eq. (8)), scatter to the alpha^2 matrices V^(xi,nu)[c][b].
// Bound by memory traffic: every input element is needed once, alpha^2/m^2 values are written
// per input element.
#include <stdlib.h>

#include "wino_internal.h"
#include "stage_bodies.h"

namespace wino {

template <int M, typename T, bool VEC = false>
__global__ __launch_bounds__(256) void input_transform_kernel(const T *__restrict__ D, T *__restrict__ V, Geo g)
{
    input_transform_block<M, T, VEC>(D, V, g, blockIdx.x, blockIdx.y);
}

template <int M>
__global__ __launch_bounds__(256) void input_transform_pair_kernel(const float *__restrict__ D, float *__restrict__ V,
                                                                   Geo g)
{
    input_transform_pair_block<M>(D, V, g, blockIdx.x, blockIdx.y);
}

// fp16 storage.  V is laid out [e][c/8][b][c%8] (8 channels of one tile are the 16 bytes a lane
// feeds to the fp16 MFMA), so a (c, b) thread owns isolated 2-byte elements of V.  A workgroup
// therefore takes 8 channels x 64 tiles, transforms in fp32, rounds once to fp16, transposes
// through LDS and writes V in 16-byte units: 1 KB contiguous per component and wavefront.
template <int M, bool VEC>
__global__ __launch_bounds__(512) void input_transform_f16_kernel(const __half *__restrict__ D,
                                                                   __half *__restrict__ V, Geo g)
{
    constexpr int A = M + 2, A2 = A * A, TB = 64;
    __shared__ __half stage[A2 * TB * 8];
    const int bl = threadIdx.x % TB, cl = threadIdx.x / TB;
    const int b = blockIdx.x * TB + bl;
    const int c = blockIdx.y * 8 + cl;
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
                    // pad 1, W a multiple of 4, M = 4: columns 1..4 are one aligned 8-byte load
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
    const int c8 = blockIdx.y;
    uint4 *out = reinterpret_cast<uint4 *>(V);
    const uint4 *in = reinterpret_cast<const uint4 *>(stage);
    for (int u = threadIdx.x; u < A2 * TB; u += 512) {
        const int e = u / TB, ub = blockIdx.x * TB + u % TB;
        if (ub < g.Pp) out[((size_t)e * (g.Cp / 8) + c8) * g.Pp + ub] = in[u];
    }
}

hipError_t launch_input_transform(const Geo &g, const void *D, void *V, hipStream_t s)
{
    dim3 grid((g.Pp + 255) / 256, g.Cp), block(256);
    if (g.dt == WINO_F32 && g.m == 4 && g.pad == 1 && g.W % 8 == 0) {
        dim3 grid2((g.Pp / 2 + 255) / 256, g.Cp);
        input_transform_pair_kernel<4><<<grid2, block, 0, s>>>((const float *)D, (float *)V, g);
        return hipGetLastError();
    }
    if (g.dt == WINO_F32 && g.m == 4 && g.pad == 1 && g.W % 4 == 0) {
        input_transform_kernel<4, float, true><<<grid, block, 0, s>>>((const float *)D, (float *)V, g);
        return hipGetLastError();
    }
    if (g.dt == WINO_F32) {
        if (g.m == 2)
            input_transform_kernel<2, float><<<grid, block, 0, s>>>((const float *)D, (float *)V, g);
        else if (g.m == 4)
            input_transform_kernel<4, float><<<grid, block, 0, s>>>((const float *)D, (float *)V, g);
        else
            input_transform_kernel<6, float><<<grid, block, 0, s>>>((const float *)D, (float *)V, g);
    } else {
        dim3 gridh((g.Pp + 63) / 64, g.Cp / 8), blockh(512);
        const __half *d = (const __half *)D;
        __half *v = (__half *)V;
        if (g.m == 2)
            input_transform_f16_kernel<2, false><<<gridh, blockh, 0, s>>>(d, v, g);
        else if (g.pad == 1 && g.W % 4 == 0)
            input_transform_f16_kernel<4, true><<<gridh, blockh, 0, s>>>(d, v, g);
        else
            input_transform_f16_kernel<4, false><<<gridh, blockh, 0, s>>>(d, v, g);
    }
    return hipGetLastError();
}

}  // namespace wino

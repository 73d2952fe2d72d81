// Loop 2 of Algorithm 1 (Lavin & Gray): gather each alpha x alpha input tile d_{c,b} (tiles
// overlap by r-1 = 2, zeros outside the image -- the implicit zero padding of Section 6),
// v = B^T d B (Eq. (8)), scatter to the alpha^2 matrices V^(xi,nu)[c][b].
// Bound by memory traffic: every input element is needed once, alpha^2/m^2 values are written
// per input element.
#include <stdlib.h>

#include "wino_internal.h"
#include "transforms.h"

namespace wino {

template <typename T> __device__ __forceinline__ float ld_in(const T *p);
template <> __device__ __forceinline__ float ld_in<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float ld_in<__half>(const __half *p) { return __half2float(*p); }

// One thread per (c, b); b is the fastest index of a workgroup so the stores to every
// V^(xi,nu) row are contiguous across a wavefront.  Channels c >= C and tiles b >= P are
// padding and are written as zeros.
typedef float floatx4_v __attribute__((ext_vector_type(4)));

template <int M, typename T, bool VEC = false>
__global__ __launch_bounds__(256) void input_transform_kernel(const T *__restrict__ D, T *__restrict__ V, Geo g)
{
    constexpr int A = M + 2;
    const int b = blockIdx.x * 256 + threadIdx.x;
    const int c = blockIdx.y;
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
__global__ __launch_bounds__(256) void input_transform_pair_kernel(const float *__restrict__ D, float *__restrict__ V,
                                                                   Geo g)
{
    constexpr int A = M + 2;
    static_assert(M == 4, "two 6-wide tiles share 10 columns: 1 + 4 + 4 + 1");
    const int b0 = (blockIdx.x * 256 + threadIdx.x) * 2;   // even; Tw is even, so b0 and b0+1 share a tile row
    const int c = blockIdx.y;
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
    const char *tune = getenv("WINO_IT_PAIR");   // tuning only
    if (g.dt == WINO_F32 && g.m == 4 && g.pad == 1 && g.W % 8 == 0 && !(tune && tune[0] == '0')) {
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

// Direct evaluation of the layer definition, Eq. (1) of Lavin & Gray (2-D correlation summed
// over channels), for layers the fast algorithm does not cover: other filter sizes, strides,
// and layers with very few channels such as the 3-channel first layer of Table 3.
#include "wino_internal.h"

namespace wino {

template <typename T> __device__ __forceinline__ float ld_d(const T *p);
template <> __device__ __forceinline__ float ld_d<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float ld_d<__half>(const __half *p) { return __half2float(*p); }
template <typename T> __device__ __forceinline__ void st_d(T *p, float v);
template <> __device__ __forceinline__ void st_d<float>(float *p, float v) { *p = v; }
template <> __device__ __forceinline__ void st_d<__half>(__half *p, float v) { *p = __float2half_rn(v); }

// One thread per output pixel, KB filters at a time held in registers.  The filter block is
// staged in LDS as [c][u][v][k] so a thread fetches 4 filters per LDS read (all lanes read the
// same address: broadcast).  Loads of D and stores of Y are contiguous across a wavefront.
constexpr int DC_KB = 16;
constexpr int DC_LDS_FLOATS = 8192;

template <typename T>
__global__ __launch_bounds__(256) void direct_conv_kernel(const T *__restrict__ D, const T *__restrict__ G,
                                                          T *__restrict__ Y, int N, int C, int H, int W, int K, int R,
                                                          int S, int pad, int stride, int Ho, int Wo, int CC)
{
    __shared__ float gs[DC_LDS_FLOATS];
    const int pix = blockIdx.x * 256 + threadIdx.x;
    const int k0 = blockIdx.y * DC_KB;
    const int i = blockIdx.z;
    const bool live = pix < Ho * Wo;
    const int ox = live ? pix / Wo : 0, oy = live ? pix % Wo : 0;
    const int RS = R * S;
    float acc[DC_KB];
#pragma unroll
    for (int kk = 0; kk < DC_KB; ++kk) acc[kk] = 0.0f;
    const T *Di = D + (size_t)i * C * H * W;
    for (int c0 = 0; c0 < C; c0 += CC) {
        const int cn = min(CC, C - c0);
        __syncthreads();
        for (int idx = threadIdx.x; idx < cn * RS * DC_KB; idx += 256) {
            const int kk = idx % DC_KB, j = idx / DC_KB;  // j = cc*RS + uv
            const int k = k0 + kk;
            gs[idx] = (k < K) ? ld_d<T>(G + ((size_t)k * C + c0) * RS + j) : 0.0f;
        }
        __syncthreads();
        if (live) {
            for (int cc = 0; cc < cn; ++cc) {
                const T *Dc = Di + (size_t)(c0 + cc) * H * W;
                for (int u = 0; u < R; ++u) {
                    const int x = ox * stride + u - pad;
                    if (x < 0 || x >= H) continue;
                    for (int v = 0; v < S; ++v) {
                        const int y = oy * stride + v - pad;
                        if (y < 0 || y >= W) continue;
                        const float d = ld_d<T>(Dc + (size_t)x * W + y);
                        const float4 *w = reinterpret_cast<const float4 *>(&gs[((cc * R + u) * S + v) * DC_KB]);
#pragma unroll
                        for (int q = 0; q < DC_KB / 4; ++q) {
                            const float4 f = w[q];
                            acc[4 * q + 0] = fmaf(d, f.x, acc[4 * q + 0]);
                            acc[4 * q + 1] = fmaf(d, f.y, acc[4 * q + 1]);
                            acc[4 * q + 2] = fmaf(d, f.z, acc[4 * q + 2]);
                            acc[4 * q + 3] = fmaf(d, f.w, acc[4 * q + 3]);
                        }
                    }
                }
            }
        }
    }
    if (live) {
#pragma unroll
        for (int kk = 0; kk < DC_KB; ++kk)
            if (k0 + kk < K) st_d<T>(Y + (((size_t)i * K + k0 + kk) * Ho + ox) * Wo + oy, acc[kk]);
    }
}

hipError_t launch_direct_conv(int N, int C, int H, int W, int K, int R, int S, int pad, int stride, int dt,
                              const void *D, const void *G, void *Y, hipStream_t s)
{
    const int Ho = (H + 2 * pad - R) / stride + 1, Wo = (W + 2 * pad - S) / stride + 1;
    int CC = DC_LDS_FLOATS / (DC_KB * R * S);
    if (CC < 1) return hipErrorInvalidValue;
    if (CC > C) CC = C;
    dim3 grid((Ho * Wo + 255) / 256, (K + DC_KB - 1) / DC_KB, N), block(256);
    if (grid.y > 65535 || grid.z > 65535) return hipErrorInvalidValue;
    if (dt == WINO_F32)
        direct_conv_kernel<float><<<grid, block, 0, s>>>((const float *)D, (const float *)G, (float *)Y, N, C, H, W, K,
                                                         R, S, pad, stride, Ho, Wo, CC);
    else
        direct_conv_kernel<__half><<<grid, block, 0, s>>>((const __half *)D, (const __half *)G, (__half *)Y, N, C, H,
                                                          W, K, R, S, pad, stride, Ho, Wo, CC);
    return hipGetLastError();
}

}  // namespace wino

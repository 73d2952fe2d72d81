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

// 3 x 3, stride 1 specialisation (the 3-channel first layer of Table 3 is its main use): one
// thread computes 4 neighbouring outputs of a row for DC_KB filters.  Per channel it holds the
// 3 x 6 input window in registers (one aligned 16-byte load and two single loads per row), and
// every 16-byte broadcast LDS read of 4 filter taps feeds 16 FMAs.  Stores are 16 bytes per
// filter and contiguous across a wavefront.
typedef float floatx4_dc __attribute__((ext_vector_type(4)));

// four consecutive elements from an address aligned to four elements, widened to fp32
template <typename T> __device__ __forceinline__ floatx4_dc ld4_d(const T *p);
template <> __device__ __forceinline__ floatx4_dc ld4_d<float>(const float *p)
{
    return *reinterpret_cast<const floatx4_dc *>(p);
}
template <> __device__ __forceinline__ floatx4_dc ld4_d<__half>(const __half *p)
{
    const uint2 raw = *reinterpret_cast<const uint2 *>(p);
    const __half2 a = *reinterpret_cast<const __half2 *>(&raw.x), b = *reinterpret_cast<const __half2 *>(&raw.y);
    return floatx4_dc{__low2float(a), __high2float(a), __low2float(b), __high2float(b)};
}
template <typename T> __device__ __forceinline__ void st4_d(T *p, floatx4_dc v);
template <> __device__ __forceinline__ void st4_d<float>(float *p, floatx4_dc v)
{
    *reinterpret_cast<floatx4_dc *>(p) = v;
}
template <> __device__ __forceinline__ void st4_d<__half>(__half *p, floatx4_dc v)
{
    const __half2 a = __floats2half2_rn(v[0], v[1]), b = __floats2half2_rn(v[2], v[3]);
    uint2 raw;
    raw.x = *reinterpret_cast<const unsigned *>(&a);
    raw.y = *reinterpret_cast<const unsigned *>(&b);
    *reinterpret_cast<uint2 *>(p) = raw;
}

template <typename T>
__global__ __launch_bounds__(256) void direct_conv3x3_kernel(const T *__restrict__ D, const T *__restrict__ G,
                                                             T *__restrict__ Y, int C, int H, int W, int K, int pad,
                                                             int Ho, int Wo, int Wq, int CC)
{
    __shared__ float gs[DC_LDS_FLOATS];
    const int item = blockIdx.x * 256 + threadIdx.x;   // (output row, group of 4 columns)
    const int k0 = blockIdx.y * DC_KB;
    const int i = blockIdx.z;
    const bool live = item < Ho * Wq;
    const int ox = live ? item / Wq : 0, oy = live ? (item % Wq) * 4 : 0;
    const int y0 = oy - pad;                            // first input column of the window
    const bool vec_in = (W % 4 == 0) && (pad == 1);     // columns y0+1..y0+4 are then one aligned float4
    float acc[4][DC_KB];
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int kk = 0; kk < DC_KB; ++kk) acc[p][kk] = 0.0f;
    const T *Di = D + (size_t)i * C * H * W;
    for (int c0 = 0; c0 < C; c0 += CC) {
        const int cn = min(CC, C - c0);
        __syncthreads();
        for (int idx = threadIdx.x; idx < cn * 9 * DC_KB; idx += 256) {
            const int kk = idx % DC_KB, j = idx / DC_KB;
            const int k = k0 + kk;
            gs[idx] = (k < K) ? ld_d<T>(G + ((size_t)k * C + c0) * 9 + j) : 0.0f;
        }
        __syncthreads();
        if (!live) continue;
        for (int cc = 0; cc < cn; ++cc) {
            const T *Dc = Di + (size_t)(c0 + cc) * H * W;
            float win[3][6];
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                const int x = ox + u - pad;
                const bool rok = x >= 0 && x < H;
                const T *row = Dc + (size_t)(rok ? x : 0) * W;
                if (vec_in) {
                    const floatx4_dc mid = rok ? ld4_d<T>(row + y0 + 1) : floatx4_dc{0.f, 0.f, 0.f, 0.f};
                    win[u][0] = (rok && y0 >= 0) ? ld_d<T>(row + y0) : 0.0f;
                    win[u][1] = mid[0];
                    win[u][2] = mid[1];
                    win[u][3] = mid[2];
                    win[u][4] = mid[3];
                    win[u][5] = (rok && y0 + 5 < W) ? ld_d<T>(row + y0 + 5) : 0.0f;
                } else {
#pragma unroll
                    for (int q = 0; q < 6; ++q) {
                        const int y = y0 + q;
                        win[u][q] = (rok && y >= 0 && y < W) ? ld_d<T>(row + y) : 0.0f;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 3; ++u)
#pragma unroll
                for (int v = 0; v < 3; ++v) {
                    const floatx4_dc *wv = reinterpret_cast<const floatx4_dc *>(&gs[((cc * 3 + u) * 3 + v) * DC_KB]);
#pragma unroll
                    for (int q4 = 0; q4 < DC_KB / 4; ++q4) {
                        const floatx4_dc f = wv[q4];
#pragma unroll
                        for (int p = 0; p < 4; ++p) {
                            const float d = win[u][p + v];
                            acc[p][4 * q4 + 0] = fmaf(d, f[0], acc[p][4 * q4 + 0]);
                            acc[p][4 * q4 + 1] = fmaf(d, f[1], acc[p][4 * q4 + 1]);
                            acc[p][4 * q4 + 2] = fmaf(d, f[2], acc[p][4 * q4 + 2]);
                            acc[p][4 * q4 + 3] = fmaf(d, f[3], acc[p][4 * q4 + 3]);
                        }
                    }
                }
        }
    }
    if (!live) return;
    const bool vec_out = (Wo % 4 == 0);
#pragma unroll
    for (int kk = 0; kk < DC_KB; ++kk) {
        if (k0 + kk < K) {
            T *dst = Y + (((size_t)i * K + k0 + kk) * Ho + ox) * Wo + oy;
            if (vec_out) {
                st4_d<T>(dst, floatx4_dc{acc[0][kk], acc[1][kk], acc[2][kk], acc[3][kk]});
            } else {
#pragma unroll
                for (int p = 0; p < 4; ++p)
                    if (oy + p < Wo) st_d<T>(dst + p, acc[p][kk]);
            }
        }
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
    if (R == 3 && S == 3 && stride == 1) {
        const int Wq = (Wo + 3) / 4;
        dim3 grid3((Ho * Wq + 255) / 256, grid.y, N);
        if (dt == WINO_F32)
            direct_conv3x3_kernel<float><<<grid3, block, 0, s>>>((const float *)D, (const float *)G, (float *)Y, C, H, W,
                                                                 K, pad, Ho, Wo, Wq, CC);
        else
            direct_conv3x3_kernel<__half><<<grid3, block, 0, s>>>((const __half *)D, (const __half *)G, (__half *)Y, C,
                                                                  H, W, K, pad, Ho, Wo, Wq, CC);
        return hipGetLastError();
    }
    if (dt == WINO_F32)
        direct_conv_kernel<float><<<grid, block, 0, s>>>((const float *)D, (const float *)G, (float *)Y, N, C, H, W, K,
                                                         R, S, pad, stride, Ho, Wo, CC);
    else
        direct_conv_kernel<__half><<<grid, block, 0, s>>>((const __half *)D, (const __half *)G, (__half *)Y, N, C, H,
                                                          W, K, R, S, pad, stride, Ho, Wo, CC);
    return hipGetLastError();
}

}  // namespace wino

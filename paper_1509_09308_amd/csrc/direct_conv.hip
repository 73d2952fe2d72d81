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

// store that does not keep the line in the caches (an output plane is written once and is far larger than they are)
template <typename T> __device__ __forceinline__ void st_nt_d(T *p, float v);
template <> __device__ __forceinline__ void st_nt_d<float>(float *p, float v) { __builtin_nontemporal_store(v, p); }
template <> __device__ __forceinline__ void st_nt_d<__half>(__half *p, float v)
{
    __builtin_nontemporal_store(__builtin_bit_cast(unsigned short, __float2half_rn(v)), reinterpret_cast<unsigned short *>(p));
}

// 3 x 3, stride 1 with at most 4 channels (the first layer of Table 3) on the matrix units.  Eq. (1) for one
// output row is a product of the K x 9C matrix of filter taps with the 9C x Wo matrix whose column y holds the
// 3 x 3 x C window of output y: v_mfma_f32_32x32x2_f32 takes 32 filters x 2 taps x 32 neighbouring outputs of a
// row.  A workgroup owns DM_RB output rows of one image (one per wavefront) and 64 filters: the DM_RB + 2 input
// rows of every channel are staged in LDS once (fp32, zero halo = the padding), the taps of the 64 filters stay in
// registers as A operands for the whole kernel, and lane (y, h) fetches the B operand of step t -- tap 2t + h of
// window y -- with one LDS read at a per-lane offset fixed for the kernel.  Per 32 outputs: ceil(9C/2) LDS reads,
// 2 ceil(9C/2) MFMAs, and stores of 32 neighbouring outputs per filter (tried and slower: two outputs per lane
// with a lane swap, 64 neighbouring outputs per store).  The layer is bound by writing Y (C = 3,
// K = 64: 21 output values per input value), which this form approaches because the arithmetic no longer competes
// with the stores for the vector ALU.  A small problem (rb = 1) gives every workgroup a single output row, whose
// 32-output blocks the four wavefronts share, so that a batch of one still has a few hundred workgroups.
typedef float floatx16_dc __attribute__((ext_vector_type(16)));
constexpr int DM_RB = 4;

template <typename T, int CT>
__global__ __launch_bounds__(64 * DM_RB) void direct_conv3x3_mfma_kernel(const T *__restrict__ D,
                                                                         const T *__restrict__ G, T *__restrict__ Y,
                                                                         int H, int W, int K, int pad, int Ho, int Wo,
                                                                         int WS, int rb)
{
    constexpr int J = 9 * CT, NT = (J + 1) / 2;                   // taps, MFMA steps
    const int PR = rb + 2;                                        // staged rows per channel
    extern __shared__ float patch[];                              // [c][row][WS]; input column y sits at index y + 4
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, li = lane & 31, lg = lane >> 5;
    const int x0 = blockIdx.x * rb;                               // first output row of the workgroup
    const int k0 = blockIdx.y * 64;
    const int i = blockIdx.z;

    // A operands: filter k0 + 32 g + li, tap 2 t + lg (0 beyond the filters and beyond the 9C taps)
    float a[2][NT];
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int k = k0 + 32 * g + li, j = 2 * t + lg;
            a[g][t] = (k < K && j < J) ? ld_d<T>(G + (size_t)k * J + j) : 0.0f;
        }
    // LDS offset of tap 2 t + lg relative to (row of the output, column of the output); a tap past 9C repeats
    // tap 0 (its A operand is 0; the B operand only has to be a number the window really contains)
    int off[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int j = (2 * t + lg < J) ? 2 * t + lg : 0;
        const int c = j / 9, u = (j % 9) / 3, v = j % 3;
        off[t] = (c * PR + u) * WS + v + 4 - pad;
    }

    // stage input rows x0 - pad .. x0 - pad + PR - 1 of every channel: 16-byte loads, zeros outside the image
    const T *Di = D + (size_t)i * CT * H * W;
    const int W4 = W / 4;
    for (int idx = tid; idx < CT * PR * W4; idx += 64 * DM_RB) {
        const int q = idx % W4, r = (idx / W4) % PR, c = idx / (W4 * PR);
        const int x = x0 - pad + r;
        floatx4_dc v = {0.f, 0.f, 0.f, 0.f};
        if (x >= 0 && x < H) v = ld4_d<T>(Di + ((size_t)c * H + x) * W + 4 * q);
        *reinterpret_cast<floatx4_dc *>(&patch[(c * PR + r) * WS + 4 + 4 * q]) = v;
    }
    for (int idx = tid; idx < CT * PR; idx += 64 * DM_RB) {       // the columns left and right of the image
        patch[idx * WS + 3] = 0.0f;
        patch[idx * WS + 4 + W] = 0.0f;
    }
    __syncthreads();

    const int xl = rb == 1 ? 0 : wave;                             // this wavefront's output row within the workgroup's
    const int x = x0 + xl;
    if (x >= Ho) return;
    const float *prow = patch + xl * WS + li;
    T *yrow = Y + (((size_t)i * K + k0 + 4 * lg) * Ho + x) * Wo + li;
    const size_t kstride = (size_t)Ho * Wo;
    for (int yb = rb == 1 ? 32 * wave : 0; yb < Wo; yb += rb == 1 ? 32 * DM_RB : 32) {
        floatx16_dc acc[2];
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[g][r] = 0.0f;
        float b[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) b[t] = prow[yb + off[t]];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int g = 0; g < 2; ++g) acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g][t], b[t], acc[g], 0, 0, 0);
        // accumulator register r of lane (li, lg) is filter 32 g + 8 (r / 4) + 4 lg + r % 4, output yb + li
        if (yb + li < Wo) {
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kk = 32 * g + 8 * (r / 4) + (r % 4);
                    if (k0 + 4 * lg + kk < K) st_nt_d<T>(yrow + (size_t)kk * kstride + yb, acc[g][r]);
                }
        }
    }
}

template <typename T, int CT>
static hipError_t launch_direct_mfma(int N, int H, int W, int K, int pad, int Ho, int Wo, const void *D, const void *G,
                                     void *Y, hipStream_t s)
{
    const int WS = (Wo + 31) / 32 * 32 + 8;   // a lane past the last output still reads inside its row
    const long long wgs = (long long)((Ho + DM_RB - 1) / DM_RB) * ((K + 63) / 64) * N;
    const int rb = wgs < 512 ? 1 : DM_RB;     // one output row per workgroup when bands of rows would not fill the chip
    const size_t lds = (size_t)CT * (rb + 2) * WS * sizeof(float);
    dim3 grid((Ho + rb - 1) / rb, (K + 63) / 64, N);
    direct_conv3x3_mfma_kernel<T, CT><<<grid, dim3(64 * DM_RB), lds, s>>>((const T *)D, (const T *)G, (T *)Y, H, W, K, pad,
                                                                        Ho, Wo, WS, rb);
    return hipGetLastError();
}

// The matrix-unit form serves 3 x 3, stride 1, 1-4 channels, rows that are a whole number of 16-byte units, and
// an LDS patch within the 64 KB a launch gets without asking.
static bool direct_mfma_ok(int C, int H, int W, int K, int R, int S, int pad, int stride, int Ho, int Wo, int N)
{
    if (R != 3 || S != 3 || stride != 1 || C < 1 || C > 4 || W % 4 != 0 || pad < 0 || pad > 1) return false;
    const long long WS = (Wo + 31) / 32 * 32 + 8;
    if ((long long)C * (DM_RB + 2) * WS * 4 > 65536) return false;
    return (Ho + DM_RB - 1) / DM_RB <= 0x7fffffff && (K + 63) / 64 <= 65535 && N <= 65535;
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
    // (D is read in 16-byte units)
    if (direct_mfma_ok(C, H, W, K, R, S, pad, stride, Ho, Wo, N) && (size_t)D % 16 == 0) {
        const bool f32 = dt == WINO_F32;
        switch (C) {
        case 1: return f32 ? launch_direct_mfma<float, 1>(N, H, W, K, pad, Ho, Wo, D, G, Y, s)
                           : launch_direct_mfma<__half, 1>(N, H, W, K, pad, Ho, Wo, D, G, Y, s);
        case 2: return f32 ? launch_direct_mfma<float, 2>(N, H, W, K, pad, Ho, Wo, D, G, Y, s)
                           : launch_direct_mfma<__half, 2>(N, H, W, K, pad, Ho, Wo, D, G, Y, s);
        case 3: return f32 ? launch_direct_mfma<float, 3>(N, H, W, K, pad, Ho, Wo, D, G, Y, s)
                           : launch_direct_mfma<__half, 3>(N, H, W, K, pad, Ho, Wo, D, G, Y, s);
        default: return f32 ? launch_direct_mfma<float, 4>(N, H, W, K, pad, Ho, Wo, D, G, Y, s)
                            : launch_direct_mfma<__half, 4>(N, H, W, K, pad, Ho, Wo, D, G, Y, s);
        }
    }
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

// The 1-D transforms of F(2,3) (Eq. (7)) and F(4,3) (Eq. (15)) of Lavin & Gray, written as
// straight-line code on registers.  The 2-D transforms of Eq. (8) apply them to the rows and
// then the columns of a tile.  All arithmetic is fp32.
#pragma once
#include <hip/hip_runtime.h>

namespace wino {

// out = B^T in   (data transform, alpha inputs -> alpha outputs)
template <int M> __device__ __forceinline__ void bt_mul(const float *in, float *out);
template <> __device__ __forceinline__ void bt_mul<2>(const float *d, float *o)
{
    o[0] = d[0] - d[2];
    o[1] = d[1] + d[2];
    o[2] = d[2] - d[1];
    o[3] = d[1] - d[3];
}
template <> __device__ __forceinline__ void bt_mul<4>(const float *d, float *o)
{
    // rows of B^T: (4,0,-5,0,1,0) (0,-4,-4,1,1,0) (0,4,-4,-1,1,0) (0,-2,-1,2,1,0) (0,2,-1,-2,1,0) (0,4,0,-5,0,1)
    const float s42 = d[4] - 4.0f * d[2];   // d4 - 4 d2
    const float s31 = d[3] - 4.0f * d[1];   // d3 - 4 d1
    const float t42 = d[4] - d[2];          // d4 - d2
    const float t31 = 2.0f * (d[3] - d[1]); // 2 d3 - 2 d1
    o[0] = 4.0f * d[0] - 5.0f * d[2] + d[4];
    o[1] = s42 + s31;
    o[2] = s42 - s31;
    o[3] = t42 + t31;
    o[4] = t42 - t31;
    o[5] = 4.0f * d[1] - 5.0f * d[3] + d[5];
}

// out = G in   (filter transform, 3 inputs -> alpha outputs)
template <int M> __device__ __forceinline__ void g_mul(const float *in, float *out);
template <> __device__ __forceinline__ void g_mul<2>(const float *g, float *o)
{
    const float s = g[0] + g[2];
    o[0] = g[0];
    o[1] = 0.5f * (s + g[1]);
    o[2] = 0.5f * (s - g[1]);
    o[3] = g[2];
}
template <> __device__ __forceinline__ void g_mul<4>(const float *g, float *o)
{
    const float s = g[0] + g[2];
    const float t = g[0] + 4.0f * g[2];
    o[0] = 0.25f * g[0];
    o[1] = (-1.0f / 6.0f) * (s + g[1]);
    o[2] = (-1.0f / 6.0f) * (s - g[1]);
    o[3] = (1.0f / 24.0f) * (t + 2.0f * g[1]);
    o[4] = (1.0f / 24.0f) * (t - 2.0f * g[1]);
    o[5] = g[2];
}

// out = A^T in   (inverse transform, alpha inputs -> m outputs)
template <int M> __device__ __forceinline__ void at_mul(const float *in, float *out);
template <> __device__ __forceinline__ void at_mul<2>(const float *x, float *o)
{
    o[0] = x[0] + x[1] + x[2];
    o[1] = x[1] - x[2] - x[3];
}
template <> __device__ __forceinline__ void at_mul<4>(const float *x, float *o)
{
    const float p12 = x[1] + x[2], m12 = x[1] - x[2];
    const float p34 = x[3] + x[4], m34 = x[3] - x[4];
    o[0] = x[0] + p12 + p34;
    o[1] = m12 + 2.0f * m34;
    o[2] = p12 + 4.0f * p34;
    o[3] = m12 + 8.0f * m34 + x[5];
}

}  // namespace wino

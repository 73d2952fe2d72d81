// The 1-D transforms of F(2,3) (Eq. (7)) and F(4,3) (Eq. (15)) of Lavin & Gray, written as
// straight-line code on registers, and those of F(6,3), which Section 4.3 mentions without
// printing: interpolation points 0, 1, -1, 2, -2, 1/2, -1/2, infinity (the points of Eq. (15)
// plus +-1/2), rows scaled so that B^T and A^T have unit leading entries.  The 2-D transforms of
// Eq. (8) apply them to the rows and then the columns of a tile.  All arithmetic is fp32.
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
    o[0] = fmaf(4.0f, d[0], fmaf(-5.0f, d[2], d[4]));   // two instructions (written as a sum of products: three)
    o[1] = s42 + s31;
    o[2] = s42 - s31;
    o[3] = t42 + t31;
    o[4] = t42 - t31;
    o[5] = fmaf(4.0f, d[1], fmaf(-5.0f, d[3], d[5]));
}

template <> __device__ __forceinline__ void bt_mul<6>(const float *d, float *o)
{
    // rows of B^T: (1,0,-21/4,0,21/4,0,-1,0) (0,1,1,-17/4,-17/4,1,1,0) (0,-1,1,17/4,-17/4,-1,1,0)
    // (0,1/2,1/4,-5/2,-5/4,2,1,0) (0,-1/2,1/4,5/2,-5/4,-2,1,0) (0,2,4,-5/2,-5,1/2,1,0)
    // (0,-2,4,5/2,-5,-1/2,1,0) (0,-1,0,21/4,0,-21/4,0,1)
    const float e1 = d[2] + d[6] - 4.25f * d[4], o1 = d[1] + d[5] - 4.25f * d[3];
    const float e2 = 0.25f * d[2] - 1.25f * d[4] + d[6], o2 = 0.5f * d[1] - 2.5f * d[3] + 2.0f * d[5];
    const float e3 = 4.0f * d[2] - 5.0f * d[4] + d[6], o3 = 2.0f * d[1] - 2.5f * d[3] + 0.5f * d[5];
    o[0] = d[0] - d[6] + 5.25f * (d[4] - d[2]);
    o[1] = e1 + o1;
    o[2] = e1 - o1;
    o[3] = e2 + o2;
    o[4] = e2 - o2;
    o[5] = e3 + o3;
    o[6] = e3 - o3;
    o[7] = d[7] - d[1] + 5.25f * (d[3] - d[5]);
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

template <> __device__ __forceinline__ void g_mul<6>(const float *g, float *o)
{
    // rows of G: (1,0,0) -2/9 (1,1,1) -2/9 (1,-1,1) 1/90 (1,2,4) 1/90 (1,-2,4) 8/45 (4,2,1) 8/45 (4,-2,1) (0,0,1)
    const float s = g[0] + g[2];
    const float t = g[0] + 4.0f * g[2];
    const float w = 4.0f * g[0] + g[2];
    o[0] = g[0];
    o[1] = (-2.0f / 9.0f) * (s + g[1]);
    o[2] = (-2.0f / 9.0f) * (s - g[1]);
    o[3] = (1.0f / 90.0f) * (t + 2.0f * g[1]);
    o[4] = (1.0f / 90.0f) * (t - 2.0f * g[1]);
    o[5] = (8.0f / 45.0f) * (w + 2.0f * g[1]);
    o[6] = (8.0f / 45.0f) * (w - 2.0f * g[1]);
    o[7] = g[2];
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

template <> __device__ __forceinline__ void at_mul<6>(const float *x, float *o)
{
    // rows of A^T: (1,1,1,1,1,1,1,0) and (0, 1, -1, 2^i, -(2^i), 2^-i, -(2^-i), [i = 5]) for i = 1..5
    const float p12 = x[1] + x[2], m12 = x[1] - x[2];
    const float p34 = x[3] + x[4], m34 = x[3] - x[4];
    const float p56 = x[5] + x[6], m56 = x[5] - x[6];
    o[0] = x[0] + p12 + p34 + p56;
    o[1] = m12 + 2.0f * m34 + 0.5f * m56;
    o[2] = p12 + 4.0f * p34 + 0.25f * p56;
    o[3] = m12 + 8.0f * m34 + 0.125f * m56;
    o[4] = p12 + 16.0f * p34 + 0.0625f * p56;
    o[5] = m12 + 32.0f * m34 + 0.03125f * m56 + x[7];
}

}  // namespace wino

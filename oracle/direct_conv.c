/*
 * TEST INFRASTRUCTURE ONLY -- the CPU oracle for the convnet-layer forward pass.
 *
 * This file is the plain definition of what the fast algorithm must reproduce: the
 * layer output of Section 3, Eq. (1) of Lavin & Gray, "Fast Algorithms for
 * Convolutional Neural Networks" -- a 2-D correlation (no filter flip) of every image
 * channel with the matching filter channel, summed over channels.  Following the
 * accuracy protocol of Section 7 (Experiments), every output is reduced in a
 * double-precision accumulator.
 *
 * Readings taken where the paper is silent (Eq. (1) is 1-based with swapped summation
 * limits and never states padding): indices are 0-based; the first spatial index of G
 * pairs with the first spatial index of D (rows, H), the second with columns (W);
 * zero padding `pad` on every side, stride `stride`; output extent
 * (H + 2*pad - R)/stride + 1.  With R=S=3, pad=1, stride=1 the output is H x W, which
 * is what Table 3's GFLOP column implies.
 *
 * Nothing here is blocked, fused, vectorised by hand or shared with the GPU library.
 * Only tests, the smoke check and the CPU-baseline leg of the benchmark may call it.
 * Parity pins: tests/test_oracle_direct.py (brute force, torch float64 conv2d,
 * delta-filter identity, linearity, shift equivariance).
 */
#include <stddef.h>
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static inline int out_extent(int in, int pad, int filt, int stride)
{
    return (in + 2 * pad - filt) / stride + 1;
}

/* Eq. (1), inputs already widened to double.  Layouts: D[N][C][H][W], G[K][C][R][S],
 * Y[N][K][Ho][Wo], all dense row-major.  Summation order for one output is c, u, v. */
void oracle_conv2d_fwd_f64(int N, int C, int H, int W, int K, int R, int S, int pad, int stride,
                           const double *D, const double *G, double *Y)
{
    const int Ho = out_extent(H, pad, R, stride), Wo = out_extent(W, pad, S, stride);
    #pragma omp parallel for collapse(2) schedule(static)
    for (int i = 0; i < N; ++i)
        for (int k = 0; k < K; ++k)
            for (int x = 0; x < Ho; ++x)
                for (int y = 0; y < Wo; ++y) {
                    double acc = 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int u = 0; u < R; ++u)
                            for (int v = 0; v < S; ++v) {
                                const int xx = x * stride + u - pad;
                                const int yy = y * stride + v - pad;
                                if (xx >= 0 && xx < H && yy >= 0 && yy < W)
                                    acc += D[(((size_t)i * C + c) * H + xx) * W + yy] *
                                           G[(((size_t)k * C + c) * R + u) * S + v];
                            }
                    Y[(((size_t)i * K + k) * Ho + x) * Wo + y] = acc;
                }
}

/* Same definition on the stored single-precision tensors (fp16 tensors are widened to
 * fp32 exactly by the caller): each product and the whole reduction are in double. */
void oracle_conv2d_fwd_f32in(int N, int C, int H, int W, int K, int R, int S, int pad, int stride,
                             const float *D, const float *G, double *Y)
{
    const int Ho = out_extent(H, pad, R, stride), Wo = out_extent(W, pad, S, stride);
    #pragma omp parallel for collapse(2) schedule(static)
    for (int i = 0; i < N; ++i)
        for (int k = 0; k < K; ++k)
            for (int x = 0; x < Ho; ++x)
                for (int y = 0; y < Wo; ++y) {
                    double acc = 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int u = 0; u < R; ++u)
                            for (int v = 0; v < S; ++v) {
                                const int xx = x * stride + u - pad;
                                const int yy = y * stride + v - pad;
                                if (xx >= 0 && xx < H && yy >= 0 && yy < W)
                                    acc += (double)D[(((size_t)i * C + c) * H + xx) * W + yy] *
                                           (double)G[(((size_t)k * C + c) * R + u) * S + v];
                            }
                    Y[(((size_t)i * K + k) * Ho + x) * Wo + y] = acc;
                }
}

/* Eq. (1) evaluated one output at a time: pts holds npts quadruples (i, k, x, y); out[j]
 * receives Y[i][k][x][y].  Used where a whole layer is too large to recompute on the CPU. */
void oracle_conv2d_points_f32in(int N, int C, int H, int W, int K, int R, int S, int pad, int stride,
                                const float *D, const float *G, long npts, const int32_t *pts,
                                double *out)
{
    (void)N; (void)K;
    #pragma omp parallel for schedule(static)
    for (long j = 0; j < npts; ++j) {
        const int i = pts[4 * j + 0], k = pts[4 * j + 1], x = pts[4 * j + 2], y = pts[4 * j + 3];
        double acc = 0.0;
        for (int c = 0; c < C; ++c)
            for (int u = 0; u < R; ++u)
                for (int v = 0; v < S; ++v) {
                    const int xx = x * stride + u - pad;
                    const int yy = y * stride + v - pad;
                    if (xx >= 0 && xx < H && yy >= 0 && yy < W)
                        acc += (double)D[(((size_t)i * C + c) * H + xx) * W + yy] *
                               (double)G[(((size_t)k * C + c) * R + u) * S + v];
                }
        out[j] = acc;
    }
}

/* Gradient of Eq. (1) with respect to the images (Section 4.2: the backpropagated error, of
 * dimension N x K x Ho x Wo, correlated with the flipped filters).  Written out from Eq. (1)
 * itself: Y[i][k][x'][y'] depends on D[i][c][x'*stride+u-pad][y'*stride+v-pad] with weight
 * G[k][c][u][v], so
 *   dD[i][c][x][y] = sum_k sum_u sum_v E[i][k][x'][y'] * G[k][c][u][v]
 * over the (u, v) for which x' = (x + pad - u)/stride and y' = (y + pad - v)/stride are integers
 * inside the output.  E is the error tensor [N][K][Ho][Wo]; the result is [N][C][H][W] in fp64. */
void oracle_conv2d_bwd_data_f64(int N, int C, int H, int W, int K, int R, int S, int pad, int stride,
                                const double *E, const double *G, double *dD)
{
    const int Ho = out_extent(H, pad, R, stride), Wo = out_extent(W, pad, S, stride);
    #pragma omp parallel for collapse(2) schedule(static)
    for (int i = 0; i < N; ++i)
        for (int c = 0; c < C; ++c)
            for (int x = 0; x < H; ++x)
                for (int y = 0; y < W; ++y) {
                    double acc = 0.0;
                    for (int k = 0; k < K; ++k)
                        for (int u = 0; u < R; ++u)
                            for (int v = 0; v < S; ++v) {
                                const int xs = x + pad - u, ys = y + pad - v;
                                if (xs < 0 || ys < 0 || xs % stride || ys % stride) continue;
                                const int xo = xs / stride, yo = ys / stride;
                                if (xo < Ho && yo < Wo)
                                    acc += E[(((size_t)i * K + k) * Ho + xo) * Wo + yo] *
                                           G[(((size_t)k * C + c) * R + u) * S + v];
                            }
                    dD[(((size_t)i * C + c) * H + x) * W + y] = acc;
                }
}

/* The same sum for selected elements of dD: pts holds npts quadruples (i, c, x, y); inputs are the
 * stored single-precision tensors, products and sums in double. */
void oracle_conv2d_bwd_data_points_f32in(int N, int C, int H, int W, int K, int R, int S, int pad, int stride,
                                         const float *E, const float *G, long npts, const int32_t *pts,
                                         double *out)
{
    (void)N;
    const int Ho = out_extent(H, pad, R, stride), Wo = out_extent(W, pad, S, stride);
    #pragma omp parallel for schedule(static)
    for (long j = 0; j < npts; ++j) {
        const int i = pts[4 * j + 0], c = pts[4 * j + 1], x = pts[4 * j + 2], y = pts[4 * j + 3];
        double acc = 0.0;
        for (int k = 0; k < K; ++k)
            for (int u = 0; u < R; ++u)
                for (int v = 0; v < S; ++v) {
                    const int xs = x + pad - u, ys = y + pad - v;
                    if (xs < 0 || ys < 0 || xs % stride || ys % stride) continue;
                    const int xo = xs / stride, yo = ys / stride;
                    if (xo < Ho && yo < Wo)
                        acc += (double)E[(((size_t)i * K + k) * Ho + xo) * Wo + yo] *
                               (double)G[(((size_t)k * C + c) * R + u) * S + v];
                }
        out[j] = acc;
    }
}

/* Gradient of Eq. (1) with respect to the filters (Section 4.2, second paragraph: a convolution of
 * the layer inputs with the backpropagated errors, R x S outputs per filter and channel).  From
 * Eq. (1): Y[i][k][x][y] contains D[i][c][x*stride+u-pad][y*stride+v-pad] * G[k][c][u][v], so
 *   dG[k][c][u][v] = sum_i sum_x sum_y D[i][c][x*stride+u-pad][y*stride+v-pad] * E[i][k][x][y]
 * with out-of-image taps contributing zero.  Inputs widened to double by the caller. */
void oracle_conv2d_bwd_filter_f64(int N, int C, int H, int W, int K, int R, int S, int pad, int stride,
                                  const double *D, const double *E, double *dG)
{
    const int Ho = out_extent(H, pad, R, stride), Wo = out_extent(W, pad, S, stride);
    #pragma omp parallel for collapse(2) schedule(static)
    for (int k = 0; k < K; ++k)
        for (int c = 0; c < C; ++c)
            for (int u = 0; u < R; ++u)
                for (int v = 0; v < S; ++v) {
                    double acc = 0.0;
                    for (int i = 0; i < N; ++i)
                        for (int x = 0; x < Ho; ++x)
                            for (int y = 0; y < Wo; ++y) {
                                const int xx = x * stride + u - pad, yy = y * stride + v - pad;
                                if (xx >= 0 && xx < H && yy >= 0 && yy < W)
                                    acc += D[(((size_t)i * C + c) * H + xx) * W + yy] *
                                           E[(((size_t)i * K + k) * Ho + x) * Wo + y];
                            }
                    dG[(((size_t)k * C + c) * R + u) * S + v] = acc;
                }
}

/* Selected elements of the filter gradient above on float inputs widened exactly to double:
 * pts[j] = (k, c, u, v).  Same sum as oracle_conv2d_bwd_filter_f64, one element at a time. */
void oracle_conv2d_bwd_filter_points_f32in(int N, int C, int H, int W, int K, int R, int S, int pad, int stride,
                                           const float *D, const float *E, long npts, const int32_t *pts,
                                           double *out)
{
    const int Ho = out_extent(H, pad, R, stride), Wo = out_extent(W, pad, S, stride);
    #pragma omp parallel for schedule(dynamic, 1)
    for (long j = 0; j < npts; ++j) {
        const int k = pts[4 * j + 0], c = pts[4 * j + 1], u = pts[4 * j + 2], v = pts[4 * j + 3];
        double acc = 0.0;
        for (int i = 0; i < N; ++i)
            for (int x = 0; x < Ho; ++x) {
                const int xx = x * stride + u - pad;
                if (xx < 0 || xx >= H) continue;
                for (int y = 0; y < Wo; ++y) {
                    const int yy = y * stride + v - pad;
                    if (yy >= 0 && yy < W)
                        acc += (double)D[(((size_t)i * C + c) * H + xx) * W + yy] *
                               (double)E[(((size_t)i * K + k) * Ho + x) * Wo + y];
                }
            }
        out[j] = acc;
    }
}

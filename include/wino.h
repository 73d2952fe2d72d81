/*
 * wino.h -- C ABI of the MI355X (gfx950) Winograd minimal-filtering convolution library.
 *
 * The library computes the forward pass of a convnet layer (Lavin & Gray, "Fast Algorithms
 * for Convolutional Neural Networks", Section 3, Eq. (1)):
 *
 *     Y[i][k][x][y] = sum_c sum_u sum_v D[i][c][x+u-pad][y+v-pad] * G[k][c][u][v]
 *
 * (2-D correlation, no filter flip, zeros outside the image) for 3x3 filters at stride 1 with
 * the algorithm F(m x m, 3 x 3) of Section 4, m = 2 (Eq. (7), (8)), m = 4 (Eq. (15)) or m = 6
 * (Section 4.3 mentions F(6 x 6, 3 x 3) without printing its matrices; here: interpolation
 * points 0, +-1, +-2, +-1/2, infinity; fp32 storage only), in the four stages of Algorithm 1,
 * plus a direct evaluation of Eq. (1) for layers the fast algorithm does not cover.
 *
 * Conventions for every entry point
 *   - D, G, U, V, M, Y and workspaces are DEVICE pointers owned by the caller; the library
 *     never frees or keeps them.  Bases must be 16-byte aligned.
 *   - Dense layouts: D[N][C][H][W], G[K][C][3][3], Y[N][K][Ho][Wo], Ho = H + 2*pad - 2.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work on it; they never synchronise the device.
 *   - Return value: a wino_status_t.  No exceptions, no abort.  Arguments are checked before
 *     any GPU call, so bad arguments are reported even on a machine with no GPU.
 *   - Storage type `dt` is that of D, G, U and V; products are always accumulated in fp32 and
 *     M is always fp32.
 *
 * Transform-domain layouts (alpha = m + 2; component index e = xi*alpha + nu; all row-major):
 *     fp32:  U[e][c][k]          extents [alpha^2][Cp][Kp]
 *            V[e][c][b]          extents [alpha^2][Cp][Pp]
 *     fp16:  U[e][c/8][k][c%8]   extents [alpha^2][Cp/8][Kp][8]
 *            V[e][c/8][b][c%8]   extents [alpha^2][Cp/8][Pp][8]
 *     M[e][k][b]                 extents [alpha^2][Kp][Pp], fp32
 * with the padded extents reported by wino_padded_dims(); padding elements of U and V are
 * written as zeros by the transforms, padding elements of M are unspecified.  A tile index b
 * stands for (image i, tile row tx, tile column ty) as b = (i*Th + tx)*Tw + ty, Th =
 * ceil(Ho/m), Tw = ceil(Wo/m); its input origin is (m*tx - pad, m*ty - pad) (Section 4.1's
 * tiling with overlap r-1 = 2; the collapse of (i, x~, y~) to b is Eq. (12)).
 */
#ifndef WINO_H_
#define WINO_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    WINO_OK = 0,
    WINO_EINVAL = 1,       /* null / misaligned pointer, non-positive extent, bad enum */
    WINO_EUNSUPPORTED = 2, /* m not in {2,4,6} (6: fp32 only), pad not in {0,1}, empty output, unsupported dtype */
    WINO_EWORKSPACE = 3,   /* workspace smaller than wino_workspace_bytes() */
    WINO_EHIP = 4          /* a HIP call failed; see wino_last_hip_error() */
} wino_status_t;

typedef enum { WINO_F32 = 0, WINO_F16 = 1 } wino_dtype_t;

/* Variant selection for wino_conv2d_fwd_ex (`flags`). 0 lets the library choose. */
#define WINO_FLAG_AUTO 0u
#define WINO_FLAG_UNFUSED 1u      /* four separate stages exactly as in Algorithm 1 */
#define WINO_FLAG_FUSED 2u        /* loops 2-4 of Algorithm 1 in one kernel: V and M never reach memory
                                   * (F(4x4,3x3); fp32 storage writes fp32 Y; fp16 storage needs pad 1 and
                                   * W % 4 == 0 and writes fp32 or fp16 Y; WINO_EUNSUPPORTED otherwise) */
#define WINO_FLAG_ONE_LAUNCH 3u   /* all four loops of Algorithm 1 in ONE kernel launch, the filter transform
                                   * computed inside the kernel (the variant of Section 6 without separately
                                   * transformed filters): F(2x2,3x3), fp32 D, G and Y, untransformed filters G
                                   * (U must be NULL); WINO_EUNSUPPORTED otherwise.  Meant for small batches.
                                   * When the layer has few output blocks the channel sum is shared between
                                   * workgroups, which meet through arrival counters held inside the library
                                   * and partial outputs in the workspace.  Each of the first 8 streams that
                                   * make such a call has counters of its own, so calls on different streams
                                   * may overlap (with different workspaces); calls from further streams run
                                   * the channel sum unshared (same result, fewer workgroups).  The result
                                   * does not depend on the order in which workgroups finish. */

const char *wino_status_string(int status);
/* hipError_t of the most recent failing HIP call made by the calling thread (0 if none). */
int wino_last_hip_error(void);

/* ---- host-side integer bookkeeping (no GPU involved) ------------------------------------ */

/* Number of tiles P = N * ceil(Ho/m) * ceil(Wo/m) (Algorithm 1, first line); -1 on bad input. */
long long wino_num_tiles(int N, int H, int W, int pad, int m);
/* out[0..4] = image i, tile row tx, tile column ty, input row m*tx-pad, input column m*ty-pad
 * of tile b. */
int wino_tile_coords(int N, int H, int W, int pad, int m, long long b, int out[5]);
/* Padded extents used by the transform-domain layouts above. P may be 0 when only Kp, Cp are
 * wanted (then *Pp = 0). Any output pointer may be NULL. */
int wino_padded_dims(int K, int C, long long P, int m, int dt, int *Kp, int *Cp, long long *Pp);
/* Element offsets (in units of the element type) into U, V and M; -1 on bad input. */
long long wino_u_offset(int K, int C, int m, int dt, int xi, int nu, int k, int c);
long long wino_v_offset(int C, long long P, int m, int dt, int xi, int nu, int c, long long b);
long long wino_m_offset(int K, long long P, int m, int xi, int nu, int k, long long b);

/* Buffer sizes in bytes (0 on bad input). */
size_t wino_filter_bytes(int K, int C, int m, int dt);           /* U */
size_t wino_v_bytes(int C, long long P, int m, int dt);          /* V */
size_t wino_m_bytes(int K, long long P, int m);                  /* M */
/* Workspace wino_conv2d_fwd_ex needs: room for U, V and M of this problem (M several times over
 * when the library splits the channel reduction of a small problem across workgroups).  The
 * one-kernel paths keep only U there; the fp32 one may use the part behind U (up to 32 MiB of it, where
 * V and M leave that much) for partial outputs and arrival counters of workgroups that share an
 * item, so calls that overlap on one GPU need workspaces of their own. */
size_t wino_workspace_bytes(int N, int C, int H, int W, int K, int pad, int m, int dt);

/* ---- the four stages of Algorithm 1, one entry point each ------------------------------- */

/* Loop 1: u = G g G^T for every (k, c), scattered to U (Algorithm 1; the "FX" external filter
 * transform of Section 6).  fp32 G -> fp32 U. */
int wino_filter_transform(int K, int C, int m, const void *G, void *U, void *stream);
/* Same with a storage type: G and U both of type dt; arithmetic in fp32, one rounding to dt. */
int wino_filter_transform_ex(int K, int C, int m, int dt, const void *G, void *U, void *stream);
/* Loop 2: gather tile d_{c,b} (zeros outside the image), v = B^T d B, scatter to V. */
int wino_input_transform(int N, int C, int H, int W, int pad, int m, int dt, const void *D, void *V,
                         void *stream);
/* Loop 3: M^(xi,nu) = U^(xi,nu) V^(xi,nu) for all alpha^2 components (Eq. (13)). */
int wino_batched_gemm(int K, int C, long long P, int m, int dt, const void *U, const void *V, void *M,
                      void *stream);
/* Host-side query: the launch shape of loop 3 inside the whole-layer entry points for these extents:
 * out[0] x out[1] = filters x tiles of M one workgroup computes, out[2] = number of shares the channel sum
 * is split into (their partial M's are added by loop 4; wino_batched_gemm itself never splits). */
int wino_gemm_launch_shape(int K, int C, long long P, int m, int dt, int out[3]);
/* Loop 4: gather m_{k,b} from M, Y_{k,b} = A^T m A, write the outputs that fall inside
 * Ho x Wo.  y_dt is the storage type of Y. */
int wino_output_transform(int N, int K, int H, int W, int pad, int m, int y_dt, const void *M, void *Y,
                          void *stream);

/* ---- whole layer ------------------------------------------------------------------------ */

/* fp32 layer with F(m x m, 3 x 3): all four loops of Algorithm 1.  Uses a workspace the
 * library allocates on first use (hipMalloc: not for callers under stream capture) and replaces by
 * a larger one when needed; one workspace per (device, stream), so calls on different streams may
 * overlap.  Never waits for the device: a replaced workspace is kept until wino_shutdown(), which
 * releases all of them. */
int wino_conv2d_fwd(int N, int C, int H, int W, int K, int pad, int m, const void *D, const void *G, void *Y,
                    void *stream);
/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): wino_conv2d_fwd with the workspace in a buffer that is part of the
 * library's image on every GPU (WINO_STATIC_WORKSPACE_BYTES, held from load to exit).  Calls no hipMalloc,
 * hipFree or other allocating routine.  Same arguments, same kernels and same results as wino_conv2d_fwd.
 * A layer that needs more (wino_workspace_bytes(N, C, H, W, K, pad, m, WINO_F32) >
 * WINO_STATIC_WORKSPACE_BYTES) is rejected with WINO_EWORKSPACE before any GPU call; the limit holds e.g.
 * every layer of the VGG stack at batch 1 with F(4x4,3x3).  All calls on one GPU share the one buffer, which
 * keeps the last call's contents (nothing in it needs clearing between calls): calls that may overlap on one
 * GPU -- different streams without an event between them -- race; calls on one stream never do.  The first
 * call on a GPU looks the buffer's address up (hipGetSymbolAddress), so make it outside stream capture. */
#define WINO_STATIC_WORKSPACE_BYTES (64u << 20)
int wino_conv2d_fwd_noalloc(int N, int C, int H, int W, int K, int pad, int m, const void *D, const void *G,
                            void *Y, void *stream);
/* General form.  U may be NULL (then G is transformed into the workspace first) or the output
 * of wino_filter_transform_ex for the same (K, C, m, dt) (then G may be NULL).  Never
 * allocates.  `workspace` must hold wino_workspace_bytes() bytes; its contents on entry do not
 * matter and are unspecified on return. */
int wino_conv2d_fwd_ex(int N, int C, int H, int W, int K, int pad, int m, int dt, int y_dt, const void *D,
                       const void *G, const void *U, void *Y, void *workspace, size_t workspace_bytes,
                       unsigned flags, void *stream);
/* ---- gradient with respect to the input (Section 4.2 of the paper) --------------------------
 * dD[i][c][x][y] = sum_k sum_u sum_v E[i][k][x+pad-u][y+pad-v] * G[k][c][u][v]: the forward algorithm
 * applied to the error tensor E[N][K][H][W] with every filter rotated by 180 degrees and K, C
 * exchanged.  Only pad = 1 (then E has the extent of D); other pads give WINO_EUNSUPPORTED. */

/* G[K][C][3][3] -> U' for the exchanged layer: the layout is that of a forward U with C filters
 * and K channels (sizes and offsets from wino_filter_bytes(C, K, ...), wino_u_offset(C, K, ...)). */
int wino_filter_transform_bwd(int K, int C, int m, int dt, const void *G, void *U, void *stream);
/* E[N][K][H][W] (type dt), G[K][C][3][3] (type dt) or its wino_filter_transform_bwd output U (then
 * G may be NULL) -> dD[N][C][H][W] (type d_dt).  Workspace: wino_workspace_bytes(N, K, H, W, C, 1, m, dt)
 * (the forward query with K and C exchanged).  `flags` as for wino_conv2d_fwd_ex. */
int wino_conv2d_bwd_data(int N, int C, int H, int W, int K, int pad, int m, int dt, int d_dt, const void *E,
                         const void *G, const void *U, void *dD, void *workspace, size_t workspace_bytes,
                         unsigned flags, void *stream);

/* ---- gradient with respect to the filters (Section 4.2, Eq. (14): F(3x3, 2x2)) ---------------
 * dG[k][c][u][v] = sum_i sum_x sum_y D[i][c][x+u-pad][y+v-pad] * E[i][k][x][y].  The error tensor is
 * cut into 2 x 2 blocks, each paired with the 4 x 4 input tile around it (tiles overlap by 2);
 * w = G e G^T, v = B^T d B, M = sum over blocks and images of w . v, dG = A^T M A.
 * fp32 only, pad = 1, stride 1 (else WINO_EUNSUPPORTED). */
size_t wino_bwd_filter_workspace_bytes(int N, int C, int H, int W, int K);   /* 0 on bad input */
/* D[N][C][H][W], E[N][K][H][W] -> dG[K][C][3][3]; overwrites dG; never allocates. */
int wino_conv2d_bwd_filter(int N, int C, int H, int W, int K, int pad, int dt, const void *D, const void *E, void *dG,
                           void *workspace, size_t workspace_bytes, void *stream);

/* Host-side query: the variant wino_conv2d_fwd_ex runs for these arguments -- WINO_FLAG_UNFUSED,
 * WINO_FLAG_FUSED or WINO_FLAG_ONE_LAUNCH -- when called with `flags` (WINO_FLAG_AUTO resolves to one of
 * the first two; WINO_FLAG_ONE_LAUNCH is answered for untransformed filters, G given); a negative
 * wino_status_t (e.g. -WINO_EUNSUPPORTED) if the call would be rejected. */
int wino_conv2d_variant(int N, int C, int H, int W, int K, int pad, int m, int dt, int y_dt, unsigned flags);
/* Host-side query: how the one-kernel fp32 F(4x4,3x3) layer (64 filters x 16 tiles per item, Section 6's
 * fusion of the transforms into the multiply) deals its items to the GPU's 8 XCDs when the workspace has room for
 * partial outputs (m = 4 or 2).  out[4 x + 0..3] for XCD x: number of items, how many of them run in rounds that
 * occupy all resident workgroups of the XCD (64 for m = 4, 96 for m = 2), how many are left for the last round,
 * and the number of shares each of those is cut into (1: none; shares x items of the last round <= the resident
 * workgroups, and the shares divide the item's channel steps of 16 channels).  Returns the number of workgroups
 * of the launch, or a negative wino_status_t (-WINO_EUNSUPPORTED where that kernel does not apply). */
int wino_one_kernel_plan(int N, int C, int H, int W, int K, int pad, int m, int dt, int out[32]);
/* Eq. (1) evaluated directly on the GPU: any R x S filter, stride and padding; for layers the
 * fast algorithm does not cover (e.g. the 3-channel first layer of Table 3).
 * D[N][C][H][W], G[K][C][R][S] -> Y[N][K][Ho][Wo] with Ho = (H + 2 pad - R) / stride + 1 (Wo alike); D, G and Y
 * are device pointers of element type `dt` (fp32, or fp16 with fp32 accumulation), caller-owned; Y is
 * overwritten.  Asynchronous on `stream`, never allocates.  3 x 3, stride 1 layers with at most 4 channels and
 * W % 4 == 0 run on the matrix units, everything else on the vector ALUs.
 * WINO_EINVAL for null pointers or non-positive extents, WINO_EUNSUPPORTED for an empty output or extents
 * beyond the launch limits (N or K / 16 above 65535, R S above 512). */
int direct_conv2d_fwd(int N, int C, int H, int W, int K, int R, int S, int pad, int stride, int dt,
                      const void *D, const void *G, void *Y, void *stream);

/* Frees the cached workspaces of wino_conv2d_fwd (synchronises the device first). */
int wino_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* WINO_H_ */

// Internal declarations shared by the kernels and the C-ABI layer of libwino (gfx950 only).
#pragma once
#include <stdlib.h>
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/wino.h"

namespace wino {


// Problem geometry and the padded extents of the transform-domain buffers.
struct Geo {
    int m, alpha, a2;      // output tile, input tile (m + 2), number of components alpha^2
    int N, C, H, W, K, pad;
    int Ho, Wo, Th, Tw;    // output extent and tiles per image
    int P;                 // number of tiles N*Th*Tw
    int Kp, Cp, Pp;        // padded extents of U, V, M
    int dt;                // storage type of D, G, U, V
};

inline int round_up(long long x, int q) { return (int)(((x + q - 1) / q) * q); }

// Padding rules: K to the MFMA tile edge, C to the reduction chunk, P to the MFMA tile edge.
inline int pad_k(int K) { return round_up(K, 32); }
inline int pad_c(int C, int dt) { return round_up(C, dt == WINO_F16 ? 32 : 16); }
inline int pad_p(long long P) { return round_up(P, 32); }

// Kernel launchers (each enqueues on `s` and returns the launch status).
// `zero1024` (fp32 only, may be null): 1024 words the first block sets to zero for the kernel that follows
hipError_t launch_filter_transform(const Geo &g, const void *G, void *U, hipStream_t s, unsigned int *zero1024 = nullptr);
hipError_t launch_filter_transform_bwd(const Geo &g, const void *G, void *U, hipStream_t s,
                                       unsigned int *zero1024 = nullptr);
hipError_t launch_input_transform(const Geo &g, const void *D, void *V, hipStream_t s);
int gemm_splits(const Geo &g);
void gemm_launch_shape(const Geo &g, int *bm, int *bn, int *splits);
hipError_t launch_batched_gemm(const Geo &g, const void *U, const void *V, float *M, int splits, hipStream_t s);
hipError_t launch_output_transform(const Geo &g, int y_dt, const float *M, void *Y, int splits, hipStream_t s);
bool fused_eligible(const Geo &g);
bool fused_preferred(const Geo &g);
hipError_t launch_fused(const Geo &g, const void *D, const void *U, void *Y, int y_dt, hipStream_t s);
bool fused_f16_eligible(const Geo &g);
bool fused_lds_eligible(const Geo &g);
hipError_t launch_fused_lds(const Geo &g, const float *D, const float *U, float *Y, hipStream_t s);
bool fused_wide_eligible(const Geo &g);
// `part`: room for arrival counters and partial outputs (fused_wide_part_bytes(g), 256-byte aligned), or null;
// `cleared`: the counters (the first 512 words of `part`) have been set to zero by a kernel in front on the stream.
// fused_wide_shares: whether the launch will use `part` at all.
hipError_t launch_fused_wide(const Geo &g, const float *D, const float *U, float *Y, void *part, size_t part_bytes,
                             bool cleared, hipStream_t s);
bool fused_wide_shares(const Geo &g, const void *part, size_t part_bytes);
int fused_wide_plan(const Geo &g, int out[32]);      // per XCD: items, in full rounds, in the last round, shares; returns the grid
size_t fused_wide_part_bytes(const Geo &g);
double fused_wide_fill(const Geo &g);      // 0 .. 1: how well the launch fills its rounds of resident workgroups
hipError_t launch_fused_f16(const Geo &g, const void *D, const void *U, void *Y, int y_dt, hipStream_t s);
bool fused_f2_eligible(const Geo &g);
hipError_t launch_fused_f2(const Geo &g, const float *D, const float *G, float *Y, void *workspace,
                           size_t workspace_bytes, bool bwd, hipStream_t s);
bool prep_eligible(const Geo &g);
hipError_t launch_prep(const Geo &g, const void *G, void *U, const void *D, void *V, hipStream_t s);
bool wgrad_supported(long long N, long long C, long long H, long long W, long long K);
size_t wgrad_workspace_bytes(int N, int C, int H, int W, int K);
hipError_t launch_wgrad(int N, int C, int H, int W, int K, const float *D, const float *E, float *dG, void *workspace,
                        hipStream_t s);
hipError_t launch_direct_conv(int N, int C, int H, int W, int K, int R, int S, int pad, int stride, int dt,
                              const void *D, const void *G, void *Y, hipStream_t s);

}  // namespace wino

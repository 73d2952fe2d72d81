// Loops 1 and 2 of Algorithm 1 (Lavin & Gray) in one launch.  The filter transform and the input
// transform do not depend on each other, and for small batches each is far too small to fill the
// GPU, so a layer that has to do both pays one kernel's start-up and drain instead of two: the
// first blocks of the grid transform filters, the rest transform input tiles.
#include <stdlib.h>

#include "stage_bodies.h"

namespace wino {

// IT: 0 = one tile per thread, 1 = the same with 16-byte row loads, 2 = two tiles per thread
template <int M, int IT>
__global__ __launch_bounds__(256) void prep_kernel(const float *__restrict__ G, float *__restrict__ U,
                                                   const float *__restrict__ D, float *__restrict__ V, Geo g,
                                                   int ft_gx, int ft_blocks, int it_gx)
{
    __shared__ float gs[FT_LDS];
    const int id = blockIdx.x;
    if (id < ft_blocks) {
        filter_transform_block<M, float>(G, U, g.K, g.C, g.Kp, g.Cp, id % ft_gx, id / ft_gx, gs);
        return;
    }
    const int j = id - ft_blocks;
    if constexpr (IT == 2)
        input_transform_pair_block<M>(D, V, g, j % it_gx, j / it_gx);
    else
        input_transform_block<M, float, IT == 1>(D, V, g, j % it_gx, j / it_gx);
}

// fp16 storage: 512 threads, both bodies collect their results in the same LDS bytes
template <int M, bool VEC>
__global__ __launch_bounds__(512) void prep_f16_kernel(const __half *__restrict__ G, __half *__restrict__ U,
                                                       const __half *__restrict__ D, __half *__restrict__ V, Geo g,
                                                       int ft_gx, int ft_blocks, int it_gx)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[f16_stage_bytes(M)];
    const int id = blockIdx.x;
    if (id < ft_blocks) {
        filter_transform_f16_block<M, 512>(G, U, g.K, g.C, g.Kp, g.Cp, id % ft_gx, id / ft_gx, smem);
        return;
    }
    const int j = id - ft_blocks;
    input_transform_f16_block<M, VEC>(D, V, g, j % it_gx, j / it_gx, smem);
}

bool prep_eligible(const Geo &g) { return g.dt == WINO_F32 || g.dt == WINO_F16; }

static hipError_t launch_prep_f16(const Geo &g, const __half *G, __half *U, const __half *D, __half *V, hipStream_t s)
{
    const int ft_gx = (g.Kp + F16_KT - 1) / F16_KT, it_gx = (g.Pp + F16_TB - 1) / F16_TB;
    const long long ft_blocks = (long long)ft_gx * (g.Cp / 8);
    const long long blocks = ft_blocks + (long long)it_gx * (g.Cp / 8);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(512);
    const int fb = (int)ft_blocks;
    if (g.m == 2)
        prep_f16_kernel<2, false><<<grid, block, 0, s>>>(G, U, D, V, g, ft_gx, fb, it_gx);
    else if (g.pad == 1 && g.W % 4 == 0)
        prep_f16_kernel<4, true><<<grid, block, 0, s>>>(G, U, D, V, g, ft_gx, fb, it_gx);
    else
        prep_f16_kernel<4, false><<<grid, block, 0, s>>>(G, U, D, V, g, ft_gx, fb, it_gx);
    return hipGetLastError();
}

hipError_t launch_prep(const Geo &g, const void *Gv, void *Uv, const void *Dv, void *Vv, hipStream_t s)
{
    if (g.dt == WINO_F16)
        return launch_prep_f16(g, (const __half *)Gv, (__half *)Uv, (const __half *)Dv, (__half *)Vv, s);
    const float *G = (const float *)Gv, *D = (const float *)Dv;
    float *U = (float *)Uv, *V = (float *)Vv;
    const int ft_gx = (g.Kp + FT_KT - 1) / FT_KT, ft_gy = (g.Cp + FT_CT - 1) / FT_CT;
    const long long ft_blocks = (long long)ft_gx * ft_gy;
    int it = 0;
    if (g.m == 4 && g.pad == 1 && g.W % 8 == 0) it = 2;
    else if (g.m == 4 && g.pad == 1 && g.W % 4 == 0) it = 1;
    const int it_gx = it == 2 ? (g.Pp / 2 + 255) / 256 : (g.Pp + 255) / 256;
    const long long blocks = ft_blocks + (long long)it_gx * g.Cp;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(256);
    const int fb = (int)ft_blocks;
    if (g.m == 2)
        prep_kernel<2, 0><<<grid, block, 0, s>>>(G, U, D, V, g, ft_gx, fb, it_gx);
    else if (g.m == 6)
        prep_kernel<6, 0><<<grid, block, 0, s>>>(G, U, D, V, g, ft_gx, fb, it_gx);
    else if (it == 2)
        prep_kernel<4, 2><<<grid, block, 0, s>>>(G, U, D, V, g, ft_gx, fb, it_gx);
    else if (it == 1)
        prep_kernel<4, 1><<<grid, block, 0, s>>>(G, U, D, V, g, ft_gx, fb, it_gx);
    else
        prep_kernel<4, 0><<<grid, block, 0, s>>>(G, U, D, V, g, ft_gx, fb, it_gx);
    return hipGetLastError();
}

}  // namespace wino

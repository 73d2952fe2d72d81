// Loop 2 of Algorithm 1 (Lavin & Gray): gather each alpha x alpha input tile d_{c,b} (tiles
// overlap by r-1 = 2, zeros outside the image -- the implicit zero padding of Section 6),
// v = B^T d B (Eq. (8)), scatter to the alpha^2 matrices V^(xi,nu)[c][b].
// Bound by memory traffic: every input element is needed once, alpha^2/m^2 values are written
// per input element.
#include <stdlib.h>

#include "wino_internal.h"
#include "stage_bodies.h"

namespace wino {

template <int M, typename T, bool VEC = false>
__global__ __launch_bounds__(256) void input_transform_kernel(const T *__restrict__ D, T *__restrict__ V, Geo g)
{
    input_transform_block<M, T, VEC>(D, V, g, blockIdx.x, blockIdx.y);
}

template <int M>
__global__ __launch_bounds__(256) void input_transform_pair_kernel(const float *__restrict__ D, float *__restrict__ V,
                                                                   Geo g)
{
    input_transform_pair_block<M>(D, V, g, blockIdx.x, blockIdx.y);
}

// fp16 storage: see input_transform_f16_block.
template <int M, bool VEC>
__global__ __launch_bounds__(512) void input_transform_f16_kernel(const __half *__restrict__ D,
                                                                   __half *__restrict__ V, Geo g)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[f16_stage_bytes(M)];
    input_transform_f16_block<M, VEC>(D, V, g, blockIdx.x, blockIdx.y, smem);
}

hipError_t launch_input_transform(const Geo &g, const void *D, void *V, hipStream_t s)
{
    dim3 grid((g.Pp + 255) / 256, g.Cp), block(256);
    if (g.dt == WINO_F32 && g.m == 4 && g.pad == 1 && g.W % 8 == 0) {
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

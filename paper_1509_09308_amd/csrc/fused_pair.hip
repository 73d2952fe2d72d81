// Loops 2-4 of Algorithm 1 (Lavin & Gray) in one kernel, fp32 F(4x4,3x3), second design: small
// workgroups that alternate transform and multiply phases, two per CU so that one multiplies while
// the other transforms, waits for memory or stores (on this chip MFMA and ordinary vector
// instructions of one SIMD do not overlap, so what a second workgroup can fill is the waiting).
//
// Workgroup = 4 wavefronts owning 32 filters x 32 tiles x 36 components (144 accumulators per lane).
// Per step of 8 channels:
//   1. transform phase: every thread gathers the 6 x 6 tile of one (tile, channel) pair (per row one
//      aligned 16-byte load and the two outer columns from clamped addresses, masked afterwards),
//      computes v = B^T (d B) and writes the 36 values to LDS as [e][c / 2][tile][c % 2]; the
//      step's transformed filters, stored by the filter transform in the same pair order
//      [e][c / 2][k][c % 2], arrive by direct global -> LDS loads (16 bytes per lane, no registers)
//      requested right after the previous multiply phase;
//   2. multiply phase: wavefront cg owns components 9 cg .. 9 cg + 8; lane (i, h) reads channels
//      4j + 2h, 4j + 2h + 1 of its filter row and of its tile column with one 8-byte read each
//      (conflict-free) and feeds two v_mfma_f32_32x32x2_f32.
// After the last step the accumulators go through LDS in four pieces of 8 filters; every thread
// gathers the 36 components of one (filter, tile) pair, applies Y = A^T m A and writes the rows
// of its 4 x 4 outputs that are inside the image as 16-byte stores.
// Needs pad = 1 and W % 4 == 0; filters transformed by filter_transform_pair_kernel.
#include "stage_bodies.h"

namespace wino {

typedef float floatx16_p __attribute__((ext_vector_type(16)));
typedef float floatx4_p __attribute__((ext_vector_type(4)));
typedef float floatx2_p __attribute__((ext_vector_type(2)));

constexpr int FB_K = 32, FB_P = 32, FB_C = 8, FB_T = 256;           // filters, tiles, channels per step, threads
constexpr int FB_U_WORDS = 36 * (FB_C / 2) * FB_K * 2 / 4;          // 16-byte words of U per step (2304)
constexpr int FB_V_FLOATS = 36 * (FB_C / 2) * FB_P * 2;             // floats of V per step (9216)
constexpr int FB_M_FLOATS = 36 * 8 * FB_P;                          // one piece of M in the epilogue
static_assert(FB_U_WORDS % (64 * 4) == 0, "every wavefront copies the same number of 64-word chunks");
static_assert(FB_M_FLOATS <= FB_U_WORDS * 4 + FB_V_FLOATS, "the epilogue reuses the operand area");

#define WINO_P_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define WINO_P_GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

// u = G g G^T written in the pair order the kernel below copies: U2[e][c / 2][k][c % 2].  K, C, Kp, Cp
// describe the layer the kernel computes.  BWD: that layer is the input gradient (Section 4.2 of the
// paper): its filter (k, c) is filter (c, k) of the stored G[C][K][3][3], rotated by 180 degrees.
template <int M, bool BWD>
__global__ __launch_bounds__(256) void filter_transform_pair_kernel(const float *__restrict__ G, float *__restrict__ U2,
                                                                    int K, int C, int Kp, int Cp)
{
    constexpr int A = M + 2;
    const int k = blockIdx.x * 64 + (threadIdx.x & 63);
    const int c = blockIdx.y * 4 + (threadIdx.x >> 6);
    if (k >= Kp || c >= Cp) return;
    float g[3][3], t[A][3], u[A][A];
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            float v = 0.0f;
            if (k < K && c < C)
                v = BWD ? G[((size_t)c * K + k) * 9 + (2 - i) * 3 + (2 - j)] : G[((size_t)k * C + c) * 9 + i * 3 + j];
            g[i][j] = v;
        }
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        float col[3] = {g[0][j], g[1][j], g[2][j]}, o[A];
        g_mul<M>(col, o);
#pragma unroll
        for (int i = 0; i < A; ++i) t[i][j] = o[i];
    }
#pragma unroll
    for (int i = 0; i < A; ++i) g_mul<M>(t[i], u[i]);
#pragma unroll
    for (int xi = 0; xi < A; ++xi)
#pragma unroll
        for (int nu = 0; nu < A; ++nu)
            U2[(((size_t)(xi * A + nu) * (Cp / 2) + c / 2) * Kp + k) * 2 + (c & 1)] = u[xi][nu];
}

__device__ __forceinline__ int xcd_group_p(int bid, int nblocks)
{
    // workgroups are dealt to the 8 XCDs round-robin; make logically consecutive blocks (which share
    // input tiles) share an XCD and its L2
    const int per = nblocks / 8;
    if (bid >= per * 8) return bid;
    return (bid % 8) * per + bid / 8;
}

__global__ __launch_bounds__(FB_T, 2) void fused_pair_kernel(const float *__restrict__ D, const uint4 *__restrict__ U2,
                                                             float *__restrict__ Y, Geo g, int n_kb)
{
    __shared__ uint4 smem[FB_U_WORDS + FB_V_FLOATS / 4];
    uint4 *Us = smem;
    float *Vs = reinterpret_cast<float *>(smem + FB_U_WORDS);

    const int bid = xcd_group_p(blockIdx.x, gridDim.x);
    const int kb = bid % n_kb, tb = bid / n_kb;
    const int k0 = kb * FB_K, b0 = tb * FB_P;
    const int tid = threadIdx.x;

    // ---- transform-phase role: (tile, channel of the step) ------------------------------------
    const int tl = tid & 31, cl = tid >> 5;
    const int b = b0 + tl;
    const bool tile_ok = b < g.P;
    int x0 = 0, y0 = 0, orow = 0;
    const float *src = D;
    float *ybase = Y;
    {
        const int bb = tile_ok ? b : 0;
        const int ty = bb % g.Tw;
        const int t2 = bb / g.Tw;
        const int tx = t2 % g.Th;
        const int i = t2 / g.Th;
        x0 = 4 * tx - 1;
        y0 = 4 * ty - 1;
        orow = 4 * tx;
        src = D + (size_t)i * g.C * g.H * g.W;
        ybase = Y + ((size_t)i * g.K * g.Ho + orow) * g.Wo + 4 * ty;
    }
    const size_t plane = (size_t)g.H * g.W;
    const bool okl = y0 >= 0, okr = y0 + 5 < g.W;

    // ---- multiply-phase role -------------------------------------------------------------------
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int cg = wave;
    const int li = lane & 31, lh = lane >> 5;
    floatx16_p acc[9];
#pragma unroll
    for (int e = 0; e < 9; ++e)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[e][r] = 0.0f;

    const int nsteps = g.Cp / FB_C;
    const int Cp2 = g.Cp / 2;

    // Transformed filters of a step: LDS word ((e * 4 + p) * 16 + kw) <- U2 word
    // ((e * Cp/2 + 4 * step + p) * Kp + k0) / 2 + kw; each wavefront copies 9 chunks of 64 words.
    constexpr int NCH = FB_U_WORDS / 256;
    unsigned uoff[NCH];
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        const int w = (wave + 4 * j) * 64 + lane;
        const int e = w / 64, p = (w / 16) & 3, kw = w & 15;
        uoff[j] = (unsigned)(((size_t)(e * Cp2 + p) * g.Kp + k0) / 2 + kw);
    }
    auto load_u = [&](int step) {
        const uint4 *ub = U2 + (size_t)step * 4 * g.Kp / 2;
#pragma unroll
        for (int j = 0; j < NCH; ++j)
            __builtin_amdgcn_global_load_lds(WINO_P_GLB_PTR(ub + uoff[j]), WINO_P_LDS_PTR(Us + (wave + 4 * j) * 64), 16, 0,
                                             0);
    };

    const float *As = reinterpret_cast<const float *>(Us);
    const int op_off = (lh * 32 + li) * 2;          // within one (e, j): pair 2j + lh, row/column li
    load_u(0);
    for (int step = 0; step < nsteps; ++step) {
        // 1. one input tile: gather, transform rows then columns (v = B^T (d B)), scatter
        {
            const int c = step * FB_C + cl;
            const bool ok = tile_ok && c < g.C;
            const float *pc = src + (size_t)min(c, g.C - 1) * plane;
            floatx4_p mid[6];
            float l[6], r[6];
#pragma unroll
            for (int p = 0; p < 6; ++p) {
                const float *row = pc + (size_t)min(max(x0 + p, 0), g.H - 1) * g.W + y0;
                mid[p] = *reinterpret_cast<const floatx4_p *>(row + 1);
                l[p] = row[okl ? 0 : 1];
                r[p] = row[okr ? 5 : 4];
            }
            float t[6][6];
#pragma unroll
            for (int p = 0; p < 6; ++p) {
                const int x = x0 + p;
                const bool rok = ok && x >= 0 && x < g.H;
                const float d[6] = {(rok && okl) ? l[p] : 0.0f, rok ? mid[p][0] : 0.0f, rok ? mid[p][1] : 0.0f,
                                    rok ? mid[p][2] : 0.0f, rok ? mid[p][3] : 0.0f, (rok && okr) ? r[p] : 0.0f};
                bt_mul<4>(d, t[p]);
            }
            float *dst = Vs + ((size_t)(cl >> 1) * FB_P + tl) * 2 + (cl & 1);
#pragma unroll
            for (int q = 0; q < 6; ++q) {
                const float col[6] = {t[0][q], t[1][q], t[2][q], t[3][q], t[4][q], t[5][q]};
                float o[6];
                bt_mul<4>(col, o);
#pragma unroll
                for (int p = 0; p < 6; ++p) dst[(size_t)(p * 6 + q) * (4 * FB_P * 2)] = o[p];
            }
        }
        __syncthreads();      // V written, the filters of this step have arrived (all loads are waited for)
        // 2. nine components x (32 filters x 32 tiles x 8 channels)
#pragma unroll
        for (int e = 0; e < 9; ++e) {
            const int eo = (cg * 9 + e) * (4 * 32 * 2) + op_off;
            floatx2_p a[2], bb[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                a[j] = *reinterpret_cast<const floatx2_p *>(As + eo + j * (2 * 32 * 2));
                bb[j] = *reinterpret_cast<const floatx2_p *>(Vs + eo + j * (2 * 32 * 2));
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                acc[e] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[j][0], bb[j][0], acc[e], 0, 0, 0);
                acc[e] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[j][1], bb[j][1], acc[e], 0, 0, 0);
            }
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);
        __builtin_amdgcn_s_barrier();
        if (step + 1 < nsteps) load_u(step + 1);
    }
    __syncthreads();

    // ---- inverse transform: four pieces of 8 filters -------------------------------------------
    float *Ms = reinterpret_cast<float *>(smem);
    const int frow = tid >> 5;                 // 0..7: filter row of the piece handled in the gather
    const int ot = tid & 31;                   // tile of the gather (same tile as in the transform phase)
    for (int q = 0; q < 4; ++q) {
        // accumulator register r of lane (li, lh) is filter 8 * (r / 4) + 4 * lh + r % 4, tile li
#pragma unroll
        for (int e = 0; e < 9; ++e)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) Ms[((cg * 9 + e) * 8 + 4 * lh + rr) * FB_P + li] = acc[e][4 * q + rr];
        __syncthreads();
        const int k = k0 + 8 * q + frow;
        if (tile_ok && k < g.K) {
            float m[6][6], tt[4][6], y[4][4];
#pragma unroll
            for (int xi = 0; xi < 6; ++xi)
#pragma unroll
                for (int nu = 0; nu < 6; ++nu) m[xi][nu] = Ms[((xi * 6 + nu) * 8 + frow) * FB_P + ot];
#pragma unroll
            for (int nu = 0; nu < 6; ++nu) {
                const float col[6] = {m[0][nu], m[1][nu], m[2][nu], m[3][nu], m[4][nu], m[5][nu]};
                float o[4];
                at_mul<4>(col, o);
#pragma unroll
                for (int p = 0; p < 4; ++p) tt[p][nu] = o[p];
            }
#pragma unroll
            for (int p = 0; p < 4; ++p) at_mul<4>(tt[p], y[p]);
            float *dst = ybase + (size_t)k * g.Ho * g.Wo;
#pragma unroll
            for (int p = 0; p < 4; ++p)
                if (orow + p < g.Ho)
                    *reinterpret_cast<floatx4_p *>(dst + (size_t)p * g.Wo) = floatx4_p{y[p][0], y[p][1], y[p][2], y[p][3]};
        }
        __syncthreads();
    }
}

bool fused_pair_eligible(const Geo &g)
{
    return g.dt == WINO_F32 && g.m == 4 && g.pad == 1 && g.W % 4 == 0 &&
           (size_t)36 * (g.Cp / 2) * g.Kp < (1ull << 31);   // 32-bit word offsets into U2
}

hipError_t launch_filter_transform_pair(const Geo &g, const float *G, float *U2, bool bwd, hipStream_t s)
{
    dim3 grid((g.Kp + 63) / 64, (g.Cp + 3) / 4), block(256);
    if (bwd)
        filter_transform_pair_kernel<4, true><<<grid, block, 0, s>>>(G, U2, g.K, g.C, g.Kp, g.Cp);
    else
        filter_transform_pair_kernel<4, false><<<grid, block, 0, s>>>(G, U2, g.K, g.C, g.Kp, g.Cp);
    return hipGetLastError();
}

hipError_t launch_fused_pair(const Geo &g, const float *D, const float *U2, float *Y, hipStream_t s)
{
    const int n_kb = g.Kp / FB_K;
    const long long blocks = (long long)((g.P + FB_P - 1) / FB_P) * n_kb;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    fused_pair_kernel<<<dim3((unsigned)blocks), dim3(FB_T), 0, s>>>(D, (const uint4 *)U2, Y, g, n_kb);
    return hipGetLastError();
}

}  // namespace wino

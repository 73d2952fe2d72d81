// The C ABI of libwino: argument checking, buffer-size and layout queries, stage entry
// points and the whole-layer drivers.  Declarations and contracts are in include/wino.h.
#include <mutex>
#include <vector>

#include <stdlib.h>

#include "wino_internal.h"

using namespace wino;

// Workspace of wino_conv2d_fwd_noalloc: part of the library's image on every GPU, so using it needs no
// allocation.  In host code the array's name is only a handle for hipGetSymbolAddress; kernels are given the
// device address that call returns (one per GPU, looked up once with that GPU current).
static __device__ __align__(256) unsigned char scratch[WINO_STATIC_WORKSPACE_BYTES];

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return WINO_EHIP;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool bad_ptr(const void *p) { return p == nullptr || !aligned16(p); }
bool bad_dtype(int dt) { return dt != WINO_F32 && dt != WINO_F16; }
size_t elem_size(int dt) { return dt == WINO_F16 ? 2 : 4; }
// F(2x2,3x3) and F(4x4,3x3) in both storage types; F(6x6,3x3) in fp32 only (its transformed values
// span too many binades for fp16 storage)
bool bad_m(int m, int dt) { return !(m == 2 || m == 4 || (m == 6 && dt == WINO_F32)); }

// Validates the geometry shared by every Winograd entry point and fills `g`.
// N, C, K may be passed as 1 by callers that do not use them.
int make_geo(int N, int C, int H, int W, int K, int pad, int m, int dt, Geo *g)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0) return WINO_EINVAL;
    if (bad_dtype(dt)) return WINO_EINVAL;
    if (bad_m(m, dt)) return WINO_EUNSUPPORTED;
    if (pad != 0 && pad != 1) return WINO_EUNSUPPORTED;
    const int Ho = H + 2 * pad - 2, Wo = W + 2 * pad - 2;
    if (Ho <= 0 || Wo <= 0) return WINO_EUNSUPPORTED;
    const int Th = (Ho + m - 1) / m, Tw = (Wo + m - 1) / m;
    const long long P = (long long)N * Th * Tw;
    // 32-bit tile and row indices inside the kernels; grid.y limits
    if (P > (1LL << 30) || C > 65000 || K > 65000) return WINO_EUNSUPPORTED;
    g->m = m; g->alpha = m + 2; g->a2 = (m + 2) * (m + 2);
    g->N = N; g->C = C; g->H = H; g->W = W; g->K = K; g->pad = pad;
    g->Ho = Ho; g->Wo = Wo; g->Th = Th; g->Tw = Tw; g->P = (int)P;
    g->Kp = pad_k(K); g->Cp = pad_c(C, dt); g->Pp = pad_p(P);
    g->dt = dt;
    return WINO_OK;
}

// Geometry for entry points that are given P instead of an image shape.
int make_geo_kcp(int K, int C, long long P, int m, int dt, Geo *g)
{
    if (K <= 0 || C <= 0 || P <= 0) return WINO_EINVAL;
    if (bad_dtype(dt)) return WINO_EINVAL;
    if (bad_m(m, dt)) return WINO_EUNSUPPORTED;
    if (P > (1LL << 30) || C > 65000 || K > 65000) return WINO_EUNSUPPORTED;
    *g = Geo{};
    g->m = m; g->alpha = m + 2; g->a2 = (m + 2) * (m + 2);
    g->C = C; g->K = K; g->P = (int)P;
    g->Kp = pad_k(K); g->Cp = pad_c(C, dt); g->Pp = pad_p(P);
    g->dt = dt;
    return WINO_OK;
}

size_t u_bytes(const Geo &g) { return (size_t)g.a2 * g.Cp * g.Kp * elem_size(g.dt); }
size_t v_bytes(const Geo &g) { return (size_t)g.a2 * g.Cp * g.Pp * elem_size(g.dt); }
size_t m_bytes(const Geo &g) { return (size_t)g.a2 * g.Kp * g.Pp * sizeof(float); }
size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Cached workspaces of the short-form entry point, one per (device, stream): work that uses a buffer is
// always queued on the stream the buffer belongs to, so calls on different streams never share one.
// A buffer that has become too small is not freed when a larger one replaces it (work queued earlier may
// still use it, and hipFree would wait for the device): it is kept until wino_shutdown().  Buffers grow by
// at least a factor of two, so the retired ones add up to less than the live one.
struct CachedWs {
    hipStream_t stream;
    int device;
    void *ptr;
    size_t bytes;
};
std::mutex g_ws_mutex;
std::vector<CachedWs> g_ws;
std::vector<void *> g_ws_retired;

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

}  // namespace

extern "C" {

const char *wino_status_string(int status)
{
    switch (status) {
    case WINO_OK: return "ok";
    case WINO_EINVAL: return "invalid argument";
    case WINO_EUNSUPPORTED: return "unsupported configuration";
    case WINO_EWORKSPACE: return "workspace too small";
    case WINO_EHIP: return "HIP call failed";
    default: return "unknown status";
    }
}

int wino_last_hip_error(void) { return g_last_hip_error; }

long long wino_num_tiles(int N, int H, int W, int pad, int m)
{
    Geo g;
    if (make_geo(N, 1, H, W, 1, pad, m, WINO_F32, &g) != WINO_OK) return -1;
    return g.P;
}

int wino_tile_coords(int N, int H, int W, int pad, int m, long long b, int out[5])
{
    Geo g;
    const int st = make_geo(N, 1, H, W, 1, pad, m, WINO_F32, &g);
    if (st != WINO_OK) return st;
    if (out == nullptr || b < 0 || b >= g.P) return WINO_EINVAL;
    const int ty = (int)(b % g.Tw);
    const int t2 = (int)(b / g.Tw);
    const int tx = t2 % g.Th;
    out[0] = t2 / g.Th;
    out[1] = tx;
    out[2] = ty;
    out[3] = m * tx - pad;
    out[4] = m * ty - pad;
    return WINO_OK;
}

int wino_padded_dims(int K, int C, long long P, int m, int dt, int *Kp, int *Cp, long long *Pp)
{
    if (K <= 0 || C <= 0 || P < 0 || bad_dtype(dt)) return WINO_EINVAL;
    if (bad_m(m, dt)) return WINO_EUNSUPPORTED;
    if (P > (1LL << 30)) return WINO_EUNSUPPORTED;
    if (Kp) *Kp = pad_k(K);
    if (Cp) *Cp = pad_c(C, dt);
    if (Pp) *Pp = pad_p(P);
    return WINO_OK;
}

long long wino_u_offset(int K, int C, int m, int dt, int xi, int nu, int k, int c)
{
    Geo g;
    if (make_geo_kcp(K, C, 1, m, dt, &g) != WINO_OK) return -1;
    if (xi < 0 || xi >= g.alpha || nu < 0 || nu >= g.alpha || k < 0 || k >= g.Kp || c < 0 || c >= g.Cp) return -1;
    const long long e = xi * g.alpha + nu;
    if (dt == WINO_F32) return (e * g.Cp + c) * g.Kp + k;
    return ((e * (g.Cp / 8) + c / 8) * g.Kp + k) * 8 + c % 8;
}

long long wino_v_offset(int C, long long P, int m, int dt, int xi, int nu, int c, long long b)
{
    Geo g;
    if (make_geo_kcp(1, C, P, m, dt, &g) != WINO_OK) return -1;
    if (xi < 0 || xi >= g.alpha || nu < 0 || nu >= g.alpha || c < 0 || c >= g.Cp || b < 0 || b >= g.Pp) return -1;
    const long long e = xi * g.alpha + nu;
    if (dt == WINO_F32) return (e * g.Cp + c) * g.Pp + b;
    return ((e * (g.Cp / 8) + c / 8) * g.Pp + b) * 8 + c % 8;
}

long long wino_m_offset(int K, long long P, int m, int xi, int nu, int k, long long b)
{
    Geo g;
    if (make_geo_kcp(K, 1, P, m, WINO_F32, &g) != WINO_OK) return -1;
    if (xi < 0 || xi >= g.alpha || nu < 0 || nu >= g.alpha || k < 0 || k >= g.Kp || b < 0 || b >= g.Pp) return -1;
    const long long e = xi * g.alpha + nu;
    return (e * g.Kp + k) * g.Pp + b;
}

size_t wino_filter_bytes(int K, int C, int m, int dt)
{
    Geo g;
    if (make_geo_kcp(K, C, 1, m, dt, &g) != WINO_OK) return 0;
    return u_bytes(g);
}

size_t wino_v_bytes(int C, long long P, int m, int dt)
{
    Geo g;
    if (make_geo_kcp(1, C, P, m, dt, &g) != WINO_OK) return 0;
    return v_bytes(g);
}

size_t wino_m_bytes(int K, long long P, int m)
{
    Geo g;
    if (make_geo_kcp(K, 1, P, m, WINO_F32, &g) != WINO_OK) return 0;
    return m_bytes(g);
}

size_t wino_workspace_bytes(int N, int C, int H, int W, int K, int pad, int m, int dt)
{
    Geo g;
    if (make_geo(N, C, H, W, K, pad, m, dt, &g) != WINO_OK) return 0;
    return align256(u_bytes(g)) + align256(v_bytes(g)) + align256(m_bytes(g) * gemm_splits(g));
}

int wino_filter_transform_ex(int K, int C, int m, int dt, const void *G, void *U, void *stream)
{
    Geo g;
    const int st = make_geo_kcp(K, C, 1, m, dt, &g);
    if (st != WINO_OK) return st;
    if (bad_ptr(G) || bad_ptr(U)) return WINO_EINVAL;
    const hipError_t e = launch_filter_transform(g, G, U, (hipStream_t)stream);
    return e == hipSuccess ? WINO_OK : hip_fail(e);
}

int wino_filter_transform(int K, int C, int m, const void *G, void *U, void *stream)
{
    return wino_filter_transform_ex(K, C, m, WINO_F32, G, U, stream);
}

int wino_input_transform(int N, int C, int H, int W, int pad, int m, int dt, const void *D, void *V, void *stream)
{
    Geo g;
    const int st = make_geo(N, C, H, W, 1, pad, m, dt, &g);
    if (st != WINO_OK) return st;
    if (bad_ptr(D) || bad_ptr(V)) return WINO_EINVAL;
    const hipError_t e = launch_input_transform(g, D, V, (hipStream_t)stream);
    return e == hipSuccess ? WINO_OK : hip_fail(e);
}

int wino_batched_gemm(int K, int C, long long P, int m, int dt, const void *U, const void *V, void *M, void *stream)
{
    Geo g;
    const int st = make_geo_kcp(K, C, P, m, dt, &g);
    if (st != WINO_OK) return st;
    if (bad_ptr(U) || bad_ptr(V) || bad_ptr(M)) return WINO_EINVAL;
    const hipError_t e = launch_batched_gemm(g, U, V, (float *)M, 1, (hipStream_t)stream);
    if (e == hipErrorNotSupported) return WINO_EUNSUPPORTED;
    return e == hipSuccess ? WINO_OK : hip_fail(e);
}

int wino_gemm_launch_shape(int K, int C, long long P, int m, int dt, int out[3])
{
    Geo g;
    const int st = make_geo_kcp(K, C, P, m, dt, &g);
    if (st != WINO_OK) return st;
    if (out == nullptr) return WINO_EINVAL;
    gemm_launch_shape(g, &out[0], &out[1], &out[2]);
    return WINO_OK;
}

int wino_output_transform(int N, int K, int H, int W, int pad, int m, int y_dt, const void *M, void *Y, void *stream)
{
    Geo g;
    const int st = make_geo(N, 1, H, W, K, pad, m, WINO_F32, &g);
    if (st != WINO_OK) return st;
    if (bad_dtype(y_dt)) return WINO_EINVAL;
    if (bad_ptr(M) || bad_ptr(Y)) return WINO_EINVAL;
    const hipError_t e = launch_output_transform(g, y_dt, (const float *)M, Y, 1, (hipStream_t)stream);
    return e == hipSuccess ? WINO_OK : hip_fail(e);
}

// The one-kernel paths write fp32 outputs; the fp16-storage one also writes fp16.
static bool fused_y_ok(const Geo &g, int y_dt) { return y_dt == WINO_F32 || g.dt == WINO_F16; }

int wino_conv2d_variant(int N, int C, int H, int W, int K, int pad, int m, int dt, int y_dt, unsigned flags)
{
    Geo g;
    const int st = make_geo(N, C, H, W, K, pad, m, dt, &g);
    if (st != WINO_OK) return -st;
    if (bad_dtype(y_dt) || flags > WINO_FLAG_ONE_LAUNCH) return -WINO_EINVAL;
    if (flags == WINO_FLAG_ONE_LAUNCH)
        return (fused_f2_eligible(g) && y_dt == WINO_F32) ? (int)WINO_FLAG_ONE_LAUNCH : -WINO_EUNSUPPORTED;
    if (flags == WINO_FLAG_FUSED) return (fused_eligible(g) && fused_y_ok(g, y_dt)) ? (int)WINO_FLAG_FUSED : -WINO_EUNSUPPORTED;
    if (flags == WINO_FLAG_AUTO && fused_y_ok(g, y_dt) && fused_preferred(g)) return WINO_FLAG_FUSED;
    return WINO_FLAG_UNFUSED;
}

int wino_one_kernel_plan(int N, int C, int H, int W, int K, int pad, int m, int dt, int out[32])
{
    Geo g;
    const int st = make_geo(N, C, H, W, K, pad, m, dt, &g);
    if (st != WINO_OK) return -st;
    if (out == nullptr) return -WINO_EINVAL;
    if (!fused_eligible(g) || !fused_wide_eligible(g)) return -WINO_EUNSUPPORTED;
    const int grid = fused_wide_plan(g, out);
    return grid < 0 ? -WINO_EINVAL : grid;
}

// Shared driver of the forward layer and of the input gradient: `g` is the geometry the kernels see,
// `bwd` selects the filter transform (plain, or rotated and transposed).
static int run_layer(const Geo &g, int y_dt, const void *D, const void *G, const void *U, void *Y, void *workspace,
                     size_t workspace_bytes, unsigned flags, bool bwd, hipStream_t s)
{
    if (bad_dtype(y_dt)) return WINO_EINVAL;
    if (flags > WINO_FLAG_ONE_LAUNCH) return WINO_EINVAL;
    if (flags == WINO_FLAG_FUSED && (!fused_eligible(g) || !fused_y_ok(g, y_dt))) return WINO_EUNSUPPORTED;
    if (flags == WINO_FLAG_ONE_LAUNCH && (!fused_f2_eligible(g) || y_dt != WINO_F32 || U != nullptr))
        return WINO_EUNSUPPORTED;
    if (bad_ptr(D) || bad_ptr(Y) || bad_ptr(workspace)) return WINO_EINVAL;
    if (U == nullptr ? bad_ptr(G) : !aligned16(U)) return WINO_EINVAL;
    const int splits = gemm_splits(g);
    const size_t ub = align256(u_bytes(g)), vb = align256(v_bytes(g)), mb = align256(m_bytes(g) * splits);
    if (workspace_bytes < ub + vb + mb) return WINO_EWORKSPACE;
    char *ws = (char *)workspace;
    void *Uw = ws, *Vw = ws + ub;
    float *Mw = (float *)(ws + ub + vb);
    hipError_t e;
    if (flags == WINO_FLAG_ONE_LAUNCH) {
        e = launch_fused_f2(g, (const float *)D, (const float *)G, (float *)Y, workspace, workspace_bytes, bwd, s);
        return e == hipSuccess ? WINO_OK : hip_fail(e);
    }
    if (flags == WINO_FLAG_AUTO && fused_y_ok(g, y_dt) && fused_preferred(g)) flags = WINO_FLAG_FUSED;
    bool v_done = false;
    // the one-kernel fp32 layer keeps arrival counters behind U: the filter transform in front of it clears them
    const bool wide = flags == WINO_FLAG_FUSED && fused_wide_eligible(g);
    unsigned int *const counters = wide && U == nullptr && fused_wide_shares(g, Vw, vb + mb) ? (unsigned int *)Vw : nullptr;
    if (U == nullptr) {
        if (!bwd && flags != WINO_FLAG_FUSED && prep_eligible(g)) {
            // filters and input tiles are transformed by one launch
            e = launch_prep(g, G, Uw, D, Vw, s);
            v_done = true;
        } else {
            e = bwd ? launch_filter_transform_bwd(g, G, Uw, s, counters) : launch_filter_transform(g, G, Uw, s, counters);
        }
        if (e != hipSuccess) return hip_fail(e);
        U = Uw;
    }
    if (flags == WINO_FLAG_FUSED) {
        // fp32 with pad 1 and W % 4 == 0: the designs with two workgroups per CU (64 filters per workgroup where
        // there are that many); otherwise the general one
        if (wide)
            e = launch_fused_wide(g, (const float *)D, (const float *)U, (float *)Y, Vw, vb + mb, counters != nullptr, s);
        else
            e = fused_lds_eligible(g) ? launch_fused_lds(g, (const float *)D, (const float *)U, (float *)Y, s)
                                      : launch_fused(g, D, U, Y, y_dt, s);
        if (e != hipSuccess) return hip_fail(e);
        return WINO_OK;
    }
    if (!v_done && (e = launch_input_transform(g, D, Vw, s)) != hipSuccess) return hip_fail(e);
    if ((e = launch_batched_gemm(g, U, Vw, Mw, splits, s)) != hipSuccess)
        return e == hipErrorNotSupported ? (int)WINO_EUNSUPPORTED : hip_fail(e);
    if ((e = launch_output_transform(g, y_dt, Mw, Y, splits, s)) != hipSuccess) return hip_fail(e);
    return WINO_OK;
}

int wino_conv2d_fwd_ex(int N, int C, int H, int W, int K, int pad, int m, int dt, int y_dt, const void *D,
                       const void *G, const void *U, void *Y, void *workspace, size_t workspace_bytes, unsigned flags,
                       void *stream)
{
    Geo g;
    const int st = make_geo(N, C, H, W, K, pad, m, dt, &g);
    if (st != WINO_OK) return st;
    return run_layer(g, y_dt, D, G, U, Y, workspace, workspace_bytes, flags, false, (hipStream_t)stream);
}

int wino_filter_transform_bwd(int K, int C, int m, int dt, const void *G, void *U, void *stream)
{
    Geo g;
    const int st = make_geo_kcp(C, K, 1, m, dt, &g);   // the swapped layer: C "filters", K "channels"
    if (st != WINO_OK) return st;
    if (bad_ptr(G) || bad_ptr(U)) return WINO_EINVAL;
    const hipError_t e = launch_filter_transform_bwd(g, G, U, (hipStream_t)stream);
    return e == hipSuccess ? WINO_OK : hip_fail(e);
}

int wino_conv2d_bwd_data(int N, int C, int H, int W, int K, int pad, int m, int dt, int d_dt, const void *E,
                         const void *G, const void *U, void *dD, void *workspace, size_t workspace_bytes,
                         unsigned flags, void *stream)
{
    if (pad != 1) return WINO_EUNSUPPORTED;   // pad 0 would need pad 2 in the exchanged layer
    Geo g;
    const int st = make_geo(N, K, H, W, C, 1, m, dt, &g);   // error tensor in, K channels; C outputs
    if (st != WINO_OK) return st;
    return run_layer(g, d_dt, E, G, U, dD, workspace, workspace_bytes, flags, true, (hipStream_t)stream);
}

size_t wino_bwd_filter_workspace_bytes(int N, int C, int H, int W, int K)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || !wgrad_supported(N, C, H, W, K)) return 0;
    return wgrad_workspace_bytes(N, C, H, W, K);
}

int wino_conv2d_bwd_filter(int N, int C, int H, int W, int K, int pad, int dt, const void *D, const void *E, void *dG,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0) return WINO_EINVAL;
    if (bad_dtype(dt)) return WINO_EINVAL;
    if (dt != WINO_F32 || pad != 1 || !wgrad_supported(N, C, H, W, K)) return WINO_EUNSUPPORTED;
    if (bad_ptr(D) || bad_ptr(E) || bad_ptr(dG) || bad_ptr(workspace)) return WINO_EINVAL;
    if (workspace_bytes < wgrad_workspace_bytes(N, C, H, W, K)) return WINO_EWORKSPACE;
    const hipError_t e = launch_wgrad(N, C, H, W, K, (const float *)D, (const float *)E, (float *)dG, workspace,
                                      (hipStream_t)stream);
    return e == hipSuccess ? WINO_OK : hip_fail(e);
}

int wino_conv2d_fwd(int N, int C, int H, int W, int K, int pad, int m, const void *D, const void *G, void *Y,
                    void *stream)
{
    Geo g;
    const int st = make_geo(N, C, H, W, K, pad, m, WINO_F32, &g);
    if (st != WINO_OK) return st;
    if (bad_ptr(D) || bad_ptr(G) || bad_ptr(Y)) return WINO_EINVAL;
    const size_t need = wino_workspace_bytes(N, C, H, W, K, pad, m, WINO_F32);
    void *ws = nullptr;
    size_t ws_bytes = 0;
    {
        std::lock_guard<std::mutex> lock(g_ws_mutex);
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return hip_fail(e);
        CachedWs *slot = nullptr;
        for (CachedWs &c : g_ws)
            if (c.stream == (hipStream_t)stream && c.device == dev) slot = &c;
        if (slot == nullptr) {
            g_ws.push_back(CachedWs{(hipStream_t)stream, dev, nullptr, 0});
            slot = &g_ws.back();
        }
        if (slot->bytes < need) {
            const size_t want = need > 2 * slot->bytes ? need : 2 * slot->bytes;
            void *fresh = nullptr;
            if ((e = hipMalloc(&fresh, want)) != hipSuccess) return hip_fail(e);
            if (slot->ptr != nullptr) g_ws_retired.push_back(slot->ptr);
            slot->ptr = fresh;
            slot->bytes = want;
        }
        ws = slot->ptr;
        ws_bytes = slot->bytes;
    }
    return wino_conv2d_fwd_ex(N, C, H, W, K, pad, m, WINO_F32, WINO_F32, D, G, nullptr, Y, ws, ws_bytes,
                              WINO_FLAG_AUTO, stream);
}

int wino_conv2d_fwd_noalloc(int N, int C, int H, int W, int K, int pad, int m, const void *D, const void *G, void *Y,
                            void *stream)
{
    Geo g;
    const int st = make_geo(N, C, H, W, K, pad, m, WINO_F32, &g);
    if (st != WINO_OK) return st;
    if (bad_ptr(D) || bad_ptr(G) || bad_ptr(Y)) return WINO_EINVAL;
    if (wino_workspace_bytes(N, C, H, W, K, pad, m, WINO_F32) > (size_t)WINO_STATIC_WORKSPACE_BYTES)
        return WINO_EWORKSPACE;   // the layer needs more than the built-in workspace holds
    void *ws = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return hip_fail(e);
        if (dev < 0 || dev >= kMaxDevices) return WINO_EUNSUPPORTED;
        if (g_scratch_ptr[dev] == nullptr) {
            void *p = nullptr;
            if ((e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) != hipSuccess) return hip_fail(e);
            if (p == nullptr) return hip_fail(hipErrorInvalidSymbol);
            g_scratch_ptr[dev] = p;
        }
        ws = g_scratch_ptr[dev];
    }
    // Nothing in the workspace has to start at zero: the transforms write every element of U and V that the
    // multiply reads (padding included), and the multiply writes every element of M the inverse transform reads.
    return run_layer(g, WINO_F32, D, G, nullptr, Y, ws, (size_t)WINO_STATIC_WORKSPACE_BYTES, WINO_FLAG_AUTO, false,
                     (hipStream_t)stream);
}

int direct_conv2d_fwd(int N, int C, int H, int W, int K, int R, int S, int pad, int stride, int dt, const void *D,
                      const void *G, void *Y, void *stream)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0)
        return WINO_EINVAL;
    if (bad_dtype(dt)) return WINO_EINVAL;
    if (H + 2 * pad < R || W + 2 * pad < S) return WINO_EUNSUPPORTED;
    if (R * S > 512 || N > 65535 || K > 65535 * 16) return WINO_EUNSUPPORTED;
    const long long Ho = (H + 2 * pad - R) / stride + 1, Wo = (W + 2 * pad - S) / stride + 1;
    if (Ho * Wo > (1LL << 30)) return WINO_EUNSUPPORTED;
    if (bad_ptr(D) || bad_ptr(G) || bad_ptr(Y)) return WINO_EINVAL;
    const hipError_t e = launch_direct_conv(N, C, H, W, K, R, S, pad, stride, dt, D, G, Y, (hipStream_t)stream);
    return e == hipSuccess ? WINO_OK : hip_fail(e);
}

int wino_shutdown(void)
{
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    if (g_ws.empty() && g_ws_retired.empty()) return WINO_OK;
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) return hip_fail(e);
    int status = WINO_OK;
    for (CachedWs &c : g_ws)
        if (c.ptr != nullptr && (e = hipFree(c.ptr)) != hipSuccess) status = hip_fail(e);
    for (void *p : g_ws_retired)
        if ((e = hipFree(p)) != hipSuccess) status = hip_fail(e);
    g_ws.clear();
    g_ws_retired.clear();
    return status;
}

}  // extern "C"

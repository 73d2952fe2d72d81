"""ctypes binding of libwino.so: same names as include/wino.h, argument marshalling only.

Tensors are torch tensors on the GPU (PyTorch is used for device memory and streams only);
every function passes ``data_ptr()`` and the current HIP stream to the C ABI and raises
``WinoError`` on a non-zero status.  There is no CPU fallback: if the shared library is not
present, loading fails.
"""
import ctypes
import os

import numpy as np

from . import build as _build

WINO_OK, WINO_EINVAL, WINO_EUNSUPPORTED, WINO_EWORKSPACE, WINO_EHIP = range(5)
WINO_F32, WINO_F16 = 0, 1
FLAG_AUTO, FLAG_UNFUSED, FLAG_FUSED, FLAG_ONE_LAUNCH = 0, 1, 2, 3

_lib = None


class WinoError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().wino_status_string(status).decode()
        if status == WINO_EHIP:
            msg += " (hipError %d)" % lib().wino_last_hip_error()
        super().__init__("%s: %s" % (where, msg))


def lib():
    """The loaded C library (loads it on first use; raises if it has not been built)."""
    global _lib
    if _lib is None:
        path = _build.LIB_PATH
        if not os.path.exists(path):
            raise RuntimeError("libwino.so is not built: run `python -m paper_1509_09308_amd.build`")
        L = ctypes.CDLL(path)
        i, ll, p, sz, u = ctypes.c_int, ctypes.c_longlong, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint
        ip, llp = ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_longlong)
        sig = {
            "wino_status_string": (ctypes.c_char_p, [i]),
            "wino_last_hip_error": (i, []),
            "wino_num_tiles": (ll, [i] * 5),
            "wino_tile_coords": (i, [i] * 5 + [ll, ip]),
            "wino_padded_dims": (i, [i, i, ll, i, i, ip, ip, llp]),
            "wino_u_offset": (ll, [i] * 8),
            "wino_v_offset": (ll, [i, ll, i, i, i, i, i, ll]),
            "wino_m_offset": (ll, [i, ll, i, i, i, i, ll]),
            "wino_filter_bytes": (sz, [i] * 4),
            "wino_v_bytes": (sz, [i, ll, i, i]),
            "wino_m_bytes": (sz, [i, ll, i]),
            "wino_workspace_bytes": (sz, [i] * 8),
            "wino_filter_transform": (i, [i, i, i, p, p, p]),
            "wino_filter_transform_ex": (i, [i, i, i, i, p, p, p]),
            "wino_input_transform": (i, [i] * 7 + [p, p, p]),
            "wino_batched_gemm": (i, [i, i, ll, i, i, p, p, p, p]),
            "wino_gemm_launch_shape": (i, [i, i, ll, i, i, ip]),
            "wino_output_transform": (i, [i] * 7 + [p, p, p]),
            "wino_conv2d_fwd": (i, [i] * 7 + [p, p, p, p]),
            "wino_conv2d_fwd_noalloc": (i, [i] * 7 + [p, p, p, p]),
            "wino_conv2d_fwd_ex": (i, [i] * 9 + [p, p, p, p, p, sz, u, p]),
            "wino_conv2d_variant": (i, [i] * 9 + [u]),
            "wino_one_kernel_plan": (i, [i] * 8 + [ip]),
            "wino_filter_transform_bwd": (i, [i, i, i, i, p, p, p]),
            "wino_bwd_filter_workspace_bytes": (sz, [i] * 5),
            "wino_conv2d_bwd_filter": (i, [i] * 7 + [p, p, p, p, sz, p]),
            "wino_conv2d_bwd_data": (i, [i] * 9 + [p, p, p, p, p, sz, u, p]),
            "direct_conv2d_fwd": (i, [i] * 10 + [p, p, p, p]),
            "wino_shutdown": (i, []),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


EXPORTS = ["wino_status_string", "wino_last_hip_error", "wino_num_tiles", "wino_tile_coords",
           "wino_padded_dims", "wino_u_offset", "wino_v_offset", "wino_m_offset", "wino_filter_bytes",
           "wino_v_bytes", "wino_m_bytes", "wino_workspace_bytes", "wino_filter_transform",
           "wino_filter_transform_ex", "wino_input_transform", "wino_batched_gemm", "wino_gemm_launch_shape",
           "wino_output_transform", "wino_conv2d_fwd", "wino_conv2d_fwd_noalloc", "wino_conv2d_fwd_ex", "wino_conv2d_variant", "wino_one_kernel_plan", "wino_filter_transform_bwd", "wino_conv2d_bwd_data",
           "wino_bwd_filter_workspace_bytes", "wino_conv2d_bwd_filter",
           "direct_conv2d_fwd",
           "wino_shutdown"]


def _check(status, where):
    if status != WINO_OK:
        raise WinoError(status, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dt(t):
    import torch
    if t.dtype == torch.float32:
        return WINO_F32
    if t.dtype == torch.float16:
        return WINO_F16
    raise TypeError("tensor must be float32 or float16")


def _torch_dtype(dt):
    import torch
    return torch.float32 if dt == WINO_F32 else torch.float16


def _dense_cuda(t, name):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("%s must be a contiguous GPU tensor" % name)
    return t


# ---- host-side queries ------------------------------------------------------------------------

def wino_num_tiles(N, H, W, pad, m):
    return int(lib().wino_num_tiles(N, H, W, pad, m))


def wino_tile_coords(N, H, W, pad, m, b):
    out = (ctypes.c_int * 5)()
    _check(lib().wino_tile_coords(N, H, W, pad, m, b, out), "wino_tile_coords")
    return tuple(out)


def wino_padded_dims(K, C, P, m, dt=WINO_F32):
    kp, cp, pp = ctypes.c_int(), ctypes.c_int(), ctypes.c_longlong()
    _check(lib().wino_padded_dims(K, C, P, m, dt, ctypes.byref(kp), ctypes.byref(cp), ctypes.byref(pp)),
           "wino_padded_dims")
    return kp.value, cp.value, pp.value


def wino_u_offset(K, C, m, dt, xi, nu, k, c):
    return int(lib().wino_u_offset(K, C, m, dt, xi, nu, k, c))


def wino_v_offset(C, P, m, dt, xi, nu, c, b):
    return int(lib().wino_v_offset(C, P, m, dt, xi, nu, c, b))


def wino_m_offset(K, P, m, xi, nu, k, b):
    return int(lib().wino_m_offset(K, P, m, xi, nu, k, b))


def wino_filter_bytes(K, C, m, dt=WINO_F32):
    return int(lib().wino_filter_bytes(K, C, m, dt))


def wino_v_bytes(C, P, m, dt=WINO_F32):
    return int(lib().wino_v_bytes(C, P, m, dt))


def wino_m_bytes(K, P, m):
    return int(lib().wino_m_bytes(K, P, m))


def wino_workspace_bytes(N, C, H, W, K, pad, m, dt=WINO_F32):
    return int(lib().wino_workspace_bytes(N, C, H, W, K, pad, m, dt))


# ---- buffers in the library's transform-domain layouts --------------------------------------------

def alloc_u(K, C, m, dt=WINO_F32, device="cuda"):
    import torch
    n = wino_filter_bytes(K, C, m, dt) // (4 if dt == WINO_F32 else 2)
    return torch.empty(n, dtype=_torch_dtype(dt), device=device)


def alloc_v(C, P, m, dt=WINO_F32, device="cuda"):
    import torch
    n = wino_v_bytes(C, P, m, dt) // (4 if dt == WINO_F32 else 2)
    return torch.empty(n, dtype=_torch_dtype(dt), device=device)


def alloc_m(K, P, m, device="cuda"):
    import torch
    return torch.empty(wino_m_bytes(K, P, m) // 4, dtype=torch.float32, device=device)


def alloc_workspace(N, C, H, W, K, pad, m, dt=WINO_F32, device="cuda"):
    import torch
    return torch.empty(wino_workspace_bytes(N, C, H, W, K, pad, m, dt), dtype=torch.uint8, device=device)


def _unpack(flat, a, R, Cp, Rp, dt, rows_first):
    """flat buffer -> numpy [a, a, ., .] following the layouts documented in wino.h."""
    x = flat.detach().cpu().numpy()
    if dt == WINO_F32:
        x = x.reshape(a, a, Cp, Rp)                       # [xi][nu][c][row]
    else:
        x = x.reshape(a, a, Cp // 8, Rp, 8).transpose(0, 1, 2, 4, 3).reshape(a, a, Cp, Rp)
    return x.transpose(0, 1, 3, 2) if rows_first else x


def unpack_u(U, K, C, m, dt=WINO_F32, padded=False):
    """U buffer -> numpy [alpha, alpha, K, C] (or the padded [.., Kp, Cp])."""
    Kp, Cp, _ = wino_padded_dims(K, C, 0, m, dt)
    x = _unpack(U, m + 2, K, Cp, Kp, dt, rows_first=True)
    return x if padded else x[:, :, :K, :C]


def unpack_v(V, C, P, m, dt=WINO_F32, padded=False):
    """V buffer -> numpy [alpha, alpha, C, P] (or the padded [.., Cp, Pp])."""
    _, Cp, Pp = wino_padded_dims(1, C, P, m, dt)
    x = _unpack(V, m + 2, C, Cp, Pp, dt, rows_first=False)
    return x if padded else x[:, :, :C, :P]


def unpack_m(M, K, P, m):
    """M buffer -> numpy [alpha, alpha, K, P]."""
    Kp, _, Pp = wino_padded_dims(K, 1, P, m, WINO_F32)
    a = m + 2
    return M.detach().cpu().numpy().reshape(a, a, Kp, Pp)[:, :, :K, :P]


def pack_v(v, m, dt=WINO_F32, device="cuda"):
    """numpy [alpha, alpha, C, P] -> V buffer on the GPU (padding zero filled)."""
    import torch
    a = m + 2
    C, P = v.shape[2], v.shape[3]
    _, Cp, Pp = wino_padded_dims(1, C, P, m, dt)
    full = np.zeros((a, a, Cp, Pp), dtype=np.float32 if dt == WINO_F32 else np.float16)
    full[:, :, :C, :P] = v
    if dt == WINO_F16:
        full = full.reshape(a, a, Cp // 8, 8, Pp).transpose(0, 1, 2, 4, 3)
    return torch.from_numpy(np.ascontiguousarray(full).reshape(-1)).to(device)


def pack_u(u, m, dt=WINO_F32, device="cuda"):
    """numpy [alpha, alpha, K, C] -> U buffer on the GPU (padding zero filled)."""
    import torch
    a = m + 2
    K, C = u.shape[2], u.shape[3]
    Kp, Cp, _ = wino_padded_dims(K, C, 0, m, dt)
    full = np.zeros((a, a, Cp, Kp), dtype=np.float32 if dt == WINO_F32 else np.float16)
    full[:, :, :C, :K] = u.transpose(0, 1, 3, 2)
    if dt == WINO_F16:
        full = full.reshape(a, a, Cp // 8, 8, Kp).transpose(0, 1, 2, 4, 3)
    return torch.from_numpy(np.ascontiguousarray(full).reshape(-1)).to(device)


def pack_m(mm, m, device="cuda"):
    """numpy [alpha, alpha, K, P] -> M buffer on the GPU."""
    import torch
    a = m + 2
    K, P = mm.shape[2], mm.shape[3]
    Kp, _, Pp = wino_padded_dims(K, 1, P, m, WINO_F32)
    full = np.zeros((a, a, Kp, Pp), dtype=np.float32)
    full[:, :, :K, :P] = mm
    return torch.from_numpy(full.reshape(-1)).to(device)


# ---- stages ---------------------------------------------------------------------------------

def wino_filter_transform(G, m, U=None, stream=None):
    """G[K,C,3,3] -> U (library layout).  Returns U."""
    _dense_cuda(G, "G")
    K, C = G.shape[0], G.shape[1]
    dt = _dt(G)
    if U is None:
        U = alloc_u(K, C, m, dt, G.device)
    if dt == WINO_F32:
        st = lib().wino_filter_transform(K, C, m, _ptr(G), _ptr(U), _stream(stream))
    else:
        st = lib().wino_filter_transform_ex(K, C, m, dt, _ptr(G), _ptr(U), _stream(stream))
    _check(st, "wino_filter_transform")
    return U


def wino_input_transform(D, pad, m, V=None, stream=None):
    """D[N,C,H,W] -> V (library layout).  Returns V."""
    _dense_cuda(D, "D")
    N, C, H, W = D.shape
    dt = _dt(D)
    if V is None:
        V = alloc_v(C, wino_num_tiles(N, H, W, pad, m), m, dt, D.device)
    _check(lib().wino_input_transform(N, C, H, W, pad, m, dt, _ptr(D), _ptr(V), _stream(stream)),
           "wino_input_transform")
    return V


def wino_batched_gemm(U, V, K, C, P, m, M=None, stream=None):
    """M^(xi,nu) = U^(xi,nu) V^(xi,nu).  Returns M (library layout, fp32)."""
    dt = _dt(U)
    if M is None:
        M = alloc_m(K, P, m, U.device)
    _check(lib().wino_batched_gemm(K, C, P, m, dt, _ptr(U), _ptr(V), _ptr(M), _stream(stream)),
           "wino_batched_gemm")
    return M


def wino_output_transform(M, N, K, H, W, pad, m, Y=None, y_dtype=None, stream=None):
    """M (library layout) -> Y[N,K,Ho,Wo]."""
    import torch
    if Y is None:
        Y = torch.empty((N, K, H + 2 * pad - 2, W + 2 * pad - 2), dtype=y_dtype or torch.float32, device=M.device)
    _check(lib().wino_output_transform(N, K, H, W, pad, m, _dt(Y), _ptr(M), _ptr(Y), _stream(stream)),
           "wino_output_transform")
    return Y


# ---- whole layer ------------------------------------------------------------------------------

def wino_conv2d_fwd(D, G, pad=1, m=4, Y=None, stream=None):
    """fp32 layer through the library-owned workspace (the short C entry point)."""
    import torch
    _dense_cuda(D, "D"), _dense_cuda(G, "G")
    N, C, H, W = D.shape
    K = G.shape[0]
    if Y is None:
        Y = torch.empty((N, K, H + 2 * pad - 2, W + 2 * pad - 2), dtype=torch.float32, device=D.device)
    _check(lib().wino_conv2d_fwd(N, C, H, W, K, pad, m, _ptr(D), _ptr(G), _ptr(Y), _stream(stream)),
           "wino_conv2d_fwd")
    return Y


STATIC_WORKSPACE_BYTES = 64 << 20


def wino_conv2d_fwd_noalloc(D, G, Y, pad=1, m=4, stream=None):
    """fp32 layer through the workspace built into the library: the C call allocates nothing (Y is the caller's)."""
    _dense_cuda(D, "D"), _dense_cuda(G, "G"), _dense_cuda(Y, "Y")
    N, C, H, W = D.shape
    K = G.shape[0]
    if tuple(Y.shape) != (N, K, H + 2 * pad - 2, W + 2 * pad - 2) or _dt(Y) != WINO_F32:
        raise ValueError("Y must be float32 of shape [N, K, Ho, Wo]")
    _check(lib().wino_conv2d_fwd_noalloc(N, C, H, W, K, pad, m, _ptr(D), _ptr(G), _ptr(Y), _stream(stream)),
           "wino_conv2d_fwd_noalloc")
    return Y


def wino_conv2d_fwd_ex(D, G=None, U=None, pad=1, m=4, Y=None, y_dtype=None, workspace=None, flags=FLAG_AUTO,
                       K=None, stream=None):
    """General layer entry point: caller-owned workspace, optional pre-transformed filters."""
    import torch
    _dense_cuda(D, "D")
    N, C, H, W = D.shape
    if G is not None:
        K = G.shape[0]
    if K is None:
        raise ValueError("K is required when only U is given")
    dt = _dt(D)
    if Y is None:
        Y = torch.empty((N, K, H + 2 * pad - 2, W + 2 * pad - 2), dtype=y_dtype or torch.float32, device=D.device)
    if workspace is None:
        workspace = alloc_workspace(N, C, H, W, K, pad, m, dt, D.device)
    _check(lib().wino_conv2d_fwd_ex(N, C, H, W, K, pad, m, dt, _dt(Y), _ptr(D), _ptr(G), _ptr(U), _ptr(Y),
                                    _ptr(workspace), workspace.numel() * workspace.element_size(), flags,
                                    _stream(stream)), "wino_conv2d_fwd_ex")
    return Y


def wino_one_kernel_plan(N, C, H, W, K, pad=1, m=4, dt=WINO_F32):
    """(workgroups of the launch, [(items, in full rounds, in the last round, shares)] per XCD) of the one-kernel fp32 layer."""
    out = (ctypes.c_int * 32)()
    grid = int(lib().wino_one_kernel_plan(N, C, H, W, K, pad, m, dt, out))
    if grid < 0:
        raise WinoError(-grid, "wino_one_kernel_plan")
    return grid, [tuple(int(out[4 * x + j]) for j in range(4)) for x in range(8)]


def wino_gemm_launch_shape(K, C, P, m, dt=WINO_F32):
    """(filters, tiles) of M per workgroup and the number of channel shares the whole-layer entry points use."""
    out = (ctypes.c_int * 3)()
    _check(lib().wino_gemm_launch_shape(K, C, P, m, dt, out), "wino_gemm_launch_shape")
    return int(out[0]), int(out[1]), int(out[2])


def wino_conv2d_variant(N, C, H, W, K, pad, m, dt=WINO_F32, y_dt=WINO_F32, flags=FLAG_AUTO):
    """FLAG_UNFUSED, FLAG_FUSED or FLAG_ONE_LAUNCH: the path wino_conv2d_fwd_ex takes; raises if it would be rejected."""
    v = int(lib().wino_conv2d_variant(N, C, H, W, K, pad, m, dt, y_dt, flags))
    if v < 0:
        raise WinoError(-v, "wino_conv2d_variant")
    return v


def wino_filter_transform_bwd(G, m, U=None, stream=None):
    """G[K,C,3,3] -> U' of the exchanged layer (C filters, K channels), filters rotated by 180 degrees."""
    _dense_cuda(G, "G")
    K, C = G.shape[0], G.shape[1]
    dt = _dt(G)
    if U is None:
        U = alloc_u(C, K, m, dt, G.device)
    _check(lib().wino_filter_transform_bwd(K, C, m, dt, _ptr(G), _ptr(U), _stream(stream)),
           "wino_filter_transform_bwd")
    return U


def wino_conv2d_bwd_data(E, G=None, U=None, C=None, pad=1, m=4, dD=None, d_dtype=None, workspace=None,
                         flags=FLAG_AUTO, stream=None):
    """Input gradient: E[N,K,H,W] and G[K,C,3,3] (or its bwd-transformed U plus C) -> dD[N,C,H,W]."""
    import torch
    _dense_cuda(E, "E")
    N, K, H, W = E.shape
    if G is not None:
        C = G.shape[1]
    if C is None:
        raise ValueError("C is required when only U is given")
    dt = _dt(E)
    if dD is None:
        dD = torch.empty((N, C, H, W), dtype=d_dtype or torch.float32, device=E.device)
    if workspace is None:
        workspace = alloc_workspace(N, K, H, W, C, pad, m, dt, E.device)
    _check(lib().wino_conv2d_bwd_data(N, C, H, W, K, pad, m, dt, _dt(dD), _ptr(E), _ptr(G), _ptr(U), _ptr(dD),
                                      _ptr(workspace), workspace.numel() * workspace.element_size(), flags,
                                      _stream(stream)), "wino_conv2d_bwd_data")
    return dD


def wino_bwd_filter_workspace_bytes(N, C, H, W, K):
    return int(lib().wino_bwd_filter_workspace_bytes(N, C, H, W, K))


def wino_conv2d_bwd_filter(D, E, pad=1, dG=None, workspace=None, stream=None):
    """Filter gradient with F(3x3,2x2): D[N,C,H,W], E[N,K,H,W] -> dG[K,C,3,3] (fp32)."""
    import torch
    _dense_cuda(D, "D"), _dense_cuda(E, "E")
    N, C, H, W = D.shape
    K = E.shape[1]
    if dG is None:
        dG = torch.empty((K, C, 3, 3), dtype=torch.float32, device=D.device)
    if workspace is None:
        workspace = torch.empty(wino_bwd_filter_workspace_bytes(N, C, H, W, K), dtype=torch.uint8, device=D.device)
    _check(lib().wino_conv2d_bwd_filter(N, C, H, W, K, pad, _dt(D), _ptr(D), _ptr(E), _ptr(dG), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream)),
           "wino_conv2d_bwd_filter")
    return dG


def direct_conv2d_fwd(D, G, pad=1, stride=1, Y=None, stream=None):
    """Eq. (1) evaluated directly on the GPU; Y has the dtype of D."""
    import torch
    _dense_cuda(D, "D"), _dense_cuda(G, "G")
    N, C, H, W = D.shape
    K, _, R, S = G.shape
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    if Y is None:
        Y = torch.empty((N, K, Ho, Wo), dtype=D.dtype, device=D.device)
    _check(lib().direct_conv2d_fwd(N, C, H, W, K, R, S, pad, stride, _dt(D), _ptr(D), _ptr(G), _ptr(Y),
                                   _stream(stream)), "direct_conv2d_fwd")
    return Y


def wino_shutdown():
    _check(lib().wino_shutdown(), "wino_shutdown")

"""TEST INFRASTRUCTURE ONLY: ctypes front end of ``direct_conv.c`` (Section 3, Eq. (1)).

The arithmetic lives in the C file; this module only compiles it with the host
compiler, checks shapes and passes pointers.  Parity pins: tests/test_oracle_direct.py.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "direct_conv.c")
_LIB = os.path.join(_HERE, "liboracle_conv.so")
_lib = None


def build(force=False):
    """Compile direct_conv.c with gcc (no fast-math: no output's sum is reassociated)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-std=c11", "-shared",
                               "-fPIC", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i, p, l = ctypes.c_int, ctypes.c_void_p, ctypes.c_long
        lib.oracle_num_threads.restype = i
        lib.oracle_conv2d_fwd_f64.argtypes = [i] * 9 + [p, p, p]
        lib.oracle_conv2d_fwd_f32in.argtypes = [i] * 9 + [p, p, p]
        lib.oracle_conv2d_points_f32in.argtypes = [i] * 9 + [p, p, l, p, p]
        lib.oracle_conv2d_bwd_data_f64.argtypes = [i] * 9 + [p, p, p]
        lib.oracle_conv2d_bwd_data_points_f32in.argtypes = [i] * 9 + [p, p, l, p, p]
        lib.oracle_conv2d_bwd_filter_f64.argtypes = [i] * 9 + [p, p, p]
        lib.oracle_conv2d_bwd_filter_points_f32in.argtypes = [i] * 9 + [p, p, l, p, p]
        for f in (lib.oracle_conv2d_fwd_f64, lib.oracle_conv2d_fwd_f32in,
                  lib.oracle_conv2d_points_f32in, lib.oracle_conv2d_bwd_data_f64,
                  lib.oracle_conv2d_bwd_data_points_f32in, lib.oracle_conv2d_bwd_filter_f64,
                  lib.oracle_conv2d_bwd_filter_points_f32in):
            f.restype = None
        _lib = lib
    return _lib


def num_threads():
    return int(_load().oracle_num_threads())


def _shapes(D, G, pad, stride):
    if D.ndim != 4 or G.ndim != 4 or D.shape[1] != G.shape[1]:
        raise ValueError("expected D[N,C,H,W] and G[K,C,R,S] with equal C")
    N, C, H, W = D.shape
    K, _, R, S = G.shape
    Ho = (H + 2 * pad - R) // stride + 1
    Wo = (W + 2 * pad - S) // stride + 1
    if Ho <= 0 or Wo <= 0:
        raise ValueError("empty output")
    return N, C, H, W, K, R, S, Ho, Wo


def _widen(a):
    """Stored tensors: fp64 stays, fp32 stays, fp16 widens exactly to fp32."""
    a = np.asarray(a)
    if a.dtype == np.float64:
        return np.ascontiguousarray(a)
    if a.dtype in (np.float32, np.float16):
        return np.ascontiguousarray(a, dtype=np.float32)
    return np.ascontiguousarray(a, dtype=np.float64)


def conv2d_fwd(D, G, pad=1, stride=1):
    """Y[i,k,x,y] = sum_c sum_u sum_v D[i,c,x*stride+u-pad,y*stride+v-pad] * G[k,c,u,v] in fp64."""
    D, G = _widen(D), _widen(G)
    if D.dtype != G.dtype:
        D, G = D.astype(np.float64), G.astype(np.float64)
    N, C, H, W, K, R, S, Ho, Wo = _shapes(D, G, pad, stride)
    Y = np.empty((N, K, Ho, Wo), dtype=np.float64)
    fn = _load().oracle_conv2d_fwd_f64 if D.dtype == np.float64 else _load().oracle_conv2d_fwd_f32in
    fn(N, C, H, W, K, R, S, pad, stride, D.ctypes.data, G.ctypes.data, Y.ctypes.data)
    return Y


def conv2d_points(D, G, pts, pad=1, stride=1):
    """The same sum for selected outputs only; ``pts`` is an (n,4) array of (i,k,x,y)."""
    D = np.ascontiguousarray(D, dtype=np.float32)
    G = np.ascontiguousarray(G, dtype=np.float32)
    N, C, H, W, K, R, S, Ho, Wo = _shapes(D, G, pad, stride)
    pts = np.ascontiguousarray(pts, dtype=np.int32).reshape(-1, 4)
    hi = np.array([N, K, Ho, Wo])
    if pts.size and ((pts < 0).any() or (pts >= hi).any()):
        raise ValueError("sample point outside the output tensor")
    out = np.empty(len(pts), dtype=np.float64)
    _load().oracle_conv2d_points_f32in(N, C, H, W, K, R, S, pad, stride, D.ctypes.data,
                                       G.ctypes.data, len(pts), pts.ctypes.data, out.ctypes.data)
    return out


def conv2d_bwd_data(E, G, H, W, pad=1, stride=1):
    """Gradient of the layer with respect to its input: E[N,K,Ho,Wo], G[K,C,R,S] -> dD[N,C,H,W] (fp64).
    Stored fp16/fp32 tensors are widened exactly."""
    E = np.ascontiguousarray(np.asarray(E), dtype=np.float64)
    G = np.ascontiguousarray(np.asarray(G), dtype=np.float64)
    N, K = E.shape[0], E.shape[1]
    K2, C, R, S = G.shape
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    if K2 != K or E.shape[2:] != (Ho, Wo):
        raise ValueError("error tensor does not match the layer geometry")
    dD = np.empty((N, C, H, W), dtype=np.float64)
    _load().oracle_conv2d_bwd_data_f64(N, C, H, W, K, R, S, pad, stride, E.ctypes.data, G.ctypes.data,
                                       dD.ctypes.data)
    return dD


def conv2d_bwd_data_points(E, G, H, W, pts, pad=1, stride=1):
    """Selected elements of the input gradient; ``pts`` is an (n,4) array of (i,c,x,y)."""
    E = np.ascontiguousarray(E, dtype=np.float32)
    G = np.ascontiguousarray(G, dtype=np.float32)
    N, K = E.shape[0], E.shape[1]
    K2, C, R, S = G.shape
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    if K2 != K or E.shape[2:] != (Ho, Wo):
        raise ValueError("error tensor does not match the layer geometry")
    pts = np.ascontiguousarray(pts, dtype=np.int32).reshape(-1, 4)
    hi = np.array([N, C, H, W])
    if pts.size and ((pts < 0).any() or (pts >= hi).any()):
        raise ValueError("sample point outside the gradient tensor")
    out = np.empty(len(pts), dtype=np.float64)
    _load().oracle_conv2d_bwd_data_points_f32in(N, C, H, W, K, R, S, pad, stride, E.ctypes.data, G.ctypes.data,
                                                len(pts), pts.ctypes.data, out.ctypes.data)
    return out


def conv2d_bwd_filter(D, E, R=3, S=3, pad=1, stride=1):
    """Gradient of the layer with respect to its filters: D[N,C,H,W], E[N,K,Ho,Wo] -> dG[K,C,R,S] (fp64)."""
    D = np.ascontiguousarray(np.asarray(D), dtype=np.float64)
    E = np.ascontiguousarray(np.asarray(E), dtype=np.float64)
    N, C, H, W = D.shape
    K = E.shape[1]
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    if E.shape[0] != N or E.shape[2:] != (Ho, Wo):
        raise ValueError("error tensor does not match the layer geometry")
    dG = np.empty((K, C, R, S), dtype=np.float64)
    _load().oracle_conv2d_bwd_filter_f64(N, C, H, W, K, R, S, pad, stride, D.ctypes.data, E.ctypes.data,
                                         dG.ctypes.data)
    return dG


def conv2d_bwd_filter_points(D, E, pts, R=3, S=3, pad=1, stride=1):
    """Selected elements of the filter gradient; ``pts`` is an (n,4) array of (k,c,u,v)."""
    D = np.ascontiguousarray(D, dtype=np.float32)
    E = np.ascontiguousarray(E, dtype=np.float32)
    N, C, H, W = D.shape
    K = E.shape[1]
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    if E.shape[0] != N or E.shape[2:] != (Ho, Wo):
        raise ValueError("error tensor does not match the layer geometry")
    pts = np.ascontiguousarray(pts, dtype=np.int32).reshape(-1, 4)
    hi = np.array([K, C, R, S])
    if pts.size and ((pts < 0).any() or (pts >= hi).any()):
        raise ValueError("sample point outside the gradient tensor")
    out = np.empty(len(pts), dtype=np.float64)
    _load().oracle_conv2d_bwd_filter_points_f32in(N, C, H, W, K, R, S, pad, stride, D.ctypes.data, E.ctypes.data,
                                                  len(pts), pts.ctypes.data, out.ctypes.data)
    return out

"""Shared helpers of the GPU parity tests (imported by test modules; not a test itself)."""
import numpy as np
import pytest

TOL = {("f32", 2): 1e-5, ("f32", 4): 1e-4, ("f32", 6): 1e-4, ("f16", 2): 5e-3, ("f16", 4): 5e-3}


def require_gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1509_09308_amd as w
    w.build.ensure_built()
    return torch, w


def rel_err(got, ref):
    """Normwise relative error ||got - ref||_F / ||ref||_F in float64."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm((got - ref).ravel()) / max(np.linalg.norm(ref.ravel()), 1e-300))


def to_gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()

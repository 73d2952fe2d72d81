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


# squared row norms of the inverse-transform matrices A^T (Eq. (7), Eq. (15), and the F(6,3) set): the error an
# output position (p, q) inherits from the rounding of the alpha^2 products grows with |A^T_p|^2 |A^T_q|^2
_AT_ROW_NORM2 = {1: [1.0], 2: [3.0, 3.0], 4: [5.0, 10.0, 34.0, 131.0],
                 6: [7.0, 10.5, 34.125, 130.03125, 514.0078125, 2050.001953125]}


def max_abs_bound(ref, tol, m=1):
    """Element-wise companion of the normwise bound ``tol``.  If the error vector has norm tol * ||ref||, its
    elements have RMS tol * rms(ref) over the tensor; the output position of a tile with the largest rows of A^T
    carries max|A^T_p|^2 / mean|A^T_p|^2 times that (1 for F(2x2) and for direct evaluation, 2.9 for F(4x4), 4.5
    for F(6x6)), and noise of that RMS stays below 6 RMS over 10^9 elements; 8 leaves slack:
    bound = 8 * ratio(m) * tol * rms(ref).  An element that is missing, misplaced or from the wrong tile is off
    by about rms(ref), i.e. by 1 / (8 ratio tol) >= 8 times this bound even at the loosest setting (fp16 storage,
    F(4x4)), so a handful of wrong elements that the norm would hide still fails."""
    ref = np.asarray(ref, dtype=np.float64)
    n2 = _AT_ROW_NORM2[m]
    ratio = max(n2) / (sum(n2) / len(n2))
    return 8.0 * ratio * tol * float(np.sqrt(np.mean(ref * ref)))


def check_close(got, ref, tol, what="", m=1):
    """Normwise relative error <= tol AND max-abs element error <= max_abs_bound(ref, tol, m); returns both."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    e = rel_err(got, ref)
    worst = float(np.abs(got - ref).max()) if got.size else 0.0
    bound = max_abs_bound(ref, tol, m)
    assert e <= tol, "%s: normwise relative error %.3e > %.1e" % (what, e, tol)
    assert worst <= bound, "%s: max-abs element error %.3e > %.3e" % (what, worst, bound)
    return e, worst

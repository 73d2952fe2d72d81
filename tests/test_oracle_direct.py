"""Pins for oracle/direct_conv.c (Eq. (1)): brute force, a library routine on the special
case it covers, and the invariants of the operation (no GPU)."""
import numpy as np
import pytest
import torch

from oracle import direct


def _brute(D, G, pad, stride=1):
    N, C, H, W = D.shape
    K, _, R, S = G.shape
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    Y = np.zeros((N, K, Ho, Wo))
    for i in range(N):
        for k in range(K):
            for x in range(Ho):
                for y in range(Wo):
                    s = 0.0
                    for c in range(C):
                        for u in range(R):
                            for v in range(S):
                                xx, yy = x * stride + u - pad, y * stride + v - pad
                                if 0 <= xx < H and 0 <= yy < W:
                                    s += D[i, c, xx, yy] * G[k, c, u, v]
                    Y[i, k, x, y] = s
    return Y


@pytest.mark.parametrize("pad,stride", [(1, 1), (0, 1), (1, 2), (2, 1)])
def test_brute_force_tiny(pad, stride):
    rng = np.random.default_rng(11)
    D = rng.standard_normal((1, 2, 5, 6))
    G = rng.standard_normal((2, 2, 3, 3))        # asymmetric: a flipped filter would fail
    got = direct.conv2d_fwd(D, G, pad=pad, stride=stride)
    assert np.allclose(got, _brute(D, G, pad, stride), rtol=0, atol=1e-13)


@pytest.mark.parametrize("shape", [(2, 5, 12, 9, 7, 3, 3, 1, 1), (1, 3, 11, 11, 4, 5, 5, 2, 2),
                                   (1, 4, 8, 8, 3, 1, 1, 0, 1), (2, 3, 9, 7, 2, 3, 2, 1, 1)])
def test_against_torch_float64_cross_correlation(shape):
    """torch.nn.functional.conv2d is cross-correlation: an independent library routine."""
    N, C, H, W, K, R, S, pad, stride = shape
    rng = np.random.default_rng(R * 10 + S)
    D = rng.standard_normal((N, C, H, W))
    G = rng.standard_normal((K, C, R, S))
    ref = torch.nn.functional.conv2d(torch.from_numpy(D), torch.from_numpy(G), padding=pad,
                                     stride=stride).numpy()
    got = direct.conv2d_fwd(D, G, pad=pad, stride=stride)
    assert got.shape == ref.shape
    assert np.abs(got - ref).max() < 1e-12


def test_f32_inputs_are_widened_not_rounded():
    rng = np.random.default_rng(3)
    D = rng.standard_normal((2, 4, 9, 9)).astype(np.float32)
    G = rng.standard_normal((3, 4, 3, 3)).astype(np.float32)
    a = direct.conv2d_fwd(D, G)
    b = direct.conv2d_fwd(D.astype(np.float64), G.astype(np.float64))
    assert np.array_equal(a, b)
    h = direct.conv2d_fwd(D.astype(np.float16), G.astype(np.float16))
    assert np.array_equal(h, direct.conv2d_fwd(D.astype(np.float16).astype(np.float64),
                                               G.astype(np.float16).astype(np.float64)))


def test_delta_filter_is_identity():
    rng = np.random.default_rng(4)
    C = 5
    D = rng.standard_normal((2, C, 7, 10))
    G = np.zeros((C, C, 3, 3))
    G[np.arange(C), np.arange(C), 1, 1] = 1.0
    assert np.array_equal(direct.conv2d_fwd(D, G, pad=1), D)


def test_off_centre_delta_shifts_the_right_way():
    """G[u=0,v=2]=1 reads D[x-1, y+1] with pad 1: pins row/column pairing and 'no flip'."""
    D = np.arange(30, dtype=np.float64).reshape(1, 1, 5, 6)
    G = np.zeros((1, 1, 3, 3))
    G[0, 0, 0, 2] = 1.0
    Y = direct.conv2d_fwd(D, G, pad=1)
    exp = np.zeros_like(D)
    exp[0, 0, 1:, :-1] = D[0, 0, :-1, 1:]
    assert np.array_equal(Y, exp)


def test_linearity_exact_on_small_integers():
    rng = np.random.default_rng(6)
    D1 = rng.integers(-9, 10, (2, 3, 8, 8)).astype(np.float64)
    D2 = rng.integers(-9, 10, (2, 3, 8, 8)).astype(np.float64)
    G1 = rng.integers(-9, 10, (4, 3, 3, 3)).astype(np.float64)
    G2 = rng.integers(-9, 10, (4, 3, 3, 3)).astype(np.float64)
    f = direct.conv2d_fwd
    assert np.array_equal(f(3 * D1 - 2 * D2, G1), 3 * f(D1, G1) - 2 * f(D2, G1))
    assert np.array_equal(f(D1, 5 * G1 + G2), 5 * f(D1, G1) + f(D1, G2))


def test_shift_equivariance_interior():
    rng = np.random.default_rng(8)
    D = rng.standard_normal((1, 2, 12, 12))
    G = rng.standard_normal((3, 2, 3, 3))
    Ds = np.roll(D, (2, 3), axis=(2, 3))
    Y, Ys = direct.conv2d_fwd(D, G), direct.conv2d_fwd(Ds, G)
    assert np.array_equal(Ys[:, :, 4:-1, 5:-1], Y[:, :, 2:-3, 2:-4])


def test_points_equal_full_tensor():
    rng = np.random.default_rng(9)
    D = rng.standard_normal((3, 4, 9, 11)).astype(np.float32)
    G = rng.standard_normal((5, 4, 3, 3)).astype(np.float32)
    Y = direct.conv2d_fwd(D, G)
    pts = np.stack([rng.integers(0, n, 200) for n in Y.shape], axis=1)
    got = direct.conv2d_points(D, G, pts)
    assert np.array_equal(got, Y[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]])
    with pytest.raises(ValueError):
        direct.conv2d_points(D, G, [[0, 0, 9, 0]])


# ---- gradient with respect to the input (Section 4.2, first paragraph) ----------------------------

@pytest.mark.parametrize("shape", [(2, 3, 7, 9, 4, 3, 3, 1, 1), (1, 2, 8, 8, 3, 3, 3, 0, 1), (2, 3, 9, 8, 2, 3, 3, 1, 2),
                                   (1, 4, 6, 6, 5, 1, 1, 0, 1), (1, 2, 10, 7, 3, 5, 5, 2, 1)])
def test_bwd_data_is_the_adjoint_of_the_layer(shape):
    """<conv(D, G), E> == <D, bwd(E, G)> exactly on small integers: the defining property of
    the input gradient, independent of how either side is computed."""
    N, C, H, W, K, R, S, pad, stride = shape
    rng = np.random.default_rng(sum(shape))
    D = rng.integers(-5, 6, (N, C, H, W)).astype(np.float64)
    G = rng.integers(-5, 6, (K, C, R, S)).astype(np.float64)
    Y = direct.conv2d_fwd(D, G, pad=pad, stride=stride)
    E = rng.integers(-5, 6, Y.shape).astype(np.float64)
    dD = direct.conv2d_bwd_data(E, G, H, W, pad=pad, stride=stride)
    assert dD.shape == D.shape
    assert float((Y * E).sum()) == float((D * dD).sum())


@pytest.mark.parametrize("shape", [(2, 3, 7, 9, 4, 3, 3, 1, 1), (1, 2, 8, 8, 3, 3, 3, 0, 1), (2, 3, 9, 8, 2, 3, 3, 1, 2)])
def test_bwd_data_against_torch_autograd_float64(shape):
    N, C, H, W, K, R, S, pad, stride = shape
    rng = np.random.default_rng(sum(shape) + 1)
    D = torch.from_numpy(rng.standard_normal((N, C, H, W))).requires_grad_(True)
    G = torch.from_numpy(rng.standard_normal((K, C, R, S)))
    Y = torch.nn.functional.conv2d(D, G, padding=pad, stride=stride)
    E = torch.from_numpy(rng.standard_normal(tuple(Y.shape)))
    Y.backward(E)
    got = direct.conv2d_bwd_data(E.numpy(), G.numpy(), H, W, pad=pad, stride=stride)
    assert np.abs(got - D.grad.numpy()).max() < 1e-12


def test_bwd_data_equals_forward_with_flipped_swapped_filters():
    """Section 4.2: for 3x3, stride 1, pad 1 the input gradient is the forward layer applied to
    the error with the filters flipped by 180 degrees and K, C exchanged."""
    rng = np.random.default_rng(12)
    E = rng.standard_normal((2, 5, 9, 11))
    G = rng.standard_normal((5, 4, 3, 3))
    Gf = np.ascontiguousarray(G[:, :, ::-1, ::-1].transpose(1, 0, 2, 3))
    a = direct.conv2d_bwd_data(E, G, 9, 11, pad=1)
    b = direct.conv2d_fwd(E, Gf, pad=1)
    assert np.abs(a - b).max() < 1e-12


def test_bwd_data_points_equal_full_tensor():
    rng = np.random.default_rng(13)
    E = rng.standard_normal((2, 6, 9, 11)).astype(np.float32)
    G = rng.standard_normal((6, 4, 3, 3)).astype(np.float32)
    full = direct.conv2d_bwd_data(E, G, 9, 11, pad=1)
    pts = np.stack([rng.integers(0, n, 100) for n in full.shape], axis=1)
    got = direct.conv2d_bwd_data_points(E, G, 9, 11, pts, pad=1)
    assert np.array_equal(got, full[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]])


# ---- gradient with respect to the filters (Section 4.2, second paragraph) -------------------------

@pytest.mark.parametrize("shape", [(2, 3, 7, 9, 4, 3, 3, 1, 1), (1, 2, 8, 8, 3, 3, 3, 0, 1), (2, 3, 9, 8, 2, 3, 3, 1, 2),
                                   (1, 2, 10, 7, 3, 5, 5, 2, 1)])
def test_bwd_filter_is_the_adjoint_in_the_filters(shape):
    """<conv(D, G), E> == <G, bwd_filter(D, E)> exactly on small integers."""
    N, C, H, W, K, R, S, pad, stride = shape
    rng = np.random.default_rng(sum(shape) + 7)
    D = rng.integers(-5, 6, (N, C, H, W)).astype(np.float64)
    G = rng.integers(-5, 6, (K, C, R, S)).astype(np.float64)
    Y = direct.conv2d_fwd(D, G, pad=pad, stride=stride)
    E = rng.integers(-5, 6, Y.shape).astype(np.float64)
    dG = direct.conv2d_bwd_filter(D, E, R=R, S=S, pad=pad, stride=stride)
    assert dG.shape == G.shape
    assert float((Y * E).sum()) == float((G * dG).sum())


@pytest.mark.parametrize("shape", [(2, 3, 7, 9, 4, 3, 3, 1, 1), (1, 2, 8, 8, 3, 3, 3, 0, 1), (2, 3, 9, 8, 2, 3, 3, 1, 2)])
def test_bwd_filter_against_torch_autograd_float64(shape):
    N, C, H, W, K, R, S, pad, stride = shape
    rng = np.random.default_rng(sum(shape) + 8)
    D = torch.from_numpy(rng.standard_normal((N, C, H, W)))
    G = torch.from_numpy(rng.standard_normal((K, C, R, S))).requires_grad_(True)
    Y = torch.nn.functional.conv2d(D, G, padding=pad, stride=stride)
    E = torch.from_numpy(rng.standard_normal(tuple(Y.shape)))
    Y.backward(E)
    got = direct.conv2d_bwd_filter(D.numpy(), E.numpy(), R=R, S=S, pad=pad, stride=stride)
    assert np.abs(got - G.grad.numpy()).max() < 1e-11


@pytest.mark.parametrize("pad,stride", [(1, 1), (0, 1), (1, 2)])
def test_bwd_filter_points_equal_the_full_gradient(pad, stride):
    """The one-element-at-a-time form must reproduce every element of the full gradient (exact integers)."""
    rng = np.random.default_rng(77 + pad + stride)
    N, C, H, W, K = 2, 3, 9, 11, 4
    D = rng.integers(-5, 6, (N, C, H, W)).astype(np.float32)
    Ho, Wo = (H + 2 * pad - 3) // stride + 1, (W + 2 * pad - 3) // stride + 1
    E = rng.integers(-5, 6, (N, K, Ho, Wo)).astype(np.float32)
    full = direct.conv2d_bwd_filter(D, E, pad=pad, stride=stride)
    pts = np.array([(k, c, u, v) for k in range(K) for c in range(C) for u in range(3) for v in range(3)])
    got = direct.conv2d_bwd_filter_points(D, E, pts, pad=pad, stride=stride)
    assert np.array_equal(got.reshape(K, C, 3, 3), full)
    with pytest.raises(ValueError):
        direct.conv2d_bwd_filter_points(D, E, np.array([[K, 0, 0, 0]]), pad=pad, stride=stride)

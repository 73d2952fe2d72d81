"""Stage-by-stage GPU tests through the C ABI: each loop of Algorithm 1 against the oracle's
stage reference.  Integer-valued inputs make every stage exact in fp32, so index and tile
bookkeeping is compared with ==."""
import numpy as np
import pytest

from oracle import winograd as wg
from oracle import direct
from paper_1509_09308_amd import synth
from gpu_util import require_gpu, rel_err, to_gpu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("m", [2, 4, 6])
@pytest.mark.parametrize("K,C", [(32, 32), (70, 19), (5, 3), (256, 128)])
def test_filter_transform(m, K, C):
    torch, w = require_gpu()
    rng = np.random.default_rng(K * 7 + C + m)
    # multiples of 4 make G g G^T exact for F(2,3) (entries 1, 1/2); F(4,3) has 1/6, F(6,3) has 1/90: rounded
    G = (rng.integers(-8, 9, (K, C, 3, 3)) * 4).astype(np.float32)
    U = w.wino_filter_transform(to_gpu(G), m)
    torch.cuda.synchronize()
    ref = wg.filter_transform(G, m)
    got = w.unpack_u(U, K, C, m)
    if m == 2:
        assert np.array_equal(got.astype(np.float64), ref)
    else:
        assert np.abs(got - ref).max() <= 4e-7 * np.abs(ref).max()
    # padding rows and columns are zero
    full = w.unpack_u(U, K, C, m, padded=True)
    assert not full[:, :, K:, :].any() and not full[:, :, :, C:].any()


@pytest.mark.parametrize("m", [2, 4, 6])
@pytest.mark.parametrize("N,C,H,W,pad", [(1, 4, 8, 8, 1), (2, 3, 14, 14, 1), (1, 2, 7, 9, 1), (2, 5, 9, 6, 0),
                                         (1, 17, 56, 56, 1), (3, 2, 30, 34, 1)])
def test_input_transform_bit_exact(m, N, C, H, W, pad):
    torch, w = require_gpu()
    rng = np.random.default_rng(H * 31 + W + m)
    D = rng.integers(-200, 201, (N, C, H, W)).astype(np.float32)
    V = w.wino_input_transform(to_gpu(D), pad, m)
    torch.cuda.synchronize()
    P = wg.num_tiles(N, H, W, pad, m)
    ref = wg.data_transform(D, pad, m)          # B^T has integer entries (quarters for F(6,3)): exact
    got = w.unpack_v(V, C, P, m)
    assert got.shape == ref.shape
    assert np.array_equal(got.astype(np.float64), ref)
    full = w.unpack_v(V, C, P, m, padded=True)
    assert not full[:, :, C:, :].any() and not full[:, :, :, P:].any()


@pytest.mark.parametrize("m", [2, 4, 6])
@pytest.mark.parametrize("K,C,P", [(32, 32, 784), (64, 64, 256), (70, 19, 100), (128, 48, 300), (256, 256, 130),
                                   (5, 3, 17), (192, 64, 49)])
def test_batched_gemm_exact_on_integers(m, K, C, P):
    torch, w = require_gpu()
    a = m + 2
    rng = np.random.default_rng(K + C + P + m)
    u = rng.integers(-4, 5, (a, a, K, C)).astype(np.float32)
    v = rng.integers(-4, 5, (a, a, C, P)).astype(np.float32)
    M = w.wino_batched_gemm(w.pack_u(u, m), w.pack_v(v, m), K, C, P, m)
    torch.cuda.synchronize()
    ref = wg.multiply(u.astype(np.float64), v.astype(np.float64))
    assert np.array_equal(w.unpack_m(M, K, P, m).astype(np.float64), ref)


def test_batched_gemm_one_hot_routing():
    """U^(e) = e-dependent permutation-like matrix: every M row must be the right V row."""
    torch, w = require_gpu()
    m, K, C, P = 2, 64, 64, 96
    a = m + 2
    u = np.zeros((a, a, K, C), dtype=np.float32)
    for xi in range(a):
        for nu in range(a):
            for k in range(K):
                u[xi, nu, k, (k * 5 + xi * a + nu) % C] = 1.0
    v = np.arange(a * a * C * P, dtype=np.float32).reshape(a, a, C, P) % 8191
    M = w.unpack_m(w.wino_batched_gemm(w.pack_u(u, m), w.pack_v(v, m), K, C, P, m), K, P, m)
    for xi in range(a):
        for nu in range(a):
            for k in range(0, K, 7):
                assert np.array_equal(M[xi, nu, k], v[xi, nu, (k * 5 + xi * a + nu) % C])


@pytest.mark.parametrize("m", [2, 4, 6])
@pytest.mark.parametrize("N,K,H,W,pad", [(1, 4, 8, 8, 1), (2, 3, 14, 14, 1), (1, 2, 7, 9, 1), (2, 5, 9, 6, 0),
                                         (1, 33, 56, 56, 1), (3, 2, 30, 34, 1)])
def test_output_transform_bit_exact(m, N, K, H, W, pad):
    torch, w = require_gpu()
    a = m + 2
    P = wg.num_tiles(N, H, W, pad, m)
    rng = np.random.default_rng(H * 17 + W + m)
    if m == 6:   # A^T of F(6,3) has entries down to 1/32: multiples of 32 keep both passes exact in fp32
        mm = (rng.integers(-3, 4, (a, a, K, P)) * 32).astype(np.float32)
    else:
        mm = rng.integers(-500, 501, (a, a, K, P)).astype(np.float32)
    Y = w.wino_output_transform(w.pack_m(mm, m), N, K, H, W, pad, m)
    torch.cuda.synchronize()
    ref = wg.inverse_transform(mm.astype(np.float64), N, H, W, pad, m)
    assert np.array_equal(Y.cpu().numpy().astype(np.float64), ref)


@pytest.mark.parametrize("shape", [(2, 16, 20, 20, 16), (1, 8, 15, 13, 8), (3, 5, 14, 14, 5)])
def test_f2x2_delta_filter_end_to_end_bitwise(shape):
    """m = 2: with a centre-one filter U has entries 0, 1/4, 1/2, 1 and every intermediate is
    exact in fp32, so the whole pipeline must return D bit for bit."""
    torch, w = require_gpu()
    N, C, H, W, K = shape
    D = (np.arange(N * C * H * W, dtype=np.float32) % 65521).reshape(N, C, H, W)
    rng = np.random.default_rng(1)
    rng.shuffle(D.reshape(-1))
    G = np.zeros((K, C, 3, 3), dtype=np.float32)
    G[np.arange(K), np.arange(C), 1, 1] = 1.0
    Y = w.wino_conv2d_fwd(to_gpu(D), to_gpu(G), pad=1, m=2)
    torch.cuda.synchronize()
    assert np.array_equal(Y.cpu().numpy(), D)


@pytest.mark.parametrize("m", [2, 4, 6])
def test_integer_layer_end_to_end_exact(m):
    """Integer data, filters that are multiples of the transform denominators: F(2x2) is
    exact end to end; F(4x4) and F(6x6) are exact except for the rounding of 1/6- and 1/90-type
    constants (amplified, for F(6x6), by the larger entries of its matrices)."""
    torch, w = require_gpu()
    D, G = synth.make_integer_layer(2, 6, 18, 22, 7, seed=3, gscale=4.0 if m == 2 else 576.0)
    Y = w.wino_conv2d_fwd(to_gpu(D), to_gpu(G), pad=1, m=m).cpu().numpy()
    ref = direct.conv2d_fwd(D, G, pad=1)
    if m == 2:
        assert np.array_equal(Y.astype(np.float64), ref)
    else:
        e = rel_err(Y, ref)
        print("integer layer m=%d rel err %.3e" % (m, e))
        assert e < (1e-6 if m == 4 else 1e-5)


@pytest.mark.parametrize("shape", [(1, 3, 20, 20, 8, 3, 3, 1, 1), (2, 3, 17, 23, 5, 5, 5, 2, 2),
                                   (1, 20, 9, 9, 33, 1, 1, 0, 1), (2, 4, 12, 10, 16, 3, 2, 1, 1),
                                   (1, 3, 224, 224, 64, 3, 3, 1, 1),
                                   # 3 x 3, stride 1, 1-4 channels (matrix-unit form): ragged row bands, column blocks
                                   # and filter blocks, both pads
                                   (2, 1, 9, 12, 70, 3, 3, 1, 1), (1, 2, 10, 36, 33, 3, 3, 0, 1),
                                   (2, 4, 7, 40, 64, 3, 3, 1, 1), (1, 3, 6, 260, 5, 3, 3, 1, 1),
                                   (1, 3, 3, 4, 130, 3, 3, 0, 1),
                                   (40, 3, 50, 36, 70, 3, 3, 1, 1)])   # enough workgroups for four-row bands
def test_direct_fallback(shape):
    torch, w = require_gpu()
    N, C, H, W, K, R, S, pad, stride = shape
    D, G = synth.make_layer(N, C, H, W, K, seed=H + R, R=R, S=S)
    Y = w.direct_conv2d_fwd(to_gpu(D), to_gpu(G), pad=pad, stride=stride).cpu().numpy()
    ref = direct.conv2d_fwd(D, G, pad=pad, stride=stride)
    assert Y.shape == ref.shape
    assert rel_err(Y, ref) < 1e-5
    # exact on integers
    Di = np.round(D * 4).astype(np.float32)
    Gi = np.round(G * 16).astype(np.float32)
    Yi = w.direct_conv2d_fwd(to_gpu(Di), to_gpu(Gi), pad=pad, stride=stride).cpu().numpy()
    assert np.array_equal(Yi.astype(np.float64), direct.conv2d_fwd(Di, Gi, pad=pad, stride=stride))


@pytest.mark.parametrize("shape", [(1, 3, 20, 20, 8, 3, 3, 1, 1), (2, 3, 17, 23, 5, 3, 3, 1, 1), (2, 5, 12, 16, 33, 3, 3, 0, 1),
                                   (1, 4, 9, 11, 6, 5, 3, 2, 2), (2, 3, 224, 224, 64, 3, 3, 1, 1),
                                   (2, 4, 9, 36, 70, 3, 3, 0, 1), (1, 1, 5, 8, 3, 3, 3, 1, 1)])
def test_direct_fallback_f16_storage(shape):
    """fp16 D, G and Y, fp32 accumulation: within one fp16 rounding of the oracle on the same stored values,
    and exact where the result is representable."""
    torch, w = require_gpu()
    N, C, H, W, K, R, S, pad, stride = shape
    D, G = synth.make_layer(N, C, H, W, K, seed=H + R + 1, R=R, S=S, dtype=np.float16)
    Y = w.direct_conv2d_fwd(to_gpu(D), to_gpu(G), pad=pad, stride=stride).cpu().numpy()
    ref = direct.conv2d_fwd(D, G, pad=pad, stride=stride)
    assert Y.dtype == np.float16 and Y.shape == ref.shape
    assert rel_err(Y, ref) < 1e-3
    Di = np.round(D.astype(np.float32) * 2).astype(np.float16)
    Gi = np.round(G.astype(np.float32) * 8).astype(np.float16)
    Yi = w.direct_conv2d_fwd(to_gpu(Di), to_gpu(Gi), pad=pad, stride=stride).cpu().numpy()
    refi = direct.conv2d_fwd(Di, Gi, pad=pad, stride=stride)
    assert np.abs(refi).max() <= 2048          # integers this small are exact in fp16
    assert np.array_equal(Yi.astype(np.float64), refi)


# ---- fp16 storage (D, G, U, V in fp16; fp32 accumulation; M and Y in fp32) -----------------------

@pytest.mark.parametrize("m", [2, 4])
@pytest.mark.parametrize("K,C", [(32, 32), (70, 19), (256, 128)])
def test_filter_transform_f16(m, K, C):
    torch, w = require_gpu()
    rng = np.random.default_rng(K + C + m)
    G = (rng.integers(-8, 9, (K, C, 3, 3)) * 4).astype(np.float16)
    U = w.wino_filter_transform(to_gpu(G), m)
    torch.cuda.synchronize()
    ref = wg.filter_transform(G.astype(np.float64), m)
    got = w.unpack_u(U, K, C, m, w.WINO_F16).astype(np.float64)
    if m == 2:
        assert np.array_equal(got, ref)                       # exact: entries are halves of small integers
    else:
        assert np.abs(got - ref).max() <= 2.0 ** -10 * np.abs(ref).max()   # one fp16 rounding
    full = w.unpack_u(U, K, C, m, w.WINO_F16, padded=True)
    assert not full[:, :, K:, :].any() and not full[:, :, :, C:].any()


@pytest.mark.parametrize("m", [2, 4])
@pytest.mark.parametrize("N,C,H,W,pad", [(2, 3, 14, 14, 1), (1, 2, 7, 9, 1), (2, 37, 9, 6, 0), (1, 17, 56, 56, 1)])
def test_input_transform_f16_bit_exact(m, N, C, H, W, pad):
    torch, w = require_gpu()
    rng = np.random.default_rng(H + W + m)
    D = rng.integers(-3, 4, (N, C, H, W)).astype(np.float16)    # |B^T d B| <= 300: exact in fp16
    V = w.wino_input_transform(to_gpu(D), pad, m)
    torch.cuda.synchronize()
    P = wg.num_tiles(N, H, W, pad, m)
    ref = wg.data_transform(D.astype(np.float64), pad, m)
    assert np.array_equal(w.unpack_v(V, C, P, m, w.WINO_F16).astype(np.float64), ref)
    full = w.unpack_v(V, C, P, m, w.WINO_F16, padded=True)
    assert not full[:, :, C:, :].any() and not full[:, :, :, P:].any()


@pytest.mark.parametrize("m", [2, 4])
@pytest.mark.parametrize("K,C,P", [(32, 32, 784), (70, 19, 100), (128, 48, 300), (256, 256, 130), (5, 3, 17)])
def test_batched_gemm_f16_exact_on_integers(m, K, C, P):
    torch, w = require_gpu()
    a = m + 2
    rng = np.random.default_rng(K + C + P + m)
    u = rng.integers(-4, 5, (a, a, K, C)).astype(np.float16)
    v = rng.integers(-4, 5, (a, a, C, P)).astype(np.float16)
    M = w.wino_batched_gemm(w.pack_u(u, m, w.WINO_F16), w.pack_v(v, m, w.WINO_F16), K, C, P, m)
    torch.cuda.synchronize()
    ref = wg.multiply(u.astype(np.float64), v.astype(np.float64))
    assert np.array_equal(w.unpack_m(M, K, P, m).astype(np.float64), ref)

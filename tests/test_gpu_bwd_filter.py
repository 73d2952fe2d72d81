"""GPU parity of the filter gradient (Section 4.2 of the paper, F(3x3,2x2) of Eq. (14)) against the
fp64 oracle written from Eq. (1).

Tolerance: every element of dG is a sum of N*H*W products accumulated in fp32; with the reduction cut
into shares and 32-deep MFMA chains the rounding error grows like sqrt(N*H*W) * 2^-24 relative to the
result in the worst case (1e-4 at 3.2 million terms), and the F(3,2) matrices (entries 0, +-1/2, +-1)
add a small constant factor.  Random rounding errors do far better than that worst case (4e-6 was
measured at 3.2 million terms, 4e-7 on the small shapes); the bounds asserted, normwise, are 2e-5 at
full size and 2e-6 for the small shapes."""
import numpy as np
import pytest

from oracle import direct
from paper_1509_09308_amd import synth
from gpu_util import require_gpu, rel_err, to_gpu

pytestmark = pytest.mark.gpu

TOL_SMALL, TOL_FULL = 2e-6, 2e-5


@pytest.mark.parametrize("shape", [(2, 16, 12, 12, 24), (1, 19, 13, 29, 70), (3, 33, 14, 14, 65), (1, 3, 9, 9, 8),
                                   (2, 64, 28, 28, 128), (1, 130, 7, 5, 140), (4, 8, 1, 1, 8), (1, 1, 2, 2, 1),
                                   (5, 40, 33, 31, 200),
                                   # W % 4 == 0 and at most 256 filters / channels: transforms inside the multiply
                                   (2, 19, 12, 16, 70), (1, 130, 8, 8, 140), (2, 5, 7, 8, 6), (1, 8, 2, 4, 8),
                                   (3, 64, 9, 20, 33), (1, 256, 6, 12, 200),
                                   # at most 4 channels and W % 4 == 0: the direct kernel
                                   (2, 3, 12, 16, 10), (3, 1, 8, 4, 5), (2, 4, 6, 8, 7), (1, 2, 5, 12, 3), (3, 3, 31, 36, 70)])
def test_bwd_filter_matches_oracle(shape):
    torch, w = require_gpu()
    N, C, H, W, K = shape
    rng = np.random.default_rng(sum(shape))
    D, _ = synth.make_layer(N, C, H, W, 1, seed=sum(shape) + 1)
    E = rng.standard_normal((N, K, H, W), dtype=np.float32)
    ref = direct.conv2d_bwd_filter(D, E, pad=1)
    dG = w.wino_conv2d_bwd_filter(to_gpu(D), to_gpu(E), pad=1).cpu().numpy()
    assert dG.shape == ref.shape
    err = rel_err(dG, ref)
    print("bwd-filter %s rel err %.3e" % (shape, err))
    assert err <= TOL_SMALL


@pytest.mark.parametrize("shape", [(2, 8, 16, 20, 12), (3, 5, 7, 9, 33), (1, 32, 15, 15, 32), (2, 3, 10, 12, 9)])
def test_bwd_filter_exact_on_integers(shape):
    """Integer inputs with E a multiple of 4: every transform value and every partial sum is an
    integer below 2^24, so the result must equal the oracle's bit for bit."""
    torch, w = require_gpu()
    N, C, H, W, K = shape
    rng = np.random.default_rng(sum(shape) + 5)
    D = rng.integers(-4, 5, (N, C, H, W)).astype(np.float32)
    E = (rng.integers(-3, 4, (N, K, H, W)) * 4).astype(np.float32)
    ref = direct.conv2d_bwd_filter(D, E, pad=1)
    dG = w.wino_conv2d_bwd_filter(to_gpu(D), to_gpu(E), pad=1).cpu().numpy()
    assert np.array_equal(dG.astype(np.float64), ref)


def test_bwd_filter_adjoint_identity_on_gpu_results():
    """<fwd(D, G), E> == <G, bwd_filter(D, E)> with both sides computed by the library (exact data)."""
    torch, w = require_gpu()
    D, G = synth.make_integer_layer(2, 8, 16, 20, 12, seed=31, gscale=4.0)
    E = (np.random.default_rng(32).integers(-3, 4, (2, 12, 16, 20)) * 4).astype(np.float32)
    Y = w.wino_conv2d_fwd_ex(to_gpu(D), G=to_gpu(G), pad=1, m=2).cpu().numpy().astype(np.float64)
    dG = w.wino_conv2d_bwd_filter(to_gpu(D), to_gpu(E), pad=1).cpu().numpy().astype(np.float64)
    assert float((Y * E).sum()) == float((G * dG).sum())


def test_bwd_filter_overwrites_output_and_reuses_workspace():
    """dG is overwritten (not accumulated into) and a dirty workspace does not leak into the result."""
    torch, w = require_gpu()
    N, C, H, W, K = 2, 24, 10, 14, 40
    rng = np.random.default_rng(9)
    D = rng.standard_normal((N, C, H, W), dtype=np.float32)
    E = rng.standard_normal((N, K, H, W), dtype=np.float32)
    ref = direct.conv2d_bwd_filter(D, E, pad=1)
    ws = torch.full((w.wino_bwd_filter_workspace_bytes(N, C, H, W, K),), 0x7f, dtype=torch.uint8, device="cuda")
    dG = torch.full((K, C, 3, 3), 1e30, device="cuda")
    for _ in range(2):
        w.wino_conv2d_bwd_filter(to_gpu(D), to_gpu(E), pad=1, dG=dG, workspace=ws)
        assert rel_err(dG.cpu().numpy(), ref) <= TOL_SMALL


def test_bwd_filter_rejections():
    torch, w = require_gpu()
    D = torch.zeros((1, 8, 6, 6), device="cuda")
    E = torch.zeros((1, 8, 6, 6), device="cuda")
    with pytest.raises(w.WinoError) as ei:
        w.wino_conv2d_bwd_filter(D, E, pad=0)
    assert ei.value.status == w.WINO_EUNSUPPORTED
    with pytest.raises(w.WinoError) as ei:
        w.wino_conv2d_bwd_filter(D.half(), E.half(), pad=1)
    assert ei.value.status == w.WINO_EUNSUPPORTED
    with pytest.raises(w.WinoError) as ei:
        w.wino_conv2d_bwd_filter(D, E, pad=1, workspace=torch.zeros(256, dtype=torch.uint8, device="cuda"))
    assert ei.value.status == w.WINO_EWORKSPACE


@pytest.mark.parametrize("layer", [0, 1, 5, 9, 12])
def test_bwd_filter_full_size_sampled(layer):
    """VGG-16 shapes at N=64, fp32: sampled elements of dG recomputed by the oracle."""
    torch, w = require_gpu()
    name, C, HW, K = synth.VGG16_LAYERS[layer]
    N = 64
    D, _ = synth.make_layer(N, C, HW, HW, 1, seed=synth.layer_seed(7, layer))
    rng = np.random.default_rng(synth.layer_seed(7, layer) + 1)
    E = rng.standard_normal((N, K, HW, HW), dtype=np.float32)
    dG = w.wino_conv2d_bwd_filter(to_gpu(D), to_gpu(E), pad=1)
    pts = synth.sample_points((K, C, 3, 3), 400, seed=layer)
    idx = torch.from_numpy(pts.astype(np.int64)).cuda()
    got = dG[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].cpu().numpy()
    ref = direct.conv2d_bwd_filter_points(D, E, pts, pad=1)
    err = rel_err(got, ref)
    print("%s N=64 bwd-filter sampled rel err %.3e" % (name, err))
    assert err <= TOL_FULL
    assert bool(torch.isfinite(dG).all())

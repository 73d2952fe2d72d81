"""GPU parity: the HIP path through the C ABI against the fp64 direct-convolution oracle on the
same seeded inputs.  Metric: normwise relative error ||Y^ - Y||_F / ||Y||_F; bounds: 1e-5 for
fp32 F(2x2,3x3), 1e-4 for fp32 F(4x4,3x3), 5e-3 for fp16 storage with fp32 accumulation."""
import numpy as np
import pytest

from oracle import direct
from paper_1509_09308_amd import synth
from gpu_util import TOL, check_close, require_gpu, rel_err, to_gpu

pytestmark = pytest.mark.gpu


def _run_full(w, D, G, pad, m, pre_transform=True):
    d, g = to_gpu(D), to_gpu(G)
    if pre_transform:
        U = w.wino_filter_transform(g, m)
        return w.wino_conv2d_fwd_ex(d, U=U, K=G.shape[0], pad=pad, m=m).cpu().numpy()
    return w.wino_conv2d_fwd_ex(d, G=g, pad=pad, m=m).cpu().numpy()


def test_config1_small_layer():
    """N=1, C=K=32, 56x56, fp32, F(2x2,3x3) only."""
    torch, w = require_gpu()
    D, G = synth.make_layer(1, 32, 56, 56, 32, synth.layer_seed(1, 0))
    ref = direct.conv2d_fwd(D, G, pad=1)
    for pre in (True, False):
        Y = _run_full(w, D, G, 1, 2, pre)
        check_close(Y, ref, TOL[("f32", 2)], "config 1, filters pre-transformed: %s" % pre, 2)
    Y = w.wino_conv2d_fwd(to_gpu(D), to_gpu(G), pad=1, m=2).cpu().numpy()
    check_close(Y, ref, TOL[("f32", 2)], "config 1, short entry point", 2)


@pytest.mark.parametrize("m", [2, 4, 6])
def test_config2_vgg_layer(m):
    """N=8, C=K=512, 28x28, fp32, both algorithms."""
    torch, w = require_gpu()
    D, G = synth.make_layer(8, 512, 28, 28, 512, synth.layer_seed(2, 0))
    ref = direct.conv2d_fwd(D, G, pad=1)
    Y = _run_full(w, D, G, 1, m)
    e, worst = check_close(Y, ref, TOL[("f32", m)], "config 2 m=%d" % m, m)
    print("config2 m=%d rel err %.3e max abs err %.3e" % (m, e, worst))


@pytest.mark.parametrize("m", [2, 4, 6])
@pytest.mark.parametrize("shape", [(1, 1, 3, 3, 1, 1), (1, 1, 4, 4, 1, 0), (2, 3, 5, 7, 4, 1), (1, 19, 13, 29, 70, 1),
                                   (3, 33, 14, 14, 65, 1), (2, 16, 31, 18, 130, 0), (5, 130, 9, 9, 40, 1),
                                   (1, 7, 67, 131, 9, 1)])
def test_ragged_and_degenerate_shapes(m, shape):
    """Odd extents, single-tile images, pad 0, channel and filter counts that do not fill a tile."""
    torch, w = require_gpu()
    N, C, H, W, K, pad = shape
    D, G = synth.make_layer(N, C, H, W, K, seed=sum(shape) + m)
    ref = direct.conv2d_fwd(D, G, pad=pad)
    Y = _run_full(w, D, G, pad, m)
    assert Y.shape == ref.shape
    e, worst = check_close(Y, ref, TOL[("f32", m)], "ragged %s m=%d" % (shape, m), m)
    print("ragged %s m=%d rel err %.3e max abs err %.3e" % (shape, m, e, worst))


@pytest.mark.parametrize("shape", [(1, 1024, 14, 14, 1024, 1), (2, 768, 9, 23, 40, 1), (1, 48, 7, 250, 1030, 0)])
def test_large_channel_counts_and_wide_images(shape):
    """More than 512 channels / filters (several filter blocks, long channel loops) and very wide, short images."""
    torch, w = require_gpu()
    N, C, H, W, K, pad = shape
    D, G = synth.make_layer(N, C, H, W, K, seed=sum(shape))
    ref = direct.conv2d_fwd(D, G, pad=pad)
    for m in (2, 4, 6):
        e = rel_err(_run_full(w, D, G, pad, m), ref)
        print("large %s m=%d rel err %.3e" % (shape, m, e))
        assert e <= TOL[("f32", m)]
    if pad == 1:
        E = np.random.default_rng(1).standard_normal((N, K, H, W), dtype=np.float32)
        dD = w.wino_conv2d_bwd_data(to_gpu(E), G=to_gpu(G), pad=1, m=4).cpu().numpy()
        assert rel_err(dD, direct.conv2d_bwd_data(E, G, H, W, pad=1)) <= TOL[("f32", 4)]
        dG = w.wino_conv2d_bwd_filter(to_gpu(D), to_gpu(E), pad=1).cpu().numpy()
        assert rel_err(dG, direct.conv2d_bwd_filter(D, E, pad=1)) <= 2e-6


@pytest.mark.parametrize("layer", range(1, 13))
def test_config3_vgg16_stack_n1(layer):
    """Every Winograd-eligible VGG-16 layer at N=1, fp32, both algorithms, whole output."""
    torch, w = require_gpu()
    name, C, HW, K = synth.VGG16_LAYERS[layer]
    D, G = synth.make_layer(1, C, HW, HW, K, synth.layer_seed(3, layer))
    ref = direct.conv2d_fwd(D, G, pad=1)
    for m in (2, 4):
        e, worst = check_close(_run_full(w, D, G, 1, m), ref, TOL[("f32", m)], "%s N=1 m=%d" % (name, m), m)
        print("%s m=%d rel err %.3e max abs err %.3e" % (name, m, e, worst))


def test_config3_first_layer_direct():
    torch, w = require_gpu()
    name, C, HW, K = synth.VGG16_LAYERS[0]
    D, G = synth.make_layer(1, C, HW, HW, K, synth.layer_seed(3, 0))
    ref = direct.conv2d_fwd(D, G, pad=1)
    Y = w.direct_conv2d_fwd(to_gpu(D), to_gpu(G), pad=1).cpu().numpy()
    check_close(Y, ref, 1e-5, "conv1.1 N=1 direct")


def _sampled_check(torch, Y, D, G, pts, tol, what, m=1):
    """Outputs of the GPU tensor Y at ``pts`` against the oracle's one-by-one values: normwise and element-wise."""
    idx = torch.from_numpy(pts.astype(np.int64)).cuda()
    got = Y[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].float().cpu().numpy()
    ref = direct.conv2d_points(D, G, pts, pad=1)
    e, worst = check_close(got, ref, tol, what, m)
    print("%s: %d sampled outputs, rel err %.3e, max abs err %.3e" % (what, len(pts), e, worst))
    assert bool(torch.isfinite(Y).all())


@pytest.mark.parametrize("layer", range(13))
def test_config4_full_size_sampled(layer):
    """N=64 fp32, every layer of the stack, exactly as the benchmark step launches it (untransformed
    filters, caller workspace, the library's own choice of variant; F(4x4) where 4 divides the image,
    F(2x2) for 14x14; conv1.1 through the direct kernel): outputs sampled at random, at the tensor
    corners and over the whole last tile row and column of a few (image, filter) planes are recomputed
    one by one by the oracle."""
    torch, w = require_gpu()
    name, C, HW, K = synth.VGG16_LAYERS[layer]
    N = 64
    D, G = synth.make_layer(N, C, HW, HW, K, synth.layer_seed(4, layer))
    d, g = to_gpu(D), to_gpu(G)
    if C < 16:
        Y = w.direct_conv2d_fwd(d, g, pad=1)
        m, tol, what = 1, 1e-5, "%s N=64 direct" % name
    else:
        m = 4 if HW % 4 == 0 else 2
        ws = w.alloc_workspace(N, C, HW, HW, K, 1, m)
        Y = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=m, workspace=ws)
        variant = w.wino_conv2d_variant(N, C, HW, HW, K, 1, m)
        tol, what = TOL[("f32", m)], "%s N=64 m=%d variant %d" % (name, m, variant)
    pts = synth.sample_points((N, K, HW, HW), 4000, seed=layer, edge=max(m, 2))
    _sampled_check(torch, Y, D, G, pts, tol, what, m)


@pytest.mark.parametrize("layer", [1, 2, 3, 6, 9, 12])
def test_config4_full_size_sampled_pretransformed_filters(layer):
    """The same layers with the filter transform taken out of the call (Section 6, "FX": U is computed once by
    wino_filter_transform and passed in), which for the layers with few filters selects the other one-kernel
    design."""
    torch, w = require_gpu()
    name, C, HW, K = synth.VGG16_LAYERS[layer]
    N = 64
    m = 4 if HW % 4 == 0 else 2
    D, G = synth.make_layer(N, C, HW, HW, K, synth.layer_seed(4, layer))
    d, g = to_gpu(D), to_gpu(G)
    U = w.wino_filter_transform(g, m)
    ws = w.alloc_workspace(N, C, HW, HW, K, 1, m)
    Y = w.wino_conv2d_fwd_ex(d, U=U, K=K, pad=1, m=m, workspace=ws)
    pts = synth.sample_points((N, K, HW, HW), 4000, seed=100 + layer, edge=m)
    _sampled_check(torch, Y, D, G, pts, TOL[("f32", m)], "%s N=64 m=%d, U given" % (name, m), m)


def test_f4x4_on_14x14_full_size_sampled():
    """The all-F(4x4,3x3) line of the benchmark: conv5.3 at N=64 with 4 x 4 tiles on a 14 x 14 image (the last
    tile row and column reach two outputs past the image)."""
    torch, w = require_gpu()
    name, C, HW, K = synth.VGG16_LAYERS[12]
    N, m = 64, 4
    D, G = synth.make_layer(N, C, HW, HW, K, synth.layer_seed(4, 12))
    ws = w.alloc_workspace(N, C, HW, HW, K, 1, m)
    Y = w.wino_conv2d_fwd_ex(to_gpu(D), G=to_gpu(G), pad=1, m=m, workspace=ws)
    pts = synth.sample_points((N, K, HW, HW), 4000, seed=12, edge=m)
    _sampled_check(torch, Y, D, G, pts, TOL[("f32", 4)], "%s N=64 m=4" % name, 4)


@pytest.mark.parametrize("layer", [3, 5, 9])
def test_f6x6_full_size_sampled(layer):
    """F(6x6,3x3) at N=64 on VGG shapes whose images 6 does not divide (edge tiles zero-filled)."""
    torch, w = require_gpu()
    name, C, HW, K = synth.VGG16_LAYERS[layer]
    N, m = 64, 6
    D, G = synth.make_layer(N, C, HW, HW, K, synth.layer_seed(8, layer))
    d, g = to_gpu(D), to_gpu(G)
    ws = w.alloc_workspace(N, C, HW, HW, K, 1, m)
    Y = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=m, workspace=ws)
    pts = synth.sample_points((N, K, HW, HW), 4000, seed=layer, edge=m)
    _sampled_check(torch, Y, D, G, pts, TOL[("f32", 6)], "%s N=64 m=6" % name, 6)


def test_f6x6_rejects_f16_storage():
    torch, w = require_gpu()
    D = torch.zeros((1, 8, 12, 12), device="cuda", dtype=torch.float16)
    G = torch.zeros((8, 8, 3, 3), device="cuda", dtype=torch.float16)
    with pytest.raises(w.WinoError) as ei:
        w.wino_conv2d_fwd_ex(D, G=G, pad=1, m=6)
    assert ei.value.status == w.WINO_EUNSUPPORTED


# ---- fp16 storage of D, G, U, V; fp32 accumulation; fp32 Y (config 5) ----------------------------

@pytest.mark.parametrize("m", [2, 4])
@pytest.mark.parametrize("shape", [(2, 32, 28, 28, 48, 1), (1, 19, 13, 29, 70, 1), (3, 130, 14, 14, 65, 1),
                                   (2, 16, 31, 18, 130, 0), (1, 512, 14, 14, 512, 1)])
def test_f16_storage_layers(m, shape):
    torch, w = require_gpu()
    N, C, H, W, K, pad = shape
    D, G = synth.make_layer(N, C, H, W, K, seed=sum(shape) + m, dtype=np.float16)
    ref = direct.conv2d_fwd(D, G, pad=pad)            # the oracle reads the same stored fp16 values
    d, g = to_gpu(D), to_gpu(G)
    Y = w.wino_conv2d_fwd_ex(d, G=g, pad=pad, m=m)
    assert Y.dtype == torch.float32
    e, worst = check_close(Y.cpu().numpy(), ref, TOL[("f16", m)], "fp16 %s m=%d" % (shape, m), m)
    print("fp16 %s m=%d rel err %.3e max abs err %.3e" % (shape, m, e, worst))


@pytest.mark.parametrize("shape", [(2, 32, 28, 28, 48), (1, 19, 13, 28, 70), (3, 130, 14, 16, 65), (2, 16, 31, 20, 130),
                                   (1, 8, 4, 4, 8), (2, 64, 56, 56, 64), (1, 3, 17, 12, 5)])
def test_f16_fused_path_matches_oracle(shape):
    """fp16 storage, loops 2-4 in one kernel: ragged heights, channel and filter counts that do not fill
    a step or a block, tiles past the end of the last block."""
    torch, w = require_gpu()
    N, C, H, W, K = shape
    D, G = synth.make_layer(N, C, H, W, K, seed=sum(shape), dtype=np.float16)
    ref = direct.conv2d_fwd(D, G, pad=1)
    d, g = to_gpu(D), to_gpu(G)
    assert w.wino_conv2d_variant(N, C, H, W, K, 1, 4, w.WINO_F16, flags=w.FLAG_FUSED) == w.FLAG_FUSED
    Yf = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=4, flags=w.FLAG_FUSED).cpu().numpy()
    Yu = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=4, flags=w.FLAG_UNFUSED).cpu().numpy()
    e, worst = check_close(Yf, ref, TOL[("f16", 4)], "fp16 fused %s" % (shape,), 4)
    print("fp16 fused %s rel err %.3e (unfused %.3e) max abs err %.3e" % (shape, e, rel_err(Yu, ref), worst))
    # same fp16 operands, same fp32 accumulation: the two paths differ only in summation order
    assert rel_err(Yf, Yu) <= 5e-4   # v = B^T (d B) here, (B^T d) B there: an fp16 rounding of V can flip


@pytest.mark.parametrize("shape", [(2, 32, 28, 28, 48), (1, 19, 13, 28, 70), (2, 64, 56, 56, 64), (1, 8, 6, 8, 16)])
def test_f16_fused_path_writes_fp16_outputs(shape):
    """fp16 Y from the one-kernel path: the fp32 result of the same path, rounded once."""
    torch, w = require_gpu()
    N, C, H, W, K = shape
    D, G = synth.make_layer(N, C, H, W, K, seed=sum(shape) + 5, dtype=np.float16)
    d, g = to_gpu(D), to_gpu(G)
    assert w.wino_conv2d_variant(N, C, H, W, K, 1, 4, w.WINO_F16, y_dt=w.WINO_F16, flags=w.FLAG_FUSED) == w.FLAG_FUSED
    Y32 = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=4, flags=w.FLAG_FUSED)
    Y16 = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=4, flags=w.FLAG_FUSED, y_dtype=torch.float16)
    assert Y16.dtype == torch.float16
    # (the two instantiations may contract the inverse transform's multiply-adds differently: within half an
    # fp16 unit of the fp32 result, not necessarily the identical rounding)
    assert torch.allclose(Y16.float(), Y32, rtol=6e-4, atol=1e-4)
    check_close(Y16.float().cpu().numpy(), direct.conv2d_fwd(D, G, pad=1), TOL[("f16", 4)], "fp16 fused, fp16 Y %s" % (shape,), 4)


def test_f16_fused_exact_on_integers():
    """Small integers and filters scaled by 576 / 4: every fp16 rounding is exact except those of the
    1/6-type constants; every output position must be the right one."""
    torch, w = require_gpu()
    D, G = synth.make_integer_layer(3, 8, 22, 24, 70, seed=9, gscale=144.0, dmax=3, gmax=1)
    D16, G16 = D.astype(np.float16), G.astype(np.float16)
    ref = direct.conv2d_fwd(D16, G16, pad=1)
    Yf = w.wino_conv2d_fwd_ex(to_gpu(D16), G=to_gpu(G16), pad=1, m=4, flags=w.FLAG_FUSED).cpu().numpy()
    e = rel_err(Yf, ref)
    print("fp16 fused integer layer rel err %.3e" % e)
    assert e < 1e-6


@pytest.mark.parametrize("layer", range(13))
def test_config5_full_size_sampled(layer):
    """N=32, fp16 storage, every layer as the benchmark launches it: F(4x4,3x3) everywhere (ragged at 14x14),
    conv1.1 through the direct kernel; the oracle reads the same stored fp16 values."""
    torch, w = require_gpu()
    name, C, HW, K = synth.VGG16_LAYERS[layer]
    N, m = 32, 4
    D, G = synth.make_layer(N, C, HW, HW, K, synth.layer_seed(5, layer), dtype=np.float16)
    d, g = to_gpu(D), to_gpu(G)
    mm = m
    if C < 16:
        Y = w.direct_conv2d_fwd(d, g, pad=1)
        what, mm = "%s N=32 fp16 direct" % name, 1
    else:
        ws = w.alloc_workspace(N, C, HW, HW, K, 1, m, w.WINO_F16)
        Y = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=m, workspace=ws)
        what = "%s N=32 fp16 m=4 variant %d" % (name, w.wino_conv2d_variant(N, C, HW, HW, K, 1, m, w.WINO_F16))
    pts = synth.sample_points((N, K, HW, HW), 4000, seed=layer, edge=m)
    _sampled_check(torch, Y, D.astype(np.float32), G.astype(np.float32), pts, TOL[("f16", 4)], what, mm)


# ---- the one-kernel path (gather + data transform + multiply + inverse transform fused) ----------

@pytest.mark.parametrize("shape", [(2, 16, 8, 8, 16, 1), (1, 4, 12, 12, 8, 1), (2, 64, 28, 28, 64, 1),
                                   (1, 19, 13, 29, 70, 1), (3, 33, 14, 14, 65, 1), (2, 16, 31, 18, 130, 0),
                                   (1, 7, 67, 131, 9, 1), (1, 1, 3, 3, 1, 1), (1, 1, 4, 4, 1, 0), (5, 130, 9, 9, 40, 1),
                                   (8, 512, 28, 28, 512, 1),
                                   # 64 filters per workgroup (W % 4 == 0, more than 32 filters): ragged filter block,
                                   # channels not a multiple of 16, tile count not a multiple of 16, several images
                                   # per tile block, 8 x 4 filter blocks in XCD groups
                                   (3, 40, 12, 20, 96, 1), (2, 24, 8, 8, 200, 1), (1, 130, 20, 36, 70, 1),
                                   (5, 16, 4, 4, 64, 1), (2, 272, 16, 16, 256, 1)])
def test_fused_path_matches_oracle(shape):
    """F(4x4,3x3) with V and M kept on chip: whole output against the oracle, including ragged
    edges, pad 0, channel counts that are not multiples of 4 and filter counts below a block."""
    torch, w = require_gpu()
    N, C, H, W, K, pad = shape
    D, G = synth.make_layer(N, C, H, W, K, seed=sum(shape) + 40)
    ref = direct.conv2d_fwd(D, G, pad=pad)
    Y = w.wino_conv2d_fwd_ex(to_gpu(D), G=to_gpu(G), pad=pad, m=4, flags=w.FLAG_FUSED).cpu().numpy()
    assert Y.shape == ref.shape
    e, worst = check_close(Y, ref, TOL[("f32", 4)], "fused %s" % (shape,), 4)
    print("fused %s rel err %.3e max abs err %.3e" % (shape, e, worst))


@pytest.mark.parametrize("shape", [(2, 256, 96, 96, 512),    # 72 items per XCD: a last round of 8 items in 8 shares
                                   (2, 344, 96, 96, 512),    # channels not a multiple of 16: 22 steps, 2 shares
                                   (6, 256, 72, 72, 320)])   # lists of 77 and 71 items (4 and 8 shares), ragged last tile block
def test_fused_path_shares_the_items_of_a_partly_filled_last_round(shape):
    """Layers with at least 512 (tile block, filter block) items whose last round fills only part of the resident
    workgroups: the channel steps of those items are shared between workgroups that hand partial outputs over
    through the workspace.  Whole output against the oracle; a second call must reproduce the first bit for bit
    (the partial outputs are added in share order, whichever share arrives last)."""
    torch, w = require_gpu()
    N, C, H, W, K = shape
    D, G = synth.make_layer(N, C, H, W, K, seed=sum(shape) + 41)
    ref = direct.conv2d_fwd(D, G, pad=1)
    d, g = to_gpu(D), to_gpu(G)
    ws = w.alloc_workspace(N, C, H, W, K, 1, 4)
    ws.view(torch.float32).fill_(float("nan"))            # nothing may depend on what the workspace held
    Y1 = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=4, flags=w.FLAG_FUSED, workspace=ws)
    Y2 = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=4, flags=w.FLAG_FUSED, workspace=ws)
    torch.cuda.synchronize()
    e, worst = check_close(Y1.cpu().numpy(), ref, TOL[("f32", 4)], "fused with shares %s" % (shape,), 4)
    assert torch.equal(Y1, Y2)
    print("fused with shares %s rel err %.3e max abs err %.3e" % (shape, e, worst))


@pytest.mark.parametrize("shape", [(3, 40, 12, 20, 96), (2, 24, 8, 8, 200), (1, 130, 20, 36, 70), (5, 16, 4, 4, 64),
                                   (2, 272, 16, 16, 256),
                                   (2, 16, 10, 14, 64), (1, 20, 7, 6, 40), (1, 3, 5, 2, 33),     # widths that 4 does not divide
                                   (3, 256, 40, 40, 512), (2, 256, 66, 66, 512)])              # a shared last round (4 shares)
def test_fused_f2x2_path_matches_oracle(shape):
    """F(2x2,3x3) in one kernel (the 64-filter design with 4 x 4 tiles: 16 components, 8-byte rows): whole output
    against the oracle; the call repeated must give the same bits."""
    torch, w = require_gpu()
    N, C, H, W, K = shape
    D, G = synth.make_layer(N, C, H, W, K, seed=sum(shape) + 42)
    ref = direct.conv2d_fwd(D, G, pad=1)
    d, g = to_gpu(D), to_gpu(G)
    assert w.wino_conv2d_variant(N, C, H, W, K, 1, 2, flags=w.FLAG_FUSED) == w.FLAG_FUSED
    ws = w.alloc_workspace(N, C, H, W, K, 1, 2)
    ws.view(torch.float32).fill_(float("nan"))
    Y1 = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=2, flags=w.FLAG_FUSED, workspace=ws)
    Y2 = w.wino_conv2d_fwd_ex(d, U=w.wino_filter_transform(g, 2), K=K, pad=1, m=2, flags=w.FLAG_FUSED, workspace=ws)
    torch.cuda.synchronize()
    assert Y1.shape == ref.shape
    e, worst = check_close(Y1.cpu().numpy(), ref, TOL[("f32", 2)], "fused F(2x2) %s" % (shape,), 2)
    assert torch.equal(Y1, Y2)
    print("fused F(2x2) %s rel err %.3e max abs err %.3e" % (shape, e, worst))


def test_fused_f2x2_delta_filter_bitwise_and_full_size_sampled():
    """With a centre-one filter every intermediate of F(2x2) is exact in fp32: the one-kernel path must return D bit
    for bit (every tile, row and column in its place).  And conv5.x of the N=64 stack through this path (the shape it
    is chosen for: 3 full rounds and a shared one), sampled against the oracle."""
    torch, w = require_gpu()
    N, C, H, W, K = 3, 72, 14, 22, 72
    D = (np.arange(N * C * H * W, dtype=np.float32) % 65521).reshape(N, C, H, W)
    np.random.default_rng(1).shuffle(D.reshape(-1))
    G = np.zeros((K, C, 3, 3), dtype=np.float32)
    G[np.arange(K), np.arange(C), 1, 1] = 1.0
    Y = w.wino_conv2d_fwd_ex(to_gpu(D), G=to_gpu(G), pad=1, m=2, flags=w.FLAG_FUSED)
    torch.cuda.synchronize()
    assert np.array_equal(Y.cpu().numpy(), D)
    name, C, HW, K = synth.VGG16_LAYERS[12]
    N = 64
    D, G = synth.make_layer(N, C, HW, HW, K, synth.layer_seed(4, 12))
    Y = w.wino_conv2d_fwd_ex(to_gpu(D), G=to_gpu(G), pad=1, m=2, flags=w.FLAG_FUSED)
    pts = synth.sample_points((N, K, HW, HW), 4000, seed=12, edge=2)
    _sampled_check(torch, Y, D, G, pts, TOL[("f32", 2)], "%s N=64 F(2x2) in one kernel" % name, 2)


def test_fused_path_exact_on_integers_and_equals_unfused_bookkeeping():
    """Integer data and filters scaled by 576: the only roundings are those of the 1/6-type
    constants, and every output position must be the right one (distinct values per pixel)."""
    torch, w = require_gpu()
    D, G = synth.make_integer_layer(3, 8, 22, 26, 70, seed=9, gscale=576.0)
    ref = direct.conv2d_fwd(D, G, pad=1)
    d, g = to_gpu(D), to_gpu(G)
    Yf = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=4, flags=w.FLAG_FUSED).cpu().numpy()
    Yu = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=4, flags=w.FLAG_UNFUSED).cpu().numpy()
    assert rel_err(Yf, ref) < 1e-6 and rel_err(Yu, ref) < 1e-6
    assert np.abs(Yf - Yu).max() <= 1e-5 * np.abs(ref).max()


@pytest.mark.parametrize("C", [8, 24, 3, 16])
@pytest.mark.parametrize("given", ["G", "U"])
def test_fused_path_never_uses_memory_behind_the_input(C, given):
    """The channel loop of the one-kernel path runs over the padded channel count: channels past C must come
    in as zeros, not from whatever follows the input in memory.  D ends where a block of NaNs begins (0 * NaN
    would poison the sums of the last image); both one-kernel designs (untransformed filters / U given)."""
    torch, w = require_gpu()
    N, H, W, K = 2, 12, 16, 40
    D, G = synth.make_layer(N, C, H, W, K, seed=77 + C)
    ref = direct.conv2d_fwd(D, G, pad=1)
    n = D.size
    buf = torch.full((n + 64 * H * W,), float("nan"), dtype=torch.float32, device="cuda")
    buf[:n] = to_gpu(D).reshape(-1)
    d = buf[:n].view(N, C, H, W)
    g = to_gpu(G)
    if given == "G":
        Y = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=4, flags=w.FLAG_FUSED)
    else:
        Y = w.wino_conv2d_fwd_ex(d, U=w.wino_filter_transform(g, 4), K=K, pad=1, m=4, flags=w.FLAG_FUSED)
    assert bool(torch.isfinite(Y).all())
    check_close(Y.cpu().numpy(), ref, TOL[("f32", 4)], "C=%d, %s given" % (C, given), 4)


def test_fused_flag_rejected_where_unsupported():
    torch, w = require_gpu()
    D, G = synth.make_layer(1, 8, 8, 8, 8, seed=1)
    with pytest.raises(w.WinoError) as ei:
        w.wino_conv2d_fwd_ex(to_gpu(D), G=to_gpu(G), pad=1, m=2, flags=w.FLAG_FUSED)
    assert ei.value.status == w.WINO_EUNSUPPORTED
    # fp16 storage: the one-kernel path needs m = 4, pad = 1 and W % 4 == 0
    d16, g16 = to_gpu(D.astype(np.float16)), to_gpu(G.astype(np.float16))
    for kw in (dict(pad=1, m=2), dict(pad=0, m=4)):
        with pytest.raises(w.WinoError) as ei:
            w.wino_conv2d_fwd_ex(d16, G=g16, flags=w.FLAG_FUSED, **kw)
        assert ei.value.status == w.WINO_EUNSUPPORTED
    D2, G2 = synth.make_layer(1, 8, 8, 10, 8, seed=2, dtype=np.float16)
    with pytest.raises(w.WinoError) as ei:
        w.wino_conv2d_fwd_ex(to_gpu(D2), G=to_gpu(G2), pad=1, m=4, flags=w.FLAG_FUSED)
    assert ei.value.status == w.WINO_EUNSUPPORTED


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("pos", [(0, 0), (3, 27), (4, 0), (7, 28), (11, 55), (12, 31), (15, 32)])
def test_one_kernel_path_keeps_a_nan_inside_the_tiles_that_read_it(dtype, pos):
    """The one-kernel kernels take a tile's outer columns from the registers of the neighbouring lanes, which hold
    the neighbouring tiles -- or, at the image border, the last tile of the tile row above resp. the first of the
    one below, whose values must not be used.  One NaN in the input must reach exactly the outputs of the tiles
    whose 6 x 6 window (rows 4 tx - 1 .. 4 tx + 4, columns 4 ty - 1 .. 4 ty + 4) holds it, in the image that has
    it: a value leaking over from a neighbouring lane would poison a tile outside that set.  Within such a tile
    the first window row (column) enters only the first transformed component (B^T of Eq. (15) has (4, 0, ...) as
    its first column), which feeds only the first output row (column); the last one likewise only the last."""
    torch, w = require_gpu()
    N, C, H, W, K = 2, 16, 16, 56, 64          # 14 tiles per row: blocks of 16 (or 32) lanes straddle tile rows
    np_dt = np.float32 if dtype == "f32" else np.float16
    D, G = synth.make_layer(N, C, H, W, K, seed=4242, dtype=np_dt)
    x, y = pos
    D[1, 5, x, y] = np.nan
    Y = w.wino_conv2d_fwd_ex(to_gpu(D), G=to_gpu(G), pad=1, m=4, flags=w.FLAG_FUSED).float().cpu().numpy()
    want = np.zeros((N, H, W), dtype=bool)
    def reached(t, z):          # outputs of tile t along one axis that a NaN at coordinate z of that axis reaches
        q = z - (4 * t - 1)
        return [] if q < 0 or q > 5 else [4 * t] if q == 0 else [4 * t + 3] if q == 5 else list(range(4 * t, 4 * t + 4))
    for tx in range(H // 4):
        for ty in range(W // 4):
            for ox in reached(tx, x):
                for oy in reached(ty, y):
                    want[1, ox, oy] = True
    got = np.isnan(Y)
    assert (got == want[:, None, :, :]).all(), "NaN outputs %d, expected %d" % (got.sum(), want.sum() * K)

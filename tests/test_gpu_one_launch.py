"""GPU parity of the one-launch F(2x2,3x3) layer (all four loops of Algorithm 1 in one kernel, filter
transform inside; Section 6 of the paper, the variant without separately transformed filters)
against the fp64 direct-convolution oracle of Eq. (1).  Bound: 1e-5 normwise, as for every fp32
F(2x2,3x3) path.  Shapes are chosen so that the channel loop runs unsplit, split evenly, and split
with a shorter last share; tile rows and columns fall on, below and above the edges of the 8 x 8 tile blocks."""
import numpy as np
import pytest

from oracle import direct
from paper_1509_09308_amd import synth
from gpu_util import TOL, require_gpu, rel_err, to_gpu

pytestmark = pytest.mark.gpu

SHAPES = [
    (1, 1, 3, 3, 1, 1),          # one tile, one channel, one filter
    (1, 1, 4, 4, 1, 0),
    (2, 3, 5, 7, 4, 1),          # odd extents: half-empty edge tiles
    (1, 19, 13, 29, 70, 1),      # 3 filter blocks, channel steps 8 + 8 + 3
    (3, 33, 14, 14, 65, 1),      # 7 x 7 tiles per image: one partly filled block each; last step moved back
    (2, 16, 31, 18, 130, 0),
    (5, 130, 9, 9, 40, 1),       # 17 steps shared by many workgroups, last share shorter
    (1, 7, 67, 131, 9, 1),       # many tile blocks: the channel loop stays in one workgroup
    (2, 64, 8, 8, 32, 1),        # 4 x 4 tiles: the second MFMA column block holds no tile
    (1, 64, 16, 16, 32, 1),      # 8 x 8 tiles exactly
    (1, 40, 18, 16, 32, 1),      # 9 x 8 tiles: a full block and one with a single tile row
    (1, 512, 14, 14, 512, 1),    # conv5 of Table 3 at batch 1
    (1, 256, 28, 28, 512, 1),    # conv4.1
]


def _one_launch(w, D, G, pad):
    return w.wino_conv2d_fwd_ex(to_gpu(D), G=to_gpu(G), pad=pad, m=2, flags=w.FLAG_ONE_LAUNCH)


@pytest.mark.parametrize("shape", SHAPES)
def test_one_launch_matches_oracle(shape):
    torch, w = require_gpu()
    N, C, H, W, K, pad = shape
    D, G = synth.make_layer(N, C, H, W, K, seed=sum(shape) + 2)
    ref = direct.conv2d_fwd(D, G, pad=pad)
    assert w.wino_conv2d_variant(N, C, H, W, K, pad, 2, flags=w.FLAG_ONE_LAUNCH) == w.FLAG_ONE_LAUNCH
    Y = _one_launch(w, D, G, pad).cpu().numpy()
    assert Y.shape == ref.shape
    e = rel_err(Y, ref)
    print("one launch %s rel err %.3e" % (shape, e))
    assert e <= TOL[("f32", 2)]


def test_one_launch_exact_on_integer_data():
    """Small integers: every product and sum of F(2x2,3x3) is exact in fp32 (the halves of G are
    absorbed by filters that are multiples of 4), so the result must equal the oracle bit for bit,
    whatever the number of channel shares."""
    torch, w = require_gpu()
    for shape in [(2, 24, 10, 12, 40), (1, 128, 14, 14, 64)]:
        N, C, H, W, K = shape
        D, G = synth.make_integer_layer(N, C, H, W, K, seed=sum(shape), gscale=4.0)
        ref = direct.conv2d_fwd(D, G, pad=1)
        Y = _one_launch(w, D, G, 1).cpu().numpy()
        assert np.array_equal(Y.astype(np.float64), ref)


def test_one_launch_repeats_bit_for_bit():
    """The partial outputs of the channel shares are added in the order of the shares, not of arrival,
    and the arrival counters are back at zero after every call: repeated calls, with calls of other
    shapes in between, give identical bits."""
    torch, w = require_gpu()
    D, G = synth.make_layer(1, 512, 14, 14, 512, seed=77)
    D2, G2 = synth.make_layer(2, 72, 12, 20, 96, seed=78)
    d, g, d2, g2 = to_gpu(D), to_gpu(G), to_gpu(D2), to_gpu(G2)
    ws = w.alloc_workspace(2, 512, 14, 20, 512, 1, 2)
    first = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=2, workspace=ws, flags=w.FLAG_ONE_LAUNCH).clone()
    first2 = w.wino_conv2d_fwd_ex(d2, G=g2, pad=1, m=2, workspace=ws, flags=w.FLAG_ONE_LAUNCH).clone()
    for _ in range(5):
        again = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=2, workspace=ws, flags=w.FLAG_ONE_LAUNCH)
        again2 = w.wino_conv2d_fwd_ex(d2, G=g2, pad=1, m=2, workspace=ws, flags=w.FLAG_ONE_LAUNCH)
        assert torch.equal(first, again) and torch.equal(first2, again2)
    assert rel_err(first.cpu().numpy(), direct.conv2d_fwd(D, G, pad=1)) <= TOL[("f32", 2)]
    assert rel_err(first2.cpu().numpy(), direct.conv2d_fwd(D2, G2, pad=1)) <= TOL[("f32", 2)]


def test_one_launch_partial_outputs_are_fresh():
    """Two different inputs of one shape alternate through the same workspace: a share that read a
    partial output of the previous call (same address, other values) would change the result."""
    torch, w = require_gpu()
    shape = (1, 256, 14, 14, 96)
    Da, Ga = synth.make_layer(*shape, seed=301)
    Db, Gb = synth.make_layer(*shape, seed=302)
    da, ga, db, gb = to_gpu(Da), to_gpu(Ga), to_gpu(Db), to_gpu(Gb)
    ws = w.alloc_workspace(1, 256, 14, 14, 96, 1, 2)
    Ya = w.wino_conv2d_fwd_ex(da, G=ga, pad=1, m=2, workspace=ws, flags=w.FLAG_ONE_LAUNCH).clone()
    Yb = w.wino_conv2d_fwd_ex(db, G=gb, pad=1, m=2, workspace=ws, flags=w.FLAG_ONE_LAUNCH).clone()
    assert rel_err(Ya.cpu().numpy(), direct.conv2d_fwd(Da, Ga, pad=1)) <= TOL[("f32", 2)]
    assert rel_err(Yb.cpu().numpy(), direct.conv2d_fwd(Db, Gb, pad=1)) <= TOL[("f32", 2)]
    for _ in range(20):
        assert torch.equal(Ya, w.wino_conv2d_fwd_ex(da, G=ga, pad=1, m=2, workspace=ws, flags=w.FLAG_ONE_LAUNCH))
        assert torch.equal(Yb, w.wino_conv2d_fwd_ex(db, G=gb, pad=1, m=2, workspace=ws, flags=w.FLAG_ONE_LAUNCH))


def test_one_launch_agrees_with_staged_path():
    """Same algorithm, same fp32 transforms: the one-launch result and the four-stage result differ
    only by the order of the channel sum."""
    torch, w = require_gpu()
    D, G = synth.make_layer(2, 96, 20, 24, 64, seed=5)
    d, g = to_gpu(D), to_gpu(G)
    Y1 = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=2, flags=w.FLAG_ONE_LAUNCH).cpu().numpy()
    Y4 = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=2, flags=w.FLAG_UNFUSED).cpu().numpy()
    assert rel_err(Y1, Y4) <= 2e-6


@pytest.mark.parametrize("layer", [1, 2, 4, 6, 9, 12])
def test_one_launch_vgg_stack_n1(layer):
    """The launch configuration the batch-1 benchmark line uses: VGG-16 layers at N = 1, whole output."""
    torch, w = require_gpu()
    name, C, HW, K = synth.VGG16_LAYERS[layer]
    D, G = synth.make_layer(1, C, HW, HW, K, synth.layer_seed(9, layer))
    ref = direct.conv2d_fwd(D, G, pad=1)
    ws = w.alloc_workspace(1, C, HW, HW, K, 1, 2)
    Y = w.wino_conv2d_fwd_ex(to_gpu(D), G=to_gpu(G), pad=1, m=2, workspace=ws, flags=w.FLAG_ONE_LAUNCH)
    e = rel_err(Y.cpu().numpy(), ref)
    print("%s N=1 one launch rel err %.3e" % (name, e))
    assert e <= TOL[("f32", 2)]


@pytest.mark.parametrize("shape", [(2, 16, 12, 12, 24), (1, 19, 13, 29, 70), (1, 128, 14, 14, 256)])
def test_one_launch_input_gradient(shape):
    """Section 4.2: the same kernel on the error tensor, reading the stored filters transposed and
    rotated by 180 degrees."""
    torch, w = require_gpu()
    N, C, H, W, K = shape
    rng = np.random.default_rng(sum(shape))
    E = rng.standard_normal((N, K, H, W), dtype=np.float32)
    _, G = synth.make_layer(1, C, 4, 4, K, seed=sum(shape))
    ref = direct.conv2d_bwd_data(E, G, H, W, pad=1)
    dD = w.wino_conv2d_bwd_data(to_gpu(E), G=to_gpu(G), pad=1, m=2, flags=w.FLAG_ONE_LAUNCH).cpu().numpy()
    assert dD.shape == ref.shape
    assert rel_err(dD, ref) <= TOL[("f32", 2)]


def test_one_launch_rejections():
    torch, w = require_gpu()
    D = torch.zeros((1, 8, 12, 12), device="cuda")
    G = torch.zeros((8, 8, 3, 3), device="cuda")
    with pytest.raises(w.WinoError) as ei:                       # F(4x4,3x3) has no one-launch kernel
        w.wino_conv2d_fwd_ex(D, G=G, pad=1, m=4, flags=w.FLAG_ONE_LAUNCH)
    assert ei.value.status == w.WINO_EUNSUPPORTED
    U = w.wino_filter_transform(G, 2)
    with pytest.raises(w.WinoError) as ei:                       # transformed filters are not what it reads
        w.wino_conv2d_fwd_ex(D, U=U, K=8, pad=1, m=2, flags=w.FLAG_ONE_LAUNCH)
    assert ei.value.status == w.WINO_EUNSUPPORTED
    with pytest.raises(w.WinoError) as ei:                       # fp16 storage
        w.wino_conv2d_fwd_ex(D.half(), G=G.half(), pad=1, m=2, flags=w.FLAG_ONE_LAUNCH)
    assert ei.value.status == w.WINO_EUNSUPPORTED
    with pytest.raises(w.WinoError) as ei:
        w.wino_conv2d_fwd_ex(D, G=G, pad=1, m=2, flags=4)
    assert ei.value.status == w.WINO_EINVAL

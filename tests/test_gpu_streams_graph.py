"""Launch-side behaviour on the GPU: calls that overlap on different streams, and a captured HIP graph.

* The short entry point keeps one workspace per stream; the one-launch layer keeps one set of arrival counters per
  stream (the first eight): calls on different streams may overlap and must give the sequential results.
* A whole batch-1 stack captured once in a HIP graph and replayed must reproduce the eager results on every replay
  (replays alternate with eager work and synchronisations; the library records kernels only, no memset nodes)."""
import numpy as np
import pytest

from oracle import direct
from paper_1509_09308_amd import synth
from gpu_util import TOL, check_close, require_gpu, to_gpu

pytestmark = pytest.mark.gpu


def test_short_entry_point_on_overlapping_streams():
    torch, w = require_gpu()
    shapes = [(2, 32, 28, 28, 48), (1, 64, 56, 56, 64), (3, 16, 14, 14, 40), (2, 24, 20, 36, 24)]
    streams = [torch.cuda.Stream() for _ in shapes]
    data = [synth.make_layer(*s, seed=900 + i) for i, s in enumerate(shapes)]
    dev = [(to_gpu(D), to_gpu(G)) for D, G in data]
    outs = [None] * len(shapes)
    torch.cuda.synchronize()
    for rep in range(3):                                   # the same streams again: their workspaces are reused
        for i, ((d, g), st) in enumerate(zip(dev, streams)):
            with torch.cuda.stream(st):
                outs[i] = w.wino_conv2d_fwd(d, g, pad=1, m=4)
        torch.cuda.synchronize()
        for (D, G), Y in zip(data, outs):
            check_close(Y.cpu().numpy(), direct.conv2d_fwd(D, G, pad=1), TOL[("f32", 4)], "stream run %d" % rep, 4)
    w.wino_shutdown()


def test_one_launch_layers_on_overlapping_streams():
    """Ten streams (more than the eight sets of arrival counters): each runs a layer whose channel sum is shared
    between workgroups; every result must equal the one the same call gives alone, bit for bit."""
    torch, w = require_gpu()
    N, C, H, W, K = 1, 256, 14, 14, 96                       # few output blocks, long channel loop: split
    D, G = synth.make_layer(N, C, H, W, K, seed=77)
    d, g = to_gpu(D), to_gpu(G)
    alone = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=2, flags=w.FLAG_ONE_LAUNCH)
    torch.cuda.synchronize()
    check_close(alone.cpu().numpy(), direct.conv2d_fwd(D, G, pad=1), TOL[("f32", 2)], "one launch, alone", 2)
    streams = [torch.cuda.Stream() for _ in range(10)]
    wss = [w.alloc_workspace(N, C, H, W, K, 1, 2) for _ in streams]
    outs = [None] * len(streams)
    for rep in range(4):
        for i, st in enumerate(streams):
            with torch.cuda.stream(st):
                outs[i] = w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=2, flags=w.FLAG_ONE_LAUNCH, workspace=wss[i])
        torch.cuda.synchronize()
        ref = direct.conv2d_fwd(D, G, pad=1)
        for i, Y in enumerate(outs):
            # the stream of the call above holds one of the eight sets of counters, the first seven streams here the
            # others; the rest run the channel sum unshared (same sum, other rounding order)
            if i < 7:
                assert torch.equal(Y, alone), "stream %d, round %d" % (i, rep)
            check_close(Y.cpu().numpy(), ref, TOL[("f32", 2)], "stream %d" % i, 2)


def test_shared_last_round_on_overlapping_streams():
    """The one-kernel F(4x4,3x3) layer hands partial outputs and arrival counters over through the caller's
    workspace: calls on different streams with workspaces of their own may overlap, and each must give the result
    the same call gives alone, bit for bit."""
    torch, w = require_gpu()
    N, C, H, W, K = 2, 256, 96, 96, 512                     # a last round of 8 items per XCD, 8 shares each
    D, G = synth.make_layer(N, C, H, W, K, seed=78)
    d, g = to_gpu(D), to_gpu(G)
    U = w.wino_filter_transform(g, 4)
    alone = w.wino_conv2d_fwd_ex(d, U=U, K=K, pad=1, m=4, flags=w.FLAG_FUSED)
    torch.cuda.synchronize()
    check_close(alone.cpu().numpy(), direct.conv2d_fwd(D, G, pad=1), TOL[("f32", 4)], "shares, alone", 4)
    streams = [torch.cuda.Stream() for _ in range(6)]
    wss = [w.alloc_workspace(N, C, H, W, K, 1, 4) for _ in streams]
    outs = [None] * len(streams)
    for rep in range(3):
        for i, st in enumerate(streams):
            with torch.cuda.stream(st):
                outs[i] = w.wino_conv2d_fwd_ex(d, U=U, K=K, pad=1, m=4, flags=w.FLAG_FUSED, workspace=wss[i])
        torch.cuda.synchronize()
        for i, Y in enumerate(outs):
            assert torch.equal(Y, alone), "stream %d, round %d" % (i, rep)


def test_captured_graph_replays_equal_eager():
    torch, w = require_gpu()
    layers = [synth.VGG16_LAYERS[i] for i in (1, 4, 8, 11)]
    data, dev, Ys, Us = [], [], [], []
    for li, (name, C, HW, K) in enumerate(layers):
        D, G = synth.make_layer(1, C, HW, HW, K, seed=950 + li)
        data.append((D, G))
        dev.append((to_gpu(D), to_gpu(G)))
        Ys.append(torch.empty((1, K, HW, HW), dtype=torch.float32, device="cuda"))
    ms = [4, 4, 2, 2]
    ws = torch.empty(max(w.wino_workspace_bytes(1, C, HW, HW, K, 1, m) for (n, C, HW, K), m in zip(layers, ms)),
                     dtype=torch.uint8, device="cuda")
    direct_in = to_gpu(synth.make_layer(1, 3, 32, 32, 8, seed=949)[0])
    direct_g = to_gpu(synth.make_layer(1, 3, 32, 32, 8, seed=949)[1])
    direct_y = torch.empty((1, 8, 32, 32), dtype=torch.float32, device="cuda")

    def step():
        w.direct_conv2d_fwd(direct_in, direct_g, pad=1, Y=direct_y)
        for (d, g), Y, m in zip(dev, Ys, ms):
            w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=m, Y=Y, workspace=ws)

    step()
    torch.cuda.synchronize()
    eager = [Y.clone() for Y in Ys] + [direct_y.clone()]
    for (D, G), Y, m in zip(data, Ys, ms):
        check_close(Y.cpu().numpy(), direct.conv2d_fwd(D, G, pad=1), TOL[("f32", m)], "eager", m)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(4):
        for Y in Ys + [direct_y]:
            Y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager, Ys + [direct_y]):
            assert torch.equal(a, b), "replay %d differs from the eager result" % rep
        step()                                                 # the program's own eager work between replays
        torch.cuda.synchronize()

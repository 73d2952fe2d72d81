"""The entry point that allocates nothing (wino_conv2d_fwd_noalloc: workspace built into the library) against
the entry point it is a variant of (wino_conv2d_fwd: workspace from hipMalloc) and against the oracle.  Same
kernels, same launch choices: the two outputs must be equal bit for bit."""
import gc

import numpy as np
import pytest

from oracle import direct
from paper_1509_09308_amd import synth
from gpu_util import TOL, check_close, require_gpu, to_gpu

pytestmark = pytest.mark.gpu


def _one_call(torch, w, shape, m, seed):
    N, C, H, W, K = shape
    D, G = synth.make_layer(N, C, H, W, K, seed=seed)
    d, g = to_gpu(D), to_gpu(G)
    Y = torch.full((N, K, H, W), float("nan"), dtype=torch.float32, device="cuda")
    gc.collect()                                            # tensors of earlier tests must not be freed in between
    before = torch.cuda.memory_allocated()
    w.wino_conv2d_fwd_noalloc(d, g, Y, pad=1, m=m)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before          # nothing came from torch's allocator either
    want = w.wino_conv2d_fwd(d, g, pad=1, m=m)
    torch.cuda.synchronize()
    assert torch.equal(Y, want), "differs from wino_conv2d_fwd for %s m=%d" % (shape, m)
    check_close(Y.cpu().numpy(), direct.conv2d_fwd(D, G, pad=1), TOL[("f32", m)], "noalloc %s m=%d" % (shape, m), m)


@pytest.mark.parametrize("m", [2, 4])
def test_noalloc_matches_allocating_entry_point_on_two_calls_in_a_row(m):
    """Second call smaller than the first: what the first left in the shared buffer must not leak into it."""
    torch, w = require_gpu()
    _one_call(torch, w, (2, 64, 56, 56, 96), m, seed=701 + m)      # several tiles, ragged filter block
    _one_call(torch, w, (1, 19, 13, 28, 40), m, seed=703 + m)      # smaller in every extent, ragged
    _one_call(torch, w, (1, 128, 112, 112, 128), 4, seed=707)      # a VGG layer at batch 1 (37 MB of workspace)


def test_noalloc_rejects_what_does_not_fit():
    torch, w = require_gpu()
    N, C, H, W, K = 64, 64, 224, 224, 64                            # 3.7 GB of workspace
    assert w.wino_workspace_bytes(N, C, H, W, K, 1, 4) > w.STATIC_WORKSPACE_BYTES
    d = torch.empty((1,), dtype=torch.float32, device="cuda")      # never touched: rejected before any GPU work
    st = w.lib().wino_conv2d_fwd_noalloc(N, C, H, W, K, 1, 4, d.data_ptr(), d.data_ptr(), d.data_ptr(), None)
    assert st == w.WINO_EWORKSPACE

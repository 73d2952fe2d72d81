"""Host-side checks of libwino.so that need no GPU: the library loads, exports what wino.h
declares, rejects bad arguments with status codes, and its integer bookkeeping (tile maps,
padded extents, buffer offsets) agrees bit for bit with the oracle's."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1509_09308_amd as w
from paper_1509_09308_amd import binding, build
from oracle import winograd as wg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    build.ensure_built()
    return binding.lib()


def test_exports_every_declared_symbol(L):
    text = open(os.path.join(ROOT, "include", "wino.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = re.findall(r"\b(wino_\w+|direct_conv2d_fwd)\s*\(", text)
    declared = sorted(set(declared))
    assert len(declared) >= 20
    assert sorted(binding.EXPORTS) == declared
    for name in declared:
        assert hasattr(L, name), name


def test_status_strings(L):
    seen = {L.wino_status_string(s) for s in range(5)}
    assert len(seen) == 5 and all(seen)
    assert L.wino_status_string(99) == b"unknown status"


def test_argument_validation_without_gpu(L):
    null = None
    fake = ctypes.c_void_p(0x1000)       # aligned, never dereferenced: checks fail first
    odd = ctypes.c_void_p(0x1004)
    # unsupported algorithm / padding
    assert L.wino_conv2d_fwd(1, 4, 8, 8, 4, 1, 3, fake, fake, fake, null) == w.WINO_EUNSUPPORTED
    assert L.wino_conv2d_fwd(1, 4, 8, 8, 4, 2, 4, fake, fake, fake, null) == w.WINO_EUNSUPPORTED
    assert L.wino_conv2d_fwd(1, 4, 2, 2, 4, 0, 2, fake, fake, fake, null) == w.WINO_EUNSUPPORTED  # empty output
    # non-positive extents, null and misaligned pointers
    assert L.wino_conv2d_fwd(0, 4, 8, 8, 4, 1, 2, fake, fake, fake, null) == w.WINO_EINVAL
    assert L.wino_conv2d_fwd(1, 4, 8, 8, -1, 1, 2, fake, fake, fake, null) == w.WINO_EINVAL
    assert L.wino_conv2d_fwd(1, 4, 8, 8, 4, 1, 2, null, fake, fake, null) == w.WINO_EINVAL
    assert L.wino_conv2d_fwd(1, 4, 8, 8, 4, 1, 2, fake, odd, fake, null) == w.WINO_EINVAL
    assert L.wino_filter_transform(4, 4, 2, null, fake, null) == w.WINO_EINVAL
    assert L.wino_filter_transform(4, 4, 5, fake, fake, null) == w.WINO_EUNSUPPORTED
    assert L.wino_filter_transform_ex(4, 4, 2, 7, fake, fake, null) == w.WINO_EINVAL
    assert L.wino_input_transform(1, 4, 8, 8, 1, 2, 0, fake, null, null) == w.WINO_EINVAL
    assert L.wino_batched_gemm(4, 4, 0, 2, 0, fake, fake, fake, null) == w.WINO_EINVAL
    assert L.wino_output_transform(1, 4, 8, 8, 1, 2, 0, fake, odd, null) == w.WINO_EINVAL
    assert L.direct_conv2d_fwd(1, 3, 8, 8, 4, 3, 3, 1, 0, 0, fake, fake, fake, null) == w.WINO_EINVAL
    assert L.direct_conv2d_fwd(1, 3, 2, 2, 4, 5, 5, 0, 1, 0, fake, fake, fake, null) == w.WINO_EUNSUPPORTED
    # the entry point with the built-in workspace: same argument checks, and a layer that does not fit it
    assert L.wino_conv2d_fwd_noalloc(0, 4, 8, 8, 4, 1, 2, fake, fake, fake, null) == w.WINO_EINVAL
    assert L.wino_conv2d_fwd_noalloc(1, 4, 8, 8, 4, 1, 2, fake, odd, fake, null) == w.WINO_EINVAL
    assert L.wino_conv2d_fwd_noalloc(1, 4, 8, 8, 4, 1, 5, fake, fake, fake, null) == w.WINO_EUNSUPPORTED
    assert L.wino_workspace_bytes(64, 64, 224, 224, 64, 1, 4, 0) > w.STATIC_WORKSPACE_BYTES
    assert L.wino_conv2d_fwd_noalloc(64, 64, 224, 224, 64, 1, 4, fake, fake, fake, null) == w.WINO_EWORKSPACE
    # workspace too small / both G and U missing
    need = L.wino_workspace_bytes(1, 4, 8, 8, 4, 1, 2, 0)
    assert need > 0
    assert L.wino_conv2d_fwd_ex(1, 4, 8, 8, 4, 1, 2, 0, 0, fake, fake, null, fake, fake, need - 1, 0,
                                null) == w.WINO_EWORKSPACE
    assert L.wino_conv2d_fwd_ex(1, 4, 8, 8, 4, 1, 2, 0, 0, fake, null, null, fake, fake, need, 0,
                                null) == w.WINO_EINVAL
    assert L.wino_conv2d_fwd_ex(1, 4, 8, 8, 4, 1, 2, 0, 0, fake, fake, null, fake, fake, need, 99,
                                null) == w.WINO_EINVAL
    # F(6x6,3x3): fp32 storage only
    assert L.wino_workspace_bytes(1, 4, 8, 8, 4, 1, 6, 0) > 0
    assert L.wino_workspace_bytes(1, 4, 8, 8, 4, 1, 6, 1) == 0
    assert L.wino_conv2d_variant(1, 4, 8, 8, 4, 1, 6, 1, 0, 0) == -w.WINO_EUNSUPPORTED
    assert L.wino_conv2d_variant(1, 4, 8, 8, 4, 1, 6, 0, 0, 0) == w.FLAG_UNFUSED
    assert L.wino_num_tiles(2, 14, 14, 1, 6) == 2 * 3 * 3
    # filter gradient: fp32 and pad 1 only, workspace and pointers checked
    need = L.wino_bwd_filter_workspace_bytes(2, 8, 8, 8, 4)
    assert need >= 16 * 32 * 32 * 4              # at least one partial M (16 components, 32 x 32 padded)
    assert L.wino_conv2d_bwd_filter(2, 8, 8, 8, 4, 1, 0, fake, fake, fake, fake, need - 1, null) == w.WINO_EWORKSPACE
    assert L.wino_conv2d_bwd_filter(2, 8, 8, 8, 4, 0, 0, fake, fake, fake, fake, need, null) == w.WINO_EUNSUPPORTED
    assert L.wino_conv2d_bwd_filter(2, 8, 8, 8, 4, 1, 1, fake, fake, fake, fake, need, null) == w.WINO_EUNSUPPORTED
    assert L.wino_conv2d_bwd_filter(2, 8, 8, 8, 4, 1, 0, fake, null, fake, fake, need, null) == w.WINO_EINVAL
    assert L.wino_conv2d_bwd_filter(2, 8, 8, 8, 4, 1, 0, fake, fake, odd, fake, need, null) == w.WINO_EINVAL
    assert L.wino_conv2d_bwd_filter(2, 0, 8, 8, 4, 1, 0, fake, fake, fake, fake, need, null) == w.WINO_EINVAL
    # at most 4 channels and W a multiple of 4: evaluated directly, workspace = a few partial gradients per image
    assert 0 < L.wino_bwd_filter_workspace_bytes(2, 3, 8, 8, 4) < 2 * 8 * 4 * 3 * 9 * 4
    assert L.wino_bwd_filter_workspace_bytes(0, 4, 8, 8, 4) == 0
    # size queries on bad input
    assert L.wino_workspace_bytes(1, 4, 8, 8, 4, 1, 3, 0) == 0
    assert L.wino_filter_bytes(0, 4, 2, 0) == 0
    assert L.wino_num_tiles(1, 8, 8, 3, 2) == -1


SHAPES = [(1, 56, 56, 1, 2), (8, 28, 28, 1, 2), (8, 28, 28, 1, 4), (1, 224, 224, 1, 4), (2, 112, 112, 1, 4),
          (3, 14, 14, 1, 4), (3, 14, 14, 1, 2), (2, 7, 9, 1, 4), (2, 7, 9, 0, 2), (1, 5, 5, 0, 4), (64, 14, 14, 1, 4),
          (2, 56, 56, 1, 6), (3, 14, 14, 1, 6), (1, 9, 20, 0, 6)]


@pytest.mark.parametrize("N,H,W,pad,m", SHAPES)
def test_tile_bookkeeping_matches_oracle_exhaustively(L, N, H, W, pad, m):
    P = w.wino_num_tiles(N, H, W, pad, m)
    assert P == wg.num_tiles(N, H, W, pad, m)
    step = 1 if P <= 20000 else 7
    for b in list(range(0, P, step)) + [P - 1]:
        assert w.wino_tile_coords(N, H, W, pad, m, b) == wg.tile_of(b, H, W, pad, m)
    out = (ctypes.c_int * 5)()
    assert L.wino_tile_coords(N, H, W, pad, m, P, out) == w.WINO_EINVAL
    assert L.wino_tile_coords(N, H, W, pad, m, -1, out) == w.WINO_EINVAL


@pytest.mark.parametrize("K,C,P,m,dt", [(64, 64, 3136, 4, 0), (32, 32, 784, 2, 0), (512, 512, 49, 2, 0),
                                         (5, 3, 17, 4, 0), (70, 33, 100, 2, 1), (512, 512, 16, 4, 1)])
def test_padded_dims_offsets_and_sizes(L, K, C, P, m, dt):
    a = m + 2
    Kp, Cp, Pp = w.wino_padded_dims(K, C, P, m, dt)
    assert Kp >= K and Cp >= C and Pp >= P and Kp % 32 == 0 and Pp % 32 == 0 and Cp % (32 if dt else 16) == 0
    assert Kp - K < 32 and Pp - P < 32
    es = 2 if dt else 4
    assert w.wino_filter_bytes(K, C, m, dt) == a * a * Kp * Cp * es
    assert w.wino_v_bytes(C, P, m, dt) == a * a * Cp * Pp * es
    assert w.wino_m_bytes(K, P, m) == a * a * Kp * Pp * 4
    rng = np.random.default_rng(K + C)
    seen_u, seen_v, seen_m = set(), set(), set()
    for _ in range(300):
        xi, nu = int(rng.integers(a)), int(rng.integers(a))
        k, c, b = int(rng.integers(Kp)), int(rng.integers(Cp)), int(rng.integers(Pp))
        e = xi * a + nu
        ou, ov, om = (w.wino_u_offset(K, C, m, dt, xi, nu, k, c), w.wino_v_offset(C, P, m, dt, xi, nu, c, b),
                      w.wino_m_offset(K, P, m, xi, nu, k, b))
        if dt == 0:
            assert ou == (e * Cp + c) * Kp + k and ov == (e * Cp + c) * Pp + b
        else:
            assert ou == ((e * (Cp // 8) + c // 8) * Kp + k) * 8 + c % 8
            assert ov == ((e * (Cp // 8) + c // 8) * Pp + b) * 8 + c % 8
        assert om == (e * Kp + k) * Pp + b
        assert 0 <= ou < a * a * Kp * Cp and 0 <= ov < a * a * Cp * Pp and 0 <= om < a * a * Kp * Pp
        seen_u.add(ou), seen_v.add(ov), seen_m.add(om)
    assert w.wino_u_offset(K, C, m, dt, a, 0, 0, 0) == -1
    assert w.wino_v_offset(C, P, m, dt, 0, 0, Cp, 0) == -1
    assert w.wino_m_offset(K, P, m, 0, 0, 0, Pp) == -1


def test_pack_unpack_round_trip_host_only():
    """The binding's layout helpers invert each other (checked on CPU tensors)."""
    rng = np.random.default_rng(0)
    for dt, npdt in ((0, np.float32), (1, np.float16)):
        for m in ((2, 4, 6) if dt == 0 else (2, 4)):
            a = m + 2
            u = rng.standard_normal((a, a, 5, 19)).astype(npdt)
            v = rng.standard_normal((a, a, 19, 45)).astype(npdt)
            mm = rng.standard_normal((a, a, 5, 45)).astype(np.float32)
            assert np.array_equal(w.unpack_u(w.pack_u(u, m, dt, "cpu"), 5, 19, m, dt), u)
            assert np.array_equal(w.unpack_v(w.pack_v(v, m, dt, "cpu"), 19, 45, m, dt), v)
            assert np.array_equal(w.unpack_m(w.pack_m(mm, m, "cpu"), 5, 45, m), mm)
            # a spot check of the packed position against the C offset function
            flat = w.pack_u(u, m, dt, "cpu").numpy()
            assert flat[w.wino_u_offset(5, 19, m, dt, 1, 2, 3, 17)] == u[1, 2, 3, 17]
            flat = w.pack_v(v, m, dt, "cpu").numpy()
            assert flat[w.wino_v_offset(19, 45, m, dt, 2, 1, 18, 44)] == v[2, 1, 18, 44]


def test_flop_accounting_matches_table3(golden):
    """bench.py's direct-convolution flop formula reproduces Table 3 of the paper."""
    import bench
    for name, depth, C, HW, K, gf in golden("table3_vgg_e_gflops.txt"):
        if name != "total":
            got = int(depth) * bench.direct_flops(1, int(C), int(HW), int(HW), int(K)) / 1e9
            assert abs(got - float(gf)) < 0.0051


def test_variant_query_host_only(L):
    """Which path a call takes is decided on the host and can be asked without a GPU."""
    # the VGG layers with few filters and many tiles go to the one-kernel path, the rest do not
    assert w.wino_conv2d_variant(64, 64, 224, 224, 64, 1, 4) == w.FLAG_FUSED
    assert w.wino_conv2d_variant(64, 128, 112, 112, 128, 1, 4) == w.FLAG_FUSED
    assert w.wino_conv2d_variant(64, 512, 28, 28, 512, 1, 4) == w.FLAG_FUSED        # 256: where the rounds fill (3 + a shared one)
    assert w.wino_conv2d_variant(32, 512, 28, 28, 512, 1, 4) == w.FLAG_UNFUSED      # ... two rounds for 1.5
    assert w.wino_conv2d_variant(8, 512, 28, 28, 512, 1, 4) == w.FLAG_UNFUSED       # fewer items than workgroups
    assert w.wino_conv2d_variant(64, 128, 56, 56, 256, 1, 4) == w.FLAG_FUSED        # K C / (K + C) = 85
    assert w.wino_conv2d_variant(64, 256, 56, 56, 256, 1, 4) == w.FLAG_FUSED        # 128: 64 filters per workgroup win
    assert w.wino_conv2d_variant(32, 256, 56, 56, 256, 1, 4) == w.FLAG_FUSED
    assert w.wino_conv2d_variant(4, 256, 56, 56, 256, 1, 4) == w.FLAG_UNFUSED       # ... with a workgroup for every slot
    assert w.wino_conv2d_variant(64, 256, 28, 28, 512, 1, 4) == w.FLAG_FUSED        # 171: still ahead
    assert w.wino_conv2d_variant(1, 64, 224, 224, 64, 1, 4) == w.FLAG_FUSED         # batch 1, 64 -> 64: 196 workgroups suffice
    assert w.wino_conv2d_variant(1, 128, 112, 112, 128, 1, 4) == w.FLAG_UNFUSED     # too few workgroups
    assert w.wino_conv2d_variant(2, 128, 112, 112, 128, 1, 4) == w.FLAG_FUSED       # 196: one per CU
    assert w.wino_conv2d_variant(3, 128, 112, 112, 128, 1, 4) == w.FLAG_UNFUSED     # 296: some CUs hold two
    assert w.wino_conv2d_variant(64, 64, 224, 224, 64, 1, 2) == w.FLAG_FUSED        # F(2x2): the 64-filter design
    assert w.wino_conv2d_variant(64, 512, 14, 14, 512, 1, 2) == w.FLAG_FUSED
    assert w.wino_conv2d_variant(1, 512, 14, 14, 512, 1, 2) == w.FLAG_UNFUSED       # ... where it fills the GPU
    assert w.wino_conv2d_variant(64, 32, 56, 56, 32, 1, 2) == w.FLAG_UNFUSED        # ... and has 33 filters or more
    assert w.wino_conv2d_variant(64, 64, 224, 224, 64, 1, 4, flags=w.FLAG_UNFUSED) == w.FLAG_UNFUSED
    assert w.wino_conv2d_variant(2, 8, 8, 8, 8, 1, 4, flags=w.FLAG_FUSED) == w.FLAG_FUSED
    assert L.wino_conv2d_variant(2, 8, 8, 8, 8, 1, 2, 0, 0, w.FLAG_FUSED) == -w.WINO_EUNSUPPORTED
    # fp16 storage has a one-kernel path of its own: m = 4, pad = 1, W % 4 == 0, fp32 outputs
    assert L.wino_conv2d_variant(2, 8, 8, 8, 8, 1, 4, 1, 0, w.FLAG_FUSED) == w.FLAG_FUSED
    assert L.wino_conv2d_variant(2, 8, 8, 10, 8, 1, 4, 1, 0, w.FLAG_FUSED) == -w.WINO_EUNSUPPORTED
    assert L.wino_conv2d_variant(2, 8, 8, 8, 8, 0, 4, 1, 0, w.FLAG_FUSED) == -w.WINO_EUNSUPPORTED
    assert L.wino_conv2d_variant(2, 8, 8, 8, 8, 1, 4, 1, 1, w.FLAG_FUSED) == w.FLAG_FUSED           # fp16 storage, fp16 Y
    assert L.wino_conv2d_variant(2, 8, 8, 8, 8, 1, 4, 0, 1, w.FLAG_FUSED) == -w.WINO_EUNSUPPORTED   # fp32 storage, fp16 Y
    assert L.wino_conv2d_variant(32, 64, 224, 224, 64, 1, 4, 1, 0, 0) == w.FLAG_FUSED
    assert L.wino_conv2d_variant(32, 512, 28, 28, 512, 1, 4, 1, 0, 0) == w.FLAG_UNFUSED
    assert L.wino_conv2d_variant(2, 8, 8, 8, 8, 1, 3, 0, 0, 0) == -w.WINO_EUNSUPPORTED
    assert L.wino_conv2d_variant(2, 8, 8, 8, 8, 1, 4, 0, 0, 7) == -w.WINO_EINVAL
    # inputs of 2 GiB or more need 64-bit tap offsets: not eligible
    assert L.wino_conv2d_variant(256, 64, 224, 224, 64, 1, 4, 0, 0, w.FLAG_FUSED) == -w.WINO_EUNSUPPORTED
    # the one-launch layer (filter transform inside the kernel) exists for fp32 F(2x2,3x3) only, either padding
    assert w.wino_conv2d_variant(1, 512, 14, 14, 512, 1, 2, flags=w.FLAG_ONE_LAUNCH) == w.FLAG_ONE_LAUNCH
    assert w.wino_conv2d_variant(3, 5, 9, 11, 7, 0, 2, flags=w.FLAG_ONE_LAUNCH) == w.FLAG_ONE_LAUNCH
    assert L.wino_conv2d_variant(1, 512, 14, 14, 512, 1, 4, 0, 0, w.FLAG_ONE_LAUNCH) == -w.WINO_EUNSUPPORTED
    assert L.wino_conv2d_variant(1, 512, 14, 14, 512, 1, 2, 1, 0, w.FLAG_ONE_LAUNCH) == -w.WINO_EUNSUPPORTED  # fp16
    assert L.wino_conv2d_variant(1, 512, 14, 14, 512, 1, 2, 0, 1, w.FLAG_ONE_LAUNCH) == -w.WINO_EUNSUPPORTED  # fp16 Y
    # one image of 2^31 elements or more needs 64-bit offsets inside the image: not eligible; many small images are
    assert L.wino_conv2d_variant(1, 512, 2048, 2048, 64, 1, 2, 0, 0, w.FLAG_ONE_LAUNCH) == -w.WINO_EUNSUPPORTED
    assert L.wino_conv2d_variant(2048, 64, 224, 224, 64, 1, 2, 0, 0, w.FLAG_ONE_LAUNCH) == w.FLAG_ONE_LAUNCH
    assert L.wino_conv2d_variant(1, 512, 14, 14, 512, 1, 2, 0, 0, 4) == -w.WINO_EINVAL


def test_gemm_launch_shape_host_only(L):
    """The block shape and channel shares of the multiply inside a layer call can be asked on the host."""
    assert w.wino_gemm_launch_shape(256, 256, 64 * 196, 4) == (128, 128, 1)     # conv3.x at N = 64: 27.6 blocks per CU
    assert w.wino_gemm_launch_shape(512, 512, 64 * 49, 4) == (128, 64, 1)       # conv4.x: 14.06 per CU -> halved blocks
    bm, bn, shares = w.wino_gemm_launch_shape(512, 512, 49, 2)                 # conv5.x at N = 1: small blocks, split sum
    assert (bm, bn) == (64, 64) and shares >= 2
    assert w.wino_gemm_launch_shape(64, 64, 3136, 4)[:2] == (64, 128)
    out = (ctypes.c_int * 3)()
    assert L.wino_gemm_launch_shape(0, 8, 8, 2, 0, out) == w.WINO_EINVAL
    assert L.wino_gemm_launch_shape(8, 8, 8, 3, 0, out) == w.WINO_EUNSUPPORTED
    assert L.wino_gemm_launch_shape(8, 8, 8, 2, 0, None) == w.WINO_EINVAL


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N > 1 exits with a message before touching any GPU (this build is single-GPU)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0
    assert "one GPU" in res.stderr and res.stdout.strip() == ""


def test_one_kernel_plan_covers_every_item_once_and_shares_fit():
    """The deal of (tile block, filter block) items to XCDs and rounds that the one-kernel fp32 layer's workgroups
    follow (the kernel evaluates the same functions): every item belongs to exactly one XCD's list, a shared last
    round fits the XCD's 64 workgroups, the shares divide the channel steps, and only long items are shared."""
    import math
    w = binding
    rng = __import__("numpy").random.default_rng(5)
    seen_shared = 0
    cases = [(64, 256, 56, 56, 256), (64, 512, 28, 28, 512), (64, 256, 28, 28, 512), (64, 64, 224, 224, 64),
             (64, 128, 112, 112, 128), (2, 256, 96, 96, 512), (6, 256, 72, 72, 320), (2, 344, 96, 96, 512),
             (1, 64, 224, 224, 64), (8, 512, 28, 28, 512), (3, 40, 12, 20, 96)]
    for _ in range(300):
        cases.append((int(rng.integers(1, 200)), int(rng.integers(1, 700)), int(rng.integers(3, 80)),
                      4 * int(rng.integers(1, 24)), int(rng.integers(33, 700))))
    planned = 0
    for m, slots in ((4, 64), (2, 96)):            # resident workgroups per XCD: two resp. three per CU
      for N, C, H, W, K in cases:
        try:
            grid, plan = w.wino_one_kernel_plan(N, C, H, W, K, 1, m)
        except binding.WinoError as e:                      # inputs beyond the kernel's 32-bit offsets
            assert e.status == w.WINO_EUNSUPPORTED and N * C * H * W * 4 > 2 ** 29, (N, C, H, W, K)
            continue
        planned += 1
        P = w.wino_num_tiles(N, H, W, 1, m)
        Kp = w.wino_padded_dims(K, C, P, m)[0]
        items = ((P + 15) // 16) * ((Kp + 63) // 64)
        nsteps = (C + 15) // 16
        assert grid == (8 * slots if items >= 8 * slots else (items + 7) // 8 * 8), (N, C, H, W, K)
        assert sum(p[0] for p in plan) == items, (N, C, H, W, K, plan)
        for count, full, tail, shares in plan:
            assert full + tail == count and full >= 0 and tail >= 0 and shares >= 1
            if shares > 1:
                seen_shared += 1
                assert grid == 8 * slots and full % slots == 0 and 0 < tail and tail * shares <= slots
                assert shares in (2, 4, 8) and nsteps % shares == 0 and nsteps >= 16
                assert shares >= 4 or full == 0
            else:
                assert tail == 0
    assert seen_shared > 40 and planned > 400
    # the VGG layers this is made for: conv3.2 (8 items of the last round in 8 shares on every XCD), conv4.2 (4 in 8)
    assert w.wino_one_kernel_plan(64, 256, 56, 56, 256)[1] == [(392, 384, 8, 8)] * 8
    assert w.wino_one_kernel_plan(64, 512, 28, 28, 512)[1] == [(196, 192, 4, 8)] * 8
    assert all(p[3] == 1 for p in w.wino_one_kernel_plan(64, 64, 224, 224, 64)[1])
    L = binding.lib()
    out = (ctypes.c_int * 32)()
    assert L.wino_one_kernel_plan(2, 8, 8, 8, 8, 1, 4, 0, out) == -w.WINO_EUNSUPPORTED      # fewer than 33 filters
    assert L.wino_one_kernel_plan(2, 8, 8, 8, 40, 0, 4, 0, out) == -w.WINO_EUNSUPPORTED     # pad 0
    assert w.wino_one_kernel_plan(64, 512, 14, 14, 512, 1, 2)[1] == [(196, 192, 4, 8)] * 8  # F(2x2): conv5.x
    assert L.wino_one_kernel_plan(2, 8, 8, 10, 8, 1, 4, 0, out) == -w.WINO_EUNSUPPORTED     # W % 4 != 0
    assert L.wino_one_kernel_plan(2, 8, 8, 8, 8, 1, 4, 1, out) == -w.WINO_EUNSUPPORTED      # fp16 storage
    assert L.wino_one_kernel_plan(0, 8, 8, 8, 8, 1, 4, 0, out) == -w.WINO_EINVAL

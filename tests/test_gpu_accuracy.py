"""The accuracy experiment of the paper (Section 7 set-up, Section 8 Table 4) on the GPU path: data and
filters uniform on [-1, 1], maximum absolute element error against direct convolution accumulated in
double precision, for the direct kernel, F(2x2,3x3) and F(4x4,3x3) with fp32 storage, and for fp16
storage of data and filters (ground truth from the UNROUNDED inputs there: the paper's fp16 column
is limited by the precision of the inputs, which only that reading reproduces).

One column cannot be reproduced by construction: the paper rounds only data and filters to fp16 and keeps
the transformed operands in fp32, whereas the fp16 workload of this library also stores U and V in fp16.
For F(2x2,3x3) that changes little; for F(4x4,3x3) the rounding of V (values up to 100 times the data) is
amplified by the inverse transform, so its fp16 error lies above Table 4's column (and within the bound
the workload states for it), which the test asserts as such."""
import numpy as np
import pytest

from conftest import read_golden
from oracle import direct
from paper_1509_09308_amd import synth
from gpu_util import max_abs_bound, require_gpu, to_gpu

pytestmark = pytest.mark.gpu

ROWS = read_golden("table4_max_error.txt")


def measure(w, torch, C, HW, K, seed, N=1):
    """Max-abs errors (direct fp32, F(2x2) fp32, F(4x4) fp32, F(2x2) fp16 data, F(4x4) fp16 data, direct fp16 data)."""
    D, G = synth.make_uniform_layer(N, C, HW, HW, K, seed)
    ref = direct.conv2d_fwd(D, G, pad=1)
    d, g = to_gpu(D), to_gpu(G)
    d16, g16 = to_gpu(D.astype(np.float16)), to_gpu(G.astype(np.float16))
    err = lambda Y: float(np.abs(Y.float().cpu().numpy().astype(np.float64) - ref).max())
    return ref, {
        "direct_fp32": err(w.direct_conv2d_fwd(d, g, pad=1)),
        "f2x2_fp32": err(w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=2)),
        "f4x4_fp32": err(w.wino_conv2d_fwd_ex(d, G=g, pad=1, m=4)),
        "f2x2_fp16": err(w.wino_conv2d_fwd_ex(d16, G=g16, pad=1, m=2)),
        "f4x4_fp16": err(w.wino_conv2d_fwd_ex(d16, G=g16, pad=1, m=4)),
        "direct_fp16": err(w.direct_conv2d_fwd(d16, g16, pad=1).float()),
    }


@pytest.mark.parametrize("row", ROWS, ids=[r[0] for r in ROWS])
def test_error_magnitudes_land_in_the_decade_of_table4(row):
    torch, w = require_gpu()
    name, C, HW, K = row[0], int(row[1]), int(row[2]), int(row[3])
    p_direct, p_f2, p_f4, p_f16 = (float(x) for x in row[4:8])
    ref, got = measure(w, torch, C, HW, K, seed=synth.layer_seed(9, ROWS.index(row)))
    print(name, {k: "%.2e" % v for k, v in got.items()}, "paper:", row[4:8])
    decade = lambda mine, paper: paper / 10.0 <= mine <= paper * 10.0
    assert decade(got["direct_fp32"], p_direct)
    assert decade(got["f2x2_fp32"], p_f2)
    assert decade(got["f4x4_fp32"], p_f4)
    # "All tested algorithms are equally accurate with fp16 data": one column for all of them
    for k in ("f2x2_fp16", "direct_fp16"):
        assert decade(got[k], p_f16), k
    # fp16 storage of U and V as well (not the paper's experiment): above the column, inside the workload's bound
    assert got["f2x2_fp16"] < got["f4x4_fp16"] <= max_abs_bound(ref, 5e-3, 4)
    # the ordering the paper reports: F(2x2) no worse than direct fp32; F(4x4) worse than both but better than fp16 data
    assert got["f2x2_fp32"] <= got["direct_fp32"] * 1.5
    assert got["f2x2_fp32"] < got["f4x4_fp32"] < min(got["f2x2_fp16"], got["direct_fp16"])

"""Pins for oracle/complexity.py against the tables the paper prints (no GPU)."""
import pytest

from oracle import complexity as cx


def test_minimal_multiplication_counts():
    """Eq. (3), Eq. (4) and the counts quoted in Sections 4.1 and 4.3."""
    assert cx.mu_1d(2, 3) == 4 and cx.mu_1d(4, 3) == 6
    assert cx.mu_2d(2, 2, 3, 3) == 16 and cx.mu_2d(4, 4, 3, 3) == 36
    assert cx.mu_2d(3, 3, 2, 2) == 16
    assert 2 * 2 * 3 * 3 / cx.mu_2d(2, 2, 3, 3) == 2.25
    assert 4 * 4 * 3 * 3 / cx.mu_2d(4, 4, 3, 3) == 4.0
    assert cx.mu_2d(1, 1, 3, 3) == 9          # m = 1 is direct convolution (Section 5)


def test_table1_winograd_rows(golden):
    for tile, ap, bp, gp, dp in golden("table1_winograd_rows.txt"):
        m = int(tile) - 2
        got = cx.normalized_complexity(m)
        for g, e in zip(got, (ap, bp, gp, dp)):
            assert abs(g - float(e)) < 0.005 + 1e-12, (tile, got)


def test_table3_gflops(golden):
    rows = golden("table3_vgg_e_gflops.txt")
    ours = dict(cx.vgg_e_gflops(1))
    total = 0.0
    for name, depth, C, HW, K, gf in rows:
        if name == "total":
            assert abs(total - float(gf)) < 0.02
            continue
        total += ours[name]
        assert abs(ours[name] - float(gf)) < 0.0051, name
    assert [r[0] for r in rows[:-1]] == [l[0] for l in cx.VGG_E_LAYERS]


@pytest.mark.parametrize("table", ["table5_fp32_speed.txt", "table6_fp16_speed.txt"])
def test_effective_tflops_definition(golden, table):
    total = sum(g for _, g in cx.vgg_e_gflops(1))
    for N, msec, tf in golden(table):
        assert abs(cx.effective_tflops(total * int(N), float(msec)) - float(tf)) < 0.0075


def test_layer_complexity_limits():
    """Eq. (23) tends to alpha' N H W C K when K, P, C are large; speed-up bound R^2/alpha'."""
    N, C, H, W, K = 64, 4096, 224, 224, 4096
    for m, red in ((2, 2.25), (4, 4.0)):
        L = cx.layer_complexity(N, C, H, W, K, m)
        base = N * H * W * C * K
        ap = cx.normalized_complexity(m)[0]
        assert ap <= L / base < ap * 1.01
        assert 9 / ap == red

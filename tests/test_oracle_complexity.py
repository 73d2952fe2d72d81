"""Pins for oracle/complexity.py against the tables the paper prints (no GPU)."""
from fractions import Fraction

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


def test_layer_complexity_equals_the_sum_of_the_stage_counts_at_finite_sizes():
    """Eq. (23) against its own derivation, Eq. (19)-(21), expanded by hand for two layers with C != K so
    that every term is distinguishable: M = tiles * C * K * alpha^2 multiplications, T(D) = beta per
    (tile, channel), T(F) = gamma per (filter, channel), T(I) = delta per (tile, filter), with the
    per-tile instruction counts of Sections 4.1 and 4.3.  N=2, C=256, K=512, 28 x 28 (the conv4.1 shape)."""
    N, C, H, W, K = 2, 256, 28, 28, 512
    # F(2x2,3x3): 14 x 14 tiles per image -> P = 392; alpha^2 = 16; (beta, gamma, delta) = (32, 28, 24)
    M2, D2, F2, I2 = 392 * 256 * 512 * 16, 32 * 392 * 256, 28 * 256 * 512, 24 * 392 * 512
    assert (M2, D2, F2, I2) == (822083584, 3211264, 3670016, 4816896)
    assert cx.layer_complexity(N, C, H, W, K, 2) == pytest.approx(M2 + D2 + F2 + I2, rel=1e-12)
    # F(4x4,3x3): 7 x 7 tiles per image -> P = 98; alpha^2 = 36; (beta, gamma, delta) = (156, 72, 100)
    M4, D4, F4, I4 = 98 * 256 * 512 * 36, 156 * 98 * 256, 72 * 256 * 512, 100 * 98 * 512
    assert (M4, D4, F4, I4) == (462422016, 3913728, 9437184, 5017600)
    assert cx.layer_complexity(N, C, H, W, K, 4) == pytest.approx(M4 + D4 + F4 + I4, rel=1e-12)
    # a swapped pair of terms (beta'/C, delta'/K) would give these instead
    assert abs((M4 + 156 * 98 * 512 + F4 + 100 * 98 * 256) - (M4 + D4 + F4 + I4)) > 1e6
    # Eq. (19) with m = 1 is direct convolution: N H W C K R^2 multiplications
    assert 2 * 28 * 28 * 256 * 512 * 9 * 2 == cx.direct_flops(N, C, H, W, K)


class _Counted:
    """A rational number that counts the floating point instructions applied to it (an addition, a
    subtraction, a multiplication or a fused multiply-add each count one)."""
    ops = 0

    def __init__(self, v):
        self.v = Fraction(v)

    def __add__(self, o):
        _Counted.ops += 1
        return _Counted(self.v + o.v)

    def __sub__(self, o):
        _Counted.ops += 1
        return _Counted(self.v - o.v)

    def scaled(self, c):
        _Counted.ops += 1
        return _Counted(self.v * Fraction(c))

    def fma(self, c, o):
        """self * c + o as one instruction."""
        _Counted.ops += 1
        return _Counted(self.v * Fraction(c) + o.v)


def _bt_f2(d):
    return [d[0] - d[2], d[1] + d[2], d[2] - d[1], d[1] - d[3]]


def _at_f2(m):
    return [m[0] + m[1] + m[2], m[1] - m[2] - m[3]]


def _bt_f4(d):
    r0 = d[2].fma(-5, d[0].fma(4, d[4]))
    r5 = d[3].fma(-5, d[1].fma(4, d[5]))
    a, b = d[2].fma(-4, d[4]), d[1].fma(-4, d[3])
    c, e = d[4] - d[2], (d[3] - d[1]).scaled(2)
    return [r0, a + b, a - b, c + e, c - e, r5]


def _at_f4(m):
    p1, q1, p2, q2 = m[1] + m[2], m[1] - m[2], m[3] + m[4], m[3] - m[4]
    return [m[0] + p1 + p2, q2.fma(2, q1), p2.fma(4, p1), q2.fma(8, q1) + m[5]]


def _bt_f6(d):
    q = Fraction
    r0 = (d[4] - d[2]).fma(q(21, 4), d[0] - d[6])
    r7 = (d[3] - d[5]).fma(q(21, 4), d[7] - d[1])
    a, b = d[4].fma(q(-17, 4), d[2] + d[6]), d[3].fma(q(-17, 4), d[1] + d[5])
    c = d[4].fma(q(-5, 4), d[2].fma(q(1, 4), d[6]))
    e = d[5].fma(2, d[3].fma(q(-5, 2), d[1].scaled(q(1, 2))))
    f = d[4].fma(-5, d[2].fma(4, d[6]))
    g = d[5].fma(q(1, 2), d[3].fma(q(-5, 2), d[1].scaled(2)))
    return [r0, a + b, a - b, c + e, c - e, f + g, f - g, r7]


def _at_f6(m):
    q = Fraction
    p1, q1, p2, q2, p3, q3 = m[1] + m[2], m[1] - m[2], m[3] + m[4], m[3] - m[4], m[5] + m[6], m[5] - m[6]
    return [m[0] + p1 + p2 + p3,
            q3.fma(q(1, 2), q2.fma(2, q1)), p3.fma(q(1, 4), p2.fma(4, p1)), q3.fma(q(1, 8), q2.fma(8, q1)),
            p3.fma(q(1, 16), p2.fma(16, p1)), q3.fma(q(1, 32), q2.fma(32, q1)) + m[7]]


@pytest.mark.parametrize("m,bt,at", [(2, _bt_f2, _at_f2), (4, _bt_f4, _at_f4), (6, _bt_f6, _at_f6)])
def test_transform_instruction_counts_are_reached_by_a_counted_factorisation(m, bt, at):
    """The per-tile data- and inverse-transform counts (beta, delta) of Sections 4.1 / 4.3 -- and, for
    F(6x6,3x3), the counts behind Table 1's row for tile 8, which the text does not state -- are what a
    straight-line evaluation of the 1-D transforms costs when it is nested over the 2-D tile: alpha
    columns then alpha rows of B^T (2 alpha 1-D transforms), alpha columns then m rows of A^T.  Each
    program below is checked to BE the matrix (exact rationals) and its instructions are counted."""
    from oracle import winograd as wg
    BT, _, AT = wg.matrices(m)
    a = m + 2
    rng = __import__("random").Random(m)
    x = [Fraction(rng.randint(-9, 9), rng.randint(1, 7)) for _ in range(a)]
    for prog, mat, rows in ((bt, BT, a), (at, AT, m)):
        _Counted.ops = 0
        got = [c.v for c in prog([_Counted(v) for v in x])]
        n1d = _Counted.ops
        assert got == [sum(Fraction(mat[i][j]) * x[j] for j in range(a)) for i in range(rows)]
        per_tile = n1d * (a + rows)
        want = cx.TRANSFORM_FLOPS[m][0 if prog is bt else 2]
        assert per_tile == want, (m, prog.__name__, n1d, per_tile, want)

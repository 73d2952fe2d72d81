"""Pins for oracle/winograd.py: what the paper and exact arithmetic fix (no GPU)."""
import random
from fractions import Fraction as Fr

import numpy as np
import pytest

from oracle import winograd as wg
from oracle import direct


def _rand_frac(rng):
    return Fr(rng.randint(-9, 9), rng.randint(1, 7))


def _corr1d(d, g, m):
    return [sum(d[i + j] * g[j] for j in range(len(g))) for i in range(m)]


def _corr2d(d, g, m, n):
    r, s = len(g), len(g[0])
    return [[sum(d[i + u][j + v] * g[u][v] for u in range(r) for v in range(s))
             for j in range(n)] for i in range(m)]


@pytest.mark.parametrize("m,r", [(2, 3), (4, 3), (3, 2), (6, 3)])
def test_matrices_follow_from_their_interpolation_points(m, r):
    """Every matrix set equals the evaluation/interpolation construction of Section 4 on its
    points up to the scalings the construction leaves free: column j of A^T by a_j, row j of G by
    f_j, row j of B^T by b_j with a_j f_j b_j = 1 (a product term is unchanged).  Ties the F(6,3)
    set, which the paper does not print, to the same construction as the printed ones."""
    bt, g, at = wg.cook_toom(wg.POINTS[(m, r)], m, r)
    BT, G, AT = wg.matrices(m, r)

    def scale(ours, base):
        f = next(a / b for a, b in zip(ours, base) if b != 0)
        assert [f * b for b in base] == list(ours)
        return f
    for j in range(m + r - 1):
        a = scale([row[j] for row in AT], [row[j] for row in at])
        assert a * scale(G[j], g[j]) * scale(BT[j], bt[j]) == 1


def test_interpolation_construction_rejects_a_wrong_point():
    bt, g, at = wg.cook_toom([0, 1, -1, 3, -2, None], 4, 3)
    assert bt != wg.cook_toom(wg.POINTS[(4, 3)], 4, 3)[0]


@pytest.mark.parametrize("m,r", [(2, 3), (4, 3), (3, 2), (6, 3)])
def test_1d_matrix_form_is_exact_correlation(m, r):
    """Eq. (6) with the printed matrices equals the r-tap FIR filter exactly, using
    mu = m + r - 1 general multiplications (Eq. (3))."""
    rng = random.Random(100 * m + r)
    for _ in range(20):
        d = [_rand_frac(rng) for _ in range(m + r - 1)]
        g = [_rand_frac(rng) for _ in range(r)]
        y, nmul = wg.fir_1d(m, r, d, g)
        assert y == _corr1d(d, g, m)
        assert nmul == m + r - 1


@pytest.mark.parametrize("m,r", [(2, 3), (4, 3), (3, 2), (6, 3)])
def test_2d_nesting_is_exact_correlation(m, r):
    """Eq. (8) equals direct 2-D correlation exactly with (m+r-1)^2 multiplications (Eq. (4));
    16 vs 36 for F(2x2,3x3) and 36 vs 144 for F(4x4,3x3) (Sections 4.1, 4.3)."""
    rng = random.Random(7 * m + r)
    a = m + r - 1
    for _ in range(8):
        d = [[_rand_frac(rng) for _ in range(a)] for _ in range(a)]
        g = [[_rand_frac(rng) for _ in range(r)] for _ in range(r)]
        y, nmul = wg.fir_2d(m, r, d, g)
        assert y == _corr2d(d, g, m, m)
        assert nmul == a * a
    assert {2: 16, 4: 36, 3: 16, 6: 64}[m] == a * a
    if r == 3:
        assert Fr(m * m * 9, a * a) == {2: Fr(9, 4), 4: Fr(4), 6: Fr(81, 16)}[m]


def test_f23_printed_products():
    """The scalar form of F(2,3) printed in Eq. (5): m1..m4 and the two outputs."""
    rng = random.Random(23)
    BT, G, AT = wg.matrices(2, 3)
    for _ in range(20):
        d = [_rand_frac(rng) for _ in range(4)]
        g = [_rand_frac(rng) for _ in range(3)]
        m1 = (d[0] - d[2]) * g[0]
        m2 = (d[1] + d[2]) * (g[0] + g[1] + g[2]) / 2
        m3 = (d[2] - d[1]) * (g[0] - g[1] + g[2]) / 2
        m4 = (d[1] - d[3]) * g[2]
        Gg = [sum(G[i][j] * g[j] for j in range(3)) for i in range(4)]
        Bd = [sum(BT[i][j] * d[j] for j in range(4)) for i in range(4)]
        assert [a * b for a, b in zip(Gg, Bd)] == [m1, m2, m3, m4]
        assert wg.fir_1d(2, 3, d, g)[0] == [m1 + m2 + m3, m2 - m3 - m4]
        assert [m1 + m2 + m3, m2 - m3 - m4] == _corr1d(d, g, 2)


def test_matrix_shapes_and_a_transposed_operand_fails():
    for m in (2, 4, 6):
        BT, G, AT = wg.matrices(m)
        a = m + 2
        assert (len(BT), len(BT[0])) == (a, a)
        assert (len(G), len(G[0])) == (a, 3)
        assert (len(AT), len(AT[0])) == (m, a)
    # the pins above are sharp: swapping B^T for B breaks exactness
    BT, G, AT = wg.matrices(4)
    B = wg.transpose(BT)
    d = [[Fr(i * 6 + j + 1) for j in range(6)] for i in range(6)]
    g = [[Fr(3 * i + j + 1) for j in range(3)] for i in range(3)]
    u = wg.filter_transform_tile(4, g)
    bad = wg.inverse_transform_tile(4, wg.hadamard(u, wg.matmul(wg.matmul(B, d), BT)))
    assert bad != _corr2d(d, g, 4, 4)


@pytest.mark.parametrize("m", [2, 4, 6])
def test_delta_filter_tile_is_identity(m):
    """A filter that is 1 at its centre returns the centre m x m block of the tile."""
    a = m + 2
    d = [[Fr(7 * i - 3 * j + 1, 5) for j in range(a)] for i in range(a)]
    g = [[0, 0, 0], [0, 1, 0], [0, 0, 0]]
    y, _ = wg.fir_2d(m, 3, d, g)
    assert y == [[d[i + 1][j + 1] for j in range(m)] for i in range(m)]


@pytest.mark.parametrize("m", [2, 4, 6])
def test_tile_transform_linearity(m):
    rng = random.Random(m)
    a = m + 2
    d1 = [[_rand_frac(rng) for _ in range(a)] for _ in range(a)]
    d2 = [[_rand_frac(rng) for _ in range(a)] for _ in range(a)]
    s, t = Fr(3, 7), Fr(-5, 2)
    comb = [[s * x + t * y for x, y in zip(r1, r2)] for r1, r2 in zip(d1, d2)]
    v1, v2, vc = (wg.data_transform_tile(m, d) for d in (d1, d2, comb))
    assert vc == [[s * x + t * y for x, y in zip(r1, r2)] for r1, r2 in zip(v1, v2)]


@pytest.mark.parametrize("H,W,pad,m", [(56, 56, 1, 2), (28, 28, 1, 4), (14, 14, 1, 4), (14, 14, 1, 2),
                                       (224, 224, 1, 4), (7, 9, 1, 4), (7, 9, 0, 2), (5, 5, 0, 4),
                                       (56, 56, 1, 6), (14, 14, 1, 6), (9, 20, 0, 6)])
def test_tile_bookkeeping(H, W, pad, m):
    """Tiles cover every output exactly once; origins follow m*t - pad (Section 4.1's tiling)."""
    N = 2
    Ho, Wo = H + 2 * pad - 2, W + 2 * pad - 2
    Th, Tw = wg.tile_counts(H, W, pad, m)
    assert (Th, Tw) == (-(-Ho // m), -(-Wo // m))
    P = wg.num_tiles(N, H, W, pad, m)
    assert P == N * Th * Tw
    cover = np.zeros((N, Ho, Wo), dtype=int)
    seen = set()
    for b in range(P):
        i, tx, ty, x0, y0 = wg.tile_of(b, H, W, pad, m)
        assert 0 <= i < N and 0 <= tx < Th and 0 <= ty < Tw
        assert (x0, y0) == (m * tx - pad, m * ty - pad)
        assert b == (i * Th + tx) * Tw + ty
        seen.add((i, tx, ty))
        cover[i, m * tx:min(m * tx + m, Ho), m * ty:min(m * ty + m, Wo)] += 1
    assert len(seen) == P and (cover == 1).all()


@pytest.mark.parametrize("m", [2, 4, 6])
@pytest.mark.parametrize("shape", [(2, 3, 8, 8, 4, 1), (1, 2, 7, 9, 3, 1), (1, 2, 9, 6, 2, 0), (3, 1, 5, 5, 1, 1),
                                   (1, 2, 13, 20, 3, 1)])
def test_algorithm1_matches_direct_oracle(m, shape):
    """Algorithm 1 in float64 reproduces Eq. (1) (incl. ragged edge tiles) to rounding."""
    N, C, H, W, K, pad = shape
    rng = np.random.default_rng(m * 1000 + H)
    D = rng.standard_normal((N, C, H, W))
    G = rng.standard_normal((K, C, 3, 3))
    Y, U, V, M = wg.conv2d_fwd(D, G, pad, m)
    ref = direct.conv2d_fwd(D, G, pad=pad)
    a = m + 2
    P = wg.num_tiles(N, H, W, pad, m)
    assert U.shape == (a, a, K, C) and V.shape == (a, a, C, P) and M.shape == (a, a, K, P)
    assert Y.shape == ref.shape
    assert np.abs(Y - ref).max() <= 1e-12 * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("m", [2, 4])
def test_algorithm1_exact_on_integers(m):
    """With integer data and filters that are multiples of the transform denominators every
    stage is exact in float64, so Algorithm 1 equals Eq. (1) bit for bit."""
    rng = np.random.default_rng(5)
    D = rng.integers(-8, 9, size=(2, 3, 10, 10)).astype(np.float64)
    G = rng.integers(-4, 5, size=(4, 3, 3, 3)).astype(np.float64) * (4.0 if m == 2 else 576.0)
    Y, _, _, _ = wg.conv2d_fwd(D, G, 1, m)
    assert np.array_equal(Y, direct.conv2d_fwd(D, G, pad=1))


def test_stage_values_against_hand_computed_tile():
    """One F(2x2,3x3) tile by hand: d = outer(1..4, 1..4), g = all ones."""
    d = [[Fr((i + 1) * (j + 1)) for j in range(4)] for i in range(4)]
    g = [[Fr(1)] * 3 for _ in range(3)]
    # B^T (1,2,3,4) = (-2, 5, 1, -2); G (1,1,1) = (1, 3/2, 1/2, 1)
    bd = [Fr(-2), Fr(5), Fr(1), Fr(-2)]
    gg = [Fr(1), Fr(3, 2), Fr(1, 2), Fr(1)]
    assert wg.data_transform_tile(2, d) == [[x * y for y in bd] for x in bd]
    assert wg.filter_transform_tile(2, g) == [[x * y for y in gg] for x in gg]
    # outputs: sum of a 3x3 window of the outer product = (sum rows)(sum cols)
    assert wg.fir_2d(2, 3, d, g)[0] == [[Fr(36), Fr(54)], [Fr(54), Fr(81)]]


@pytest.mark.parametrize("shape", [(2, 3, 8, 8, 4), (1, 2, 7, 9, 3), (3, 1, 5, 6, 2), (1, 4, 14, 14, 5)])
def test_wgrad_f3x3_2x2_matches_direct_oracle(shape):
    """Section 4.2 / Eq. (14): 4 x 4 tiles overlapped by 2, 3 x 3 outputs summed over all tiles,
    reproduce the filter gradient of Eq. (1) (odd extents use zero-filled edge blocks)."""
    N, C, H, W, K = shape
    rng = np.random.default_rng(sum(shape))
    D = rng.standard_normal((N, C, H, W))
    E = rng.standard_normal((N, K, H, W))
    dG, Wt, V, M = wg.conv2d_bwd_filter(D, E, pad=1)
    ref = direct.conv2d_bwd_filter(D, E, pad=1)
    Bh, Bw = wg.wgrad_block_counts(H, W)
    assert Wt.shape == (4, 4, K, N * Bh * Bw) and V.shape == (4, 4, C, N * Bh * Bw) and M.shape == (4, 4, K, C)
    assert np.abs(dG - ref).max() <= 1e-12 * max(1.0, np.abs(ref).max())


def test_wgrad_exact_on_integers():
    rng = np.random.default_rng(3)
    D = rng.integers(-8, 9, (2, 3, 10, 12)).astype(np.float64)
    E = (rng.integers(-4, 5, (2, 4, 10, 12)) * 4).astype(np.float64)   # G of F(3,2) has halves
    dG, _, _, _ = wg.conv2d_bwd_filter(D, E, pad=1)
    assert np.array_equal(dG, direct.conv2d_bwd_filter(D, E, pad=1))

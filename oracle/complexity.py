"""TEST INFRASTRUCTURE ONLY: the paper's counting formulas, written out.

* mu(F(m,r)) and mu(F(m x n, r x s)): Section 4, Eq. (3) and Eq. (4).
* Normalised complexities alpha', beta', gamma', delta' of Section 5 (Eq. (20)-(23)), in
  the reading that reproduces Table 1: alpha = m + r - 1, alpha' = alpha^2 / m^2, and
  beta' = beta / alpha^2 (likewise gamma', delta'), with beta, gamma, delta the per-tile
  transform instruction counts stated in Section 4.1 and Section 4.3.
* Direct-convolution flop count behind Table 3 and the "effective TFLOPS" of Section 7.

Parity pins: tests/test_oracle_complexity.py against tests/golden/*.txt; Eq. (23) against the stage
counts of Eq. (19)-(21) expanded by hand at finite sizes; beta and delta against counted
factorisations of the transform matrices.  Parity unpinned: the filter-transform count gamma of
F(6x6,3x3) (see TRANSFORM_FLOPS).
"""

# per-tile transform instruction counts (data, filter, inverse), Sections 4.1 and 4.3.  For
# F(6x6,3x3) the text states no counts.  416 and 280 are what a counted straight-line evaluation
# of this file's neighbour's F(6,3) matrices costs when nested over the 8 x 8 tile (26 and 20
# instructions per 1-D transform, 16 resp. 14 of them per tile; tests/test_oracle_complexity.py
# counts them), and they give Table 1's row for tile 8 (6.50, 4.38) to its printed decimals.
# 143 (= 11 one-dimensional transforms of 13 instructions) is the only integer that rounds to the
# printed 2.23; the count depends on the row scaling of G, which the paper does not print for this
# algorithm, so it is taken from the table: PARITY UNPINNED for gamma of F(6x6,3x3) only.
TRANSFORM_FLOPS = {2: (32, 28, 24), 4: (156, 72, 100), 6: (416, 143, 280)}


def mu_1d(m, r):
    return m + r - 1


def mu_2d(m, n, r, s):
    return mu_1d(m, r) * mu_1d(n, s)


def normalized_complexity(m, r=3):
    a = m + r - 1
    beta, gamma, delta = TRANSFORM_FLOPS[m]
    return (a * a / (m * m), beta / (a * a), gamma / (a * a), delta / (a * a))


def layer_complexity(N, C, H, W, K, m, r=3):
    """Eq. (23): L = alpha'(1 + beta'/K + gamma'/P + delta'/C) N H W C K, no remainders assumed."""
    ap, bp, gp, dp = normalized_complexity(m, r)
    P = N * H * W / (m * m)
    return ap * (1 + bp / K + gp / P + dp / C) * N * H * W * C * K


def direct_flops(N, C, H, W, K, R=3, S=3):
    """2 flops per multiply-add of Eq. (1) with H x W outputs (the Table 3 convention)."""
    return 2 * N * K * C * R * S * H * W


# Table 3: (name, depth in network E, C, H=W, K)
VGG_E_LAYERS = [
    ("conv1.1", 1, 3, 224, 64), ("conv1.2", 1, 64, 224, 64), ("conv2.1", 1, 64, 112, 128),
    ("conv2.2", 1, 128, 112, 128), ("conv3.1", 1, 128, 56, 256), ("conv3.2", 3, 256, 56, 256),
    ("conv4.1", 1, 256, 28, 512), ("conv4.2", 3, 512, 28, 512), ("conv5", 4, 512, 14, 512),
]


def vgg_e_gflops(N=1):
    return [(n, d * direct_flops(N, C, HW, HW, K) / 1e9) for n, d, C, HW, K in VGG_E_LAYERS]


def effective_tflops(gflops, msec):
    """Section 7: direct-algorithm GFLOPs divided by run time in milliseconds."""
    return gflops / msec

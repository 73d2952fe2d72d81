"""TEST INFRASTRUCTURE ONLY: the minimal-filtering algorithm, stage by stage, on the CPU.

What is written out here, all from Section 4 of the paper:

* the transform matrices B^T, G, A^T of F(2,3) (Eq. (7)) and F(4,3) (Eq. (15)) as exact
  rationals, plus F(3,2) (Eq. (14)) which the weight-gradient variant uses;
* F(6,3), which Section 4.3 mentions (as F(6x6,3x3)) without printing matrices: they are
  built here by the construction Section 4 refers to (a minimal linear-convolution
  algorithm from polynomial evaluation and interpolation, transposed into a filtering
  algorithm; `cook_toom`) on the interpolation points 0, 1, -1, 2, -2, 1/2, -1/2 and
  infinity, the natural continuation of the points 0, 1, -1, 2, -2, infinity that
  reproduce Eq. (15); the row scaling between G and B^T, which the construction leaves
  free, is chosen so that B^T has the column of ones seen in Eq. (7) and Eq. (15);
* the 1-D matrix form Y = A^T[(G g) . (B^T d)] (Eq. (6)) and its 2-D nesting
  Y = A^T[[G g G^T] . [B^T d B]]A (Eq. (8)), usable on Fractions or floats;
* Algorithm 1 in its four loops -- filter transform and scatter to U, tile gather,
  data transform and scatter to V, the alpha^2 products M = U V (Eq. (13)), gather and
  inverse transform -- in numpy float64 with no blocking or fusion;
* the integer tile bookkeeping that Algorithm 1 leaves implicit.

Readings where the paper is silent: tiles per image are T_h x T_w with
T = ceil(out_extent / m); tile index b = (i*T_h + tx)*T_w + ty (ty fastest); the tile
origin in the input is (m*tx - pad, m*ty - pad); reads outside the image are zero;
outputs past the image edge are dropped.

Parity pins: tests/test_oracle_winograd.py (rational exactness against direct
correlation, the printed F(2,3) products m1..m4, multiplication counts, agreement with
the direct oracle).
"""
from fractions import Fraction as Fr

import numpy as np

_MATRICES = {
    # F(2,3), Eq. (7)
    (2, 3): dict(
        BT=[[1, 0, -1, 0],
            [0, 1, 1, 0],
            [0, -1, 1, 0],
            [0, 1, 0, -1]],
        G=[[Fr(1), 0, 0],
           [Fr(1, 2), Fr(1, 2), Fr(1, 2)],
           [Fr(1, 2), Fr(-1, 2), Fr(1, 2)],
           [0, 0, Fr(1)]],
        AT=[[1, 1, 1, 0],
            [0, 1, -1, -1]]),
    # F(4,3), Eq. (15)
    (4, 3): dict(
        BT=[[4, 0, -5, 0, 1, 0],
            [0, -4, -4, 1, 1, 0],
            [0, 4, -4, -1, 1, 0],
            [0, -2, -1, 2, 1, 0],
            [0, 2, -1, -2, 1, 0],
            [0, 4, 0, -5, 0, 1]],
        G=[[Fr(1, 4), 0, 0],
           [Fr(-1, 6), Fr(-1, 6), Fr(-1, 6)],
           [Fr(-1, 6), Fr(1, 6), Fr(-1, 6)],
           [Fr(1, 24), Fr(1, 12), Fr(1, 6)],
           [Fr(1, 24), Fr(-1, 12), Fr(1, 6)],
           [0, 0, Fr(1)]],
        AT=[[1, 1, 1, 1, 1, 0],
            [0, 1, -1, 2, -2, 0],
            [0, 1, 1, 4, 4, 0],
            [0, 1, -1, 8, -8, 1]]),
    # F(6,3): not printed in the paper (Section 4.3 defers it); from cook_toom() on the points
    # 0, 1, -1, 2, -2, 1/2, -1/2, infinity, scaled like Eq. (15); checked against the
    # construction and as an exact filter in tests/test_oracle_winograd.py
    (6, 3): dict(
        BT=[[1, 0, Fr(-21, 4), 0, Fr(21, 4), 0, -1, 0],
            [0, 1, 1, Fr(-17, 4), Fr(-17, 4), 1, 1, 0],
            [0, -1, 1, Fr(17, 4), Fr(-17, 4), -1, 1, 0],
            [0, Fr(1, 2), Fr(1, 4), Fr(-5, 2), Fr(-5, 4), 2, 1, 0],
            [0, Fr(-1, 2), Fr(1, 4), Fr(5, 2), Fr(-5, 4), -2, 1, 0],
            [0, 2, 4, Fr(-5, 2), -5, Fr(1, 2), 1, 0],
            [0, -2, 4, Fr(5, 2), -5, Fr(-1, 2), 1, 0],
            [0, -1, 0, Fr(21, 4), 0, Fr(-21, 4), 0, 1]],
        G=[[Fr(1), 0, 0],
           [Fr(-2, 9), Fr(-2, 9), Fr(-2, 9)],
           [Fr(-2, 9), Fr(2, 9), Fr(-2, 9)],
           [Fr(1, 90), Fr(1, 45), Fr(2, 45)],
           [Fr(1, 90), Fr(-1, 45), Fr(2, 45)],
           [Fr(32, 45), Fr(16, 45), Fr(8, 45)],
           [Fr(32, 45), Fr(-16, 45), Fr(8, 45)],
           [0, 0, Fr(1)]],
        AT=[[1, 1, 1, 1, 1, 1, 1, 0],
            [0, 1, -1, 2, -2, Fr(1, 2), Fr(-1, 2), 0],
            [0, 1, 1, 4, 4, Fr(1, 4), Fr(1, 4), 0],
            [0, 1, -1, 8, -8, Fr(1, 8), Fr(-1, 8), 0],
            [0, 1, 1, 16, 16, Fr(1, 16), Fr(1, 16), 0],
            [0, 1, -1, 32, -32, Fr(1, 32), Fr(-1, 32), 1]]),
    # F(3,2), Eq. (14)
    (3, 2): dict(
        BT=[[1, 0, -1, 0],
            [0, 1, 1, 0],
            [0, -1, 1, 0],
            [0, -1, 0, 1]],
        G=[[Fr(1), 0],
           [Fr(1, 2), Fr(1, 2)],
           [Fr(1, 2), Fr(-1, 2)],
           [0, Fr(1)]],
        AT=[[1, 1, 1, 0],
            [0, 1, -1, 0],
            [0, 1, 1, 1]]),
}


def matrices(m, r=3):
    """(B^T, G, A^T) of F(m, r) as lists of lists of Fractions."""
    e = _MATRICES[(m, r)]
    return tuple([[Fr(x) for x in row] for row in e[n]] for n in ("BT", "G", "AT"))


def matrices_f64(m, r=3):
    return tuple(np.array([[float(x) for x in row] for row in mat]) for mat in matrices(m, r))


# Interpolation points behind each matrix set (None = the point at infinity).
POINTS = {(2, 3): [0, 1, -1, None], (4, 3): [0, 1, -1, 2, -2, None], (3, 2): [0, 1, -1, None],
          (6, 3): [0, 1, -1, 2, -2, Fr(1, 2), Fr(-1, 2), None]}


def _inverse(A):
    """Exact inverse of a square matrix of Fractions (Gauss-Jordan)."""
    n = len(A)
    M = [[Fr(x) for x in row] + [Fr(int(i == j)) for j in range(n)] for i, row in enumerate(A)]
    for col in range(n):
        piv = next(r for r in range(col, n) if M[r][col] != 0)
        M[col], M[piv] = M[piv], M[col]
        M[col] = [x / M[col][col] for x in M[col]]
        for r in range(n):
            if r != col and M[r][col] != 0:
                f = M[r][col]
                M[r] = [x - f * y for x, y in zip(M[r], M[col])]
    return [row[n:] for row in M]


def cook_toom(points, m, r):
    """The construction Section 4 refers to, unscaled.  A product of polynomials of degrees
    r-1 and m-1 has n = m+r-1 coefficients; it is fixed by its values at n points (at
    infinity: its leading coefficient).  With E_k the n x k matrix that evaluates a polynomial
    with k coefficients at the points, linear convolution is s = E_n^-1 [(E_r g) . (E_m d)];
    exchanging the roles of d and s (transposition) gives the filter
    y = E_m^T [(E_r g) . (E_n^-T x)].  Returns (E_n^-T, E_r, E_m^T), i.e. B^T, G, A^T up to
    a scaling f_j of row j of G against 1/f_j of row j of B^T."""
    n = m + r - 1
    assert len(points) == n

    def evaluate(k):
        return [[Fr(int(j == k - 1)) if p is None else Fr(p) ** j for j in range(k)] for p in points]

    return transpose(_inverse(evaluate(n))), evaluate(r), transpose(evaluate(m))


# ---- tiny exact linear algebra on lists (works for Fractions, ints, floats) ----------------

def matmul(A, B):
    return [[sum(A[i][t] * B[t][j] for t in range(len(B))) for j in range(len(B[0]))]
            for i in range(len(A))]


def transpose(A):
    return [list(col) for col in zip(*A)]


def hadamard(A, B):
    return [[a * b for a, b in zip(ra, rb)] for ra, rb in zip(A, B)]


def fir_1d(m, r, d, g):
    """Eq. (6): the m outputs of an r-tap filter over m+r-1 inputs, via the transforms."""
    BT, G, AT = matrices(m, r)
    Gg = [sum(G[i][j] * g[j] for j in range(r)) for i in range(len(G))]
    Bd = [sum(BT[i][j] * d[j] for j in range(len(d))) for i in range(len(BT))]
    prod = [a * b for a, b in zip(Gg, Bd)]          # the m+r-1 general multiplications
    return [sum(AT[i][j] * prod[j] for j in range(len(prod))) for i in range(m)], len(prod)


def filter_transform_tile(m, g, r=3):
    """u = G g G^T (Algorithm 1, first loop) for one r x r filter."""
    _, G, _ = matrices(m, r)
    return matmul(matmul(G, g), transpose(G))


def data_transform_tile(m, d, r=3):
    """v = B^T d B (Algorithm 1, second loop) for one alpha x alpha tile."""
    BT, _, _ = matrices(m, r)
    return matmul(matmul(BT, d), transpose(BT))


def inverse_transform_tile(m, mm, r=3):
    """Y = A^T m A (Algorithm 1, fourth loop) for one alpha x alpha product tile."""
    _, _, AT = matrices(m, r)
    return matmul(matmul(AT, mm), transpose(AT))


def fir_2d(m, r, d, g):
    """Eq. (8): m x m outputs of an r x r filter over an alpha x alpha tile; also the
    number of general multiplications used."""
    u = filter_transform_tile(m, g, r)
    v = data_transform_tile(m, d, r)
    prod = hadamard(u, v)
    return inverse_transform_tile(m, prod, r), sum(len(row) for row in prod)


# ---- integer bookkeeping of Algorithm 1 ------------------------------------------------------

def tile_counts(H, W, pad, m, r=3):
    Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
    return -(-Ho // m), -(-Wo // m)


def num_tiles(N, H, W, pad, m, r=3):
    Th, Tw = tile_counts(H, W, pad, m, r)
    return N * Th * Tw


def tile_of(b, H, W, pad, m, r=3):
    """b -> (image, tile row, tile column, input row of the tile origin, input column)."""
    Th, Tw = tile_counts(H, W, pad, m, r)
    ty = b % Tw
    tx = (b // Tw) % Th
    i = b // (Tw * Th)
    return i, tx, ty, m * tx - pad, m * ty - pad


# ---- Algorithm 1, loop by loop, float64 ------------------------------------------------------

def filter_transform(G4, m):
    """Loop 1: U[xi,nu,k,c] = (G g_{k,c} G^T)[xi,nu]."""
    _, Gm, _ = matrices_f64(m)
    g = np.asarray(G4, dtype=np.float64)
    u = np.einsum("ai,kcij,bj->kcab", Gm, g, Gm)
    return np.ascontiguousarray(u.transpose(2, 3, 0, 1))


def gather_tiles(D4, pad, m, r=3):
    """The alpha x alpha input tiles d_{c,b} with r-1 overlap and zero fill: [C, P, alpha, alpha]."""
    D = np.asarray(D4, dtype=np.float64)
    N, C, H, W = D.shape
    a = m + r - 1
    Th, Tw = tile_counts(H, W, pad, m, r)
    tiles = np.zeros((C, N * Th * Tw, a, a))
    for b in range(N * Th * Tw):
        i, tx, ty, x0, y0 = tile_of(b, H, W, pad, m, r)
        for p in range(a):
            for q in range(a):
                x, y = x0 + p, y0 + q
                if 0 <= x < H and 0 <= y < W:
                    tiles[:, b, p, q] = D[i, :, x, y]
    return tiles


def data_transform(D4, pad, m):
    """Loop 2: V[xi,nu,c,b] = (B^T d_{c,b} B)[xi,nu]."""
    BT, _, _ = matrices_f64(m)
    d = gather_tiles(D4, pad, m)
    v = np.einsum("ai,cbij,ej->cbae", BT, d, BT)
    return np.ascontiguousarray(v.transpose(2, 3, 0, 1))


def multiply(U, V):
    """Loop 3: M^(xi,nu) = U^(xi,nu) V^(xi,nu), one K x C by C x P product per component."""
    a = U.shape[0]
    M = np.empty((a, a, U.shape[2], V.shape[3]))
    for xi in range(a):
        for nu in range(a):
            M[xi, nu] = U[xi, nu] @ V[xi, nu]
    return M


def inverse_transform(M, N, H, W, pad, m, r=3):
    """Loop 4: Y_{k,b} = A^T m_{k,b} A, written to Y[N,K,Ho,Wo] with edge outputs dropped."""
    _, _, AT = matrices_f64(m)
    K = M.shape[2]
    Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
    y = np.einsum("pa,abkt,qb->ktpq", AT, M, AT)
    Y = np.zeros((N, K, Ho, Wo))
    for b in range(M.shape[3]):
        i, tx, ty, _, _ = tile_of(b, H, W, pad, m, r)
        for p in range(m):
            for q in range(m):
                x, yy = m * tx + p, m * ty + q
                if x < Ho and yy < Wo:
                    Y[i, :, x, yy] = y[:, b, p, q]
    return Y


def conv2d_fwd(D4, G4, pad, m):
    """Algorithm 1 end to end; returns Y and the intermediates U, V, M."""
    N, C, H, W = np.shape(D4)
    U = filter_transform(G4, m)
    V = data_transform(D4, pad, m)
    M = multiply(U, V)
    return inverse_transform(M, N, H, W, pad, m), U, V, M


# ---- weight gradient with F(3x3, 2x2) (Section 4.2, Eq. (14)), loop by loop, float64 ---------------
#
# The error tensor is cut into 2 x 2 blocks e_{k,b}; block (bx, by) of image i pairs with the
# 4 x 4 input tile whose origin is (2*bx - pad, 2*by - pad) (tiles overlap by 2).  Each pair
# yields the 3 x 3 correlation of the tile with the block; the filter gradient is their sum
# over all blocks and images.  In transform space: w = G e G^T, v = B^T d B, M = sum_b w . v,
# dG = A^T M A, with the matrices of Eq. (14).  Readings where the paper is silent: blocks per
# image are ceil(H/2) x ceil(W/2); block index b = (i*Bh + bx)*Bw + by; error entries and
# input taps outside the tensors are zero.

def wgrad_block_counts(H, W):
    return -(-H // 2), -(-W // 2)


def wgrad_error_transform(E4):
    """W[xi,nu,k,b] = (G e_{k,b} G^T)[xi,nu] for every 2 x 2 block of the error tensor."""
    _, Gm, _ = matrices_f64(3, 2)
    E = np.asarray(E4, dtype=np.float64)
    N, K, H, W = E.shape
    Bh, Bw = wgrad_block_counts(H, W)
    Ep = np.zeros((N, K, 2 * Bh, 2 * Bw))
    Ep[:, :, :H, :W] = E
    blocks = Ep.reshape(N, K, Bh, 2, Bw, 2).transpose(1, 0, 2, 4, 3, 5).reshape(K, N * Bh * Bw, 2, 2)
    w = np.einsum("ai,kbij,ej->kbae", Gm, blocks, Gm)
    return np.ascontiguousarray(w.transpose(2, 3, 0, 1))


def wgrad_data_transform(D4, pad=1):
    """V[xi,nu,c,b] = (B^T d_{c,b} B)[xi,nu] for the 4 x 4 input tile of every error block."""
    BT, _, _ = matrices_f64(3, 2)
    D = np.asarray(D4, dtype=np.float64)
    N, C, H, W = D.shape
    Bh, Bw = wgrad_block_counts(H + 2 * pad - 2, W + 2 * pad - 2)
    tiles = np.zeros((C, N * Bh * Bw, 4, 4))
    for i in range(N):
        for bx in range(Bh):
            for by in range(Bw):
                b = (i * Bh + bx) * Bw + by
                for p in range(4):
                    for q in range(4):
                        x, y = 2 * bx - pad + p, 2 * by - pad + q
                        if 0 <= x < H and 0 <= y < W:
                            tiles[:, b, p, q] = D[i, :, x, y]
    v = np.einsum("ai,cbij,ej->cbae", BT, tiles, BT)
    return np.ascontiguousarray(v.transpose(2, 3, 0, 1))


def wgrad_multiply(Wt, V):
    """M^(xi,nu) = W^(xi,nu) (V^(xi,nu))^T: K x P by P x C, the reduction runs over blocks and images."""
    a = Wt.shape[0]
    M = np.empty((a, a, Wt.shape[2], V.shape[2]))
    for xi in range(a):
        for nu in range(a):
            M[xi, nu] = Wt[xi, nu] @ V[xi, nu].T
    return M


def wgrad_inverse_transform(M):
    """dG[k,c] = A^T m_{k,c} A (3 x 3 from 4 x 4)."""
    _, _, AT = matrices_f64(3, 2)
    return np.einsum("pa,abkc,qb->kcpq", AT, M, AT)


def conv2d_bwd_filter(D4, E4, pad=1):
    """The whole weight-gradient algorithm; returns dG[K,C,3,3] and the intermediates W, V, M."""
    Wt = wgrad_error_transform(E4)
    V = wgrad_data_transform(D4, pad)
    M = wgrad_multiply(Wt, V)
    return wgrad_inverse_transform(M), Wt, V, M

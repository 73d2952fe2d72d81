"""Seeded synthetic inputs and the layer shapes of the benchmark workloads.

Holds no arithmetic of the convolution method: only random tensors of the stated
distributions and the table of layer shapes.  The same arrays are handed to the GPU library
and to the CPU oracle by the tests and the benchmark.

Recipe: ``rng = numpy.random.default_rng(BASE_SEED + 1000*config + layer)``;
data ``D ~ N(0,1)`` drawn as float32; filters ``G ~ N(0,1) * sqrt(2/(9*C))`` (He scaling,
float32 multiply); fp16 workloads round both to float16 (round to nearest even).
"""
import numpy as np

BASE_SEED = 150909308

# VGG-16 3x3 convolution layers: (name, C, H=W, K).  Shapes as in Table 3 of the paper
# (network E has the same shapes with more repeats of 3.2, 4.2 and 5).
VGG16_LAYERS = [
    ("conv1.1", 3, 224, 64), ("conv1.2", 64, 224, 64),
    ("conv2.1", 64, 112, 128), ("conv2.2", 128, 112, 128),
    ("conv3.1", 128, 56, 256), ("conv3.2", 256, 56, 256), ("conv3.3", 256, 56, 256),
    ("conv4.1", 256, 28, 512), ("conv4.2", 512, 28, 512), ("conv4.3", 512, 28, 512),
    ("conv5.1", 512, 14, 512), ("conv5.2", 512, 14, 512), ("conv5.3", 512, 14, 512),
]

# Depth of each distinct layer shape in VGG network E (Table 3), keyed by (C, HW, K).
VGG_E_DEPTH = {(3, 224, 64): 1, (64, 224, 64): 1, (64, 112, 128): 1, (128, 112, 128): 1,
               (128, 56, 256): 1, (256, 56, 256): 3, (256, 28, 512): 1, (512, 28, 512): 3,
               (512, 14, 512): 4}


def layer_seed(config, layer):
    return BASE_SEED + 1000 * config + layer


def make_layer(N, C, H, W, K, seed, dtype=np.float32, R=3, S=3):
    """(D, G) for one layer, as numpy arrays of ``dtype``."""
    rng = np.random.default_rng(seed)
    D = rng.standard_normal((N, C, H, W), dtype=np.float32)
    G = rng.standard_normal((K, C, R, S), dtype=np.float32) * np.float32(np.sqrt(2.0 / (R * S * C)))
    return D.astype(dtype), G.astype(dtype)


def make_uniform_layer(N, C, H, W, K, seed, dtype=np.float32):
    """Data and filters uniform on [-1, 1] (the distribution of the paper's accuracy experiment)."""
    rng = np.random.default_rng(seed)
    D = rng.uniform(-1.0, 1.0, (N, C, H, W)).astype(np.float32)
    G = rng.uniform(-1.0, 1.0, (K, C, 3, 3)).astype(np.float32)
    return D.astype(dtype), G.astype(dtype)


def make_integer_layer(N, C, H, W, K, seed, dmax=8, gmax=4, gscale=1.0):
    """Small-integer data and filters (times ``gscale``): every stage is exact in fp32."""
    rng = np.random.default_rng(seed)
    D = rng.integers(-dmax, dmax + 1, (N, C, H, W)).astype(np.float32)
    G = (rng.integers(-gmax, gmax + 1, (K, C, 3, 3)) * gscale).astype(np.float32)
    return D, G


def sample_points(shape, n, seed, edge=0, planes=3):
    """n random (i, k, x, y) output coordinates of a tensor of ``shape``, plus its corners; with
    ``edge`` > 0 also every element of the last ``edge`` rows and the last ``edge`` columns (the
    last tile row and column of an algorithm with ``edge`` x ``edge`` output tiles) of ``planes``
    (i, k) planes: the first, the last and random ones."""
    rng = np.random.default_rng(seed)
    pts = np.stack([rng.integers(0, s, n) for s in shape], axis=1).astype(np.int32)
    corners = np.array([[a, b, c, d] for a in (0, shape[0] - 1) for b in (0, shape[1] - 1)
                        for c in (0, shape[2] - 1) for d in (0, shape[3] - 1)], dtype=np.int32)
    parts = [corners, pts]
    if edge > 0:
        N, K, H, W = shape
        ik = [(0, 0), (N - 1, K - 1)] + [(int(rng.integers(0, N)), int(rng.integers(0, K)))
                                         for _ in range(max(planes - 2, 0))]
        x0, y0 = max(H - edge, 0), max(W - edge, 0)
        for i, k in ik[:planes]:
            rows = [[i, k, x, y] for x in range(x0, H) for y in range(W)]
            cols = [[i, k, x, y] for x in range(x0) for y in range(y0, W)]
            parts.append(np.array(rows + cols, dtype=np.int32).reshape(-1, 4))
    return np.concatenate(parts, axis=0)

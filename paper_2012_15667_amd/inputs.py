"""Seeded synthetic conv-layer inputs shared by the tests, the smoke check and the benchmark.

This module only draws random numbers and names layer shapes.  It holds none of the method's
arithmetic, so both the CPU oracle's callers and the GPU library's callers can use it.

The layers are shaped like the CNN workloads the paper evaluates (3x3 stride-1 layers of
VGG/ResNet-style networks, Sec. 7.1 and 7.3; the AlexNet rows of Table 2).  Activations are
drawn uniform (post-ReLU-like [0,1] for the deep layers), weights He-style normal(0, sqrt(2/(C*R*S))).
"""
from collections import namedtuple

import numpy as np

Layer = namedtuple("Layer", "name algo N C H W K R S stride pad xdist wdist seed")

# algo: "direct", "wino2", "wino4";  xdist: "u11" uniform[-1,1], "u01" uniform[0,1];
# wdist: "u11" or "he" normal(0, sqrt(2/(C*R*S)))
CONFIGS = {
    "cfg1": Layer("cfg1", "direct", 1, 16, 14, 14, 16, 3, 3, 1, 1, "u11", "u11", 1001),
    "cfg2": Layer("cfg2", "wino2", 8, 64, 28, 28, 64, 3, 3, 1, 1, "u11", "he", 1002),
    "cfg3": Layer("cfg3", "direct", 32, 64, 56, 56, 64, 3, 3, 1, 1, "u01", "he", 1003),
    "cfg4": Layer("cfg4", "wino4", 64, 256, 14, 14, 256, 3, 3, 1, 1, "u01", "he", 1004),
    "cfg5a": Layer("cfg5a", "both", 64, 3, 224, 224, 64, 3, 3, 1, 1, "u01", "he", 1005),
    "cfg5b": Layer("cfg5b", "both", 64, 128, 112, 112, 128, 3, 3, 1, 1, "u01", "he", 1006),
    "cfg5c": Layer("cfg5c", "both", 64, 256, 56, 56, 256, 3, 3, 1, 1, "u01", "he", 1007),
    "cfg5d": Layer("cfg5d", "both", 64, 512, 28, 28, 512, 3, 3, 1, 1, "u01", "he", 1008),
    # AlexNet rows of Table 2 (batch is not stated there; 16 is used)
    "alex1": Layer("alex1", "direct", 16, 3, 227, 227, 96, 11, 11, 4, 0, "u01", "he", 1011),
    "alex2": Layer("alex2", "direct", 16, 96, 27, 27, 256, 5, 5, 1, 2, "u01", "he", 1012),
    "alex3": Layer("alex3", "both", 16, 256, 13, 13, 384, 3, 3, 1, 1, "u01", "he", 1013),
    "alex4": Layer("alex4", "both", 16, 384, 13, 13, 256, 3, 3, 1, 1, "u01", "he", 1014),
}


def _draw(rng, shape, dist, fan_in):
    if dist == "u11":
        return rng.uniform(-1.0, 1.0, size=shape)
    if dist == "u01":
        return rng.uniform(0.0, 1.0, size=shape)
    if dist == "he":
        return rng.normal(0.0, np.sqrt(2.0 / fan_in), size=shape)
    raise ValueError(dist)


def make_inputs(N, C, H, W, K, R, S, xdist="u11", wdist="u11", seed=0):
    """x [N][C][H][W] then w [K][C][R][S], drawn in fp64 from PCG64(seed) and cast to fp32."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = _draw(rng, (N, C, H, W), xdist, C * R * S).astype(np.float32)
    w = _draw(rng, (K, C, R, S), wdist, C * R * S).astype(np.float32)
    return x, w


def layer_inputs(layer):
    """Inputs of a named Layer (or its name)."""
    if isinstance(layer, str):
        layer = CONFIGS[layer]
    return make_inputs(layer.N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S,
                       layer.xdist, layer.wdist, layer.seed)


def sample_output_indices(N, K, P, Q, count, seed):
    """`count` random (n,k,p,q) output coordinates, always including the four corners of the
    first and last planes (the padded border is where indexing mistakes show)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    idx = np.stack([rng.integers(0, N, count), rng.integers(0, K, count),
                    rng.integers(0, P, count), rng.integers(0, Q, count)], axis=1).astype(np.int32)
    corners = [(n, k, p, q) for n in (0, N - 1) for k in (0, K - 1) for p in (0, P - 1) for q in (0, Q - 1)]
    idx[:len(corners)] = np.array(corners, dtype=np.int32)[:count]
    return idx

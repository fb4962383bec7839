"""Seeded synthetic inputs and the named parameter presets.

This module serves both the GPU library's tests/benchmark and the CPU oracle's
tests.  It holds NONE of the method's arithmetic: it only draws the random
numbers the scheme consumes (secret, errors, uniform polynomials, slot values,
layer weights, rotation offsets) and names the workload shapes.  Everything the
method computes from these draws is computed separately by each side.

Distributions (paper section 2.1 leaves them open; these are the readings used):
  secret s, encryption randomness r : i.i.d. uniform on {-1, 0, 1}
  errors e, e0, e1                  : round(N(0, 3.2^2)), redrawn while |e| > 19
  a (public key / switching keys)   : uniform on [0, q) per limb, independently
  slot values                       : uniform on the stated interval
  conv / FC weights                 : N(0, 0.05^2), encoded as round(w * q_last)
"""
from dataclasses import dataclass

import numpy as np

BASE_SEED = 20191126


@dataclass(frozen=True)
class Preset:
    name: str
    logN: int
    n_q: int
    q_bits: int
    k: int
    special_bits: int
    alpha: int
    log_scale: int
    batch: int

    @property
    def N(self):
        return 1 << self.logN


# the five workload shapes; k/alpha/special size where a shape leaves them open
# follow the hybrid form "alpha primes per digit, k = alpha special primes of
# q_bits+1 bits"
PRESETS = {
    "tiny": Preset("tiny", 12, 3, 40, 1, 41, 1, 30, 16),
    "hmul_rot_2e14": Preset("hmul_rot_2e14", 14, 8, 50, 1, 51, 1, 40, 256),
    "conv_2e15": Preset("conv_2e15", 15, 16, 50, 0, 51, 1, 40, 16384),
    "act_2e16": Preset("act_2e16", 16, 24, 50, 3, 51, 3, 50, 64),
    "cnn_2e16": Preset("cnn_2e16", 16, 30, 50, 3, 51, 3, 50, 32768),
}


def rng(seed, *stream):
    return np.random.Generator(np.random.Philox(key=[(BASE_SEED + int(seed)) & (2**64 - 1), hash_stream(stream)]))


def hash_stream(stream):
    h = 0xCBF29CE484222325
    for s in stream:
        for ch in str(s).encode():
            h = ((h ^ ch) * 0x100000001B3) & (2**64 - 1)
        h = ((h ^ 0xFF) * 0x100000001B3) & (2**64 - 1)
    return h


def ternary(N, seed, *stream):
    return rng(seed, "ternary", *stream).integers(-1, 2, size=N, dtype=np.int64)


def gaussian_error(shape, seed, *stream, sigma=3.2, bound=19):
    g = rng(seed, "error", *stream)
    e = np.rint(g.normal(0.0, sigma, size=shape)).astype(np.int64)
    bad = np.abs(e) > bound
    while bad.any():
        e[bad] = np.rint(g.normal(0.0, sigma, size=int(bad.sum()))).astype(np.int64)
        bad = np.abs(e) > bound
    return e


def uniform_limbs(moduli, N, seed, *stream, lead=()):
    """uint64 array [*lead][len(moduli)][N], limb i uniform on [0, moduli[i])."""
    g = rng(seed, "uniform", *stream)
    out = np.empty(tuple(lead) + (len(moduli), N), dtype=np.uint64)
    for i, q in enumerate(moduli):
        out[..., i, :] = g.integers(0, int(q), size=tuple(lead) + (N,), dtype=np.uint64)
    return out


def slots_complex(n_slots, seed, *stream, lo=-1.0, hi=1.0):
    g = rng(seed, "slots", *stream)
    return g.uniform(lo, hi, n_slots) + 1j * g.uniform(lo, hi, n_slots)


def slots_real(n_slots, seed, *stream, lo=-1.0, hi=1.0):
    return rng(seed, "slots", *stream).uniform(lo, hi, n_slots).astype(np.complex128)


def weights_float(shape, seed, *stream, sigma=0.05):
    return rng(seed, "weights", *stream).normal(0.0, sigma, size=shape)


def rotation_offsets(n_slots, count, seed):
    """`count` distinct slot offsets in [1, n_slots)."""
    g = rng(seed, "rot")
    return sorted(int(x) for x in g.choice(np.arange(1, n_slots), size=count, replace=False))


# ---------------------------------------------------------------------------
# Network shapes (layer lists only: no arithmetic of the method lives here)
# ---------------------------------------------------------------------------
# ("conv", out_channels, kernel, stride, pad) | ("square",) | ("poly2",) | ("pool", k[, pad]) | ("fc", out_features)
CNN_TOPOLOGIES = {
    # the AlexNet-like network of the 2^16 workload: 3x64x64 -> 32x30x30 -> 64x14x14 -> 64x14x14 -> pool 64x7x7 -> 256 -> 2
    "cnn_2e16": {"input": (3, 64, 64),
                 "layers": [("conv", 32, 5, 2, 0), ("square",), ("conv", 64, 3, 2, 0), ("square",), ("conv", 64, 3, 1, 1),
                            ("pool", 2), ("fc", 256), ("square",), ("fc", 2)]},
    # same layer sequence and depth, small enough for a CPU reference
    "cnn_reduced": {"input": (3, 16, 16),
                    "layers": [("conv", 6, 5, 2, 0), ("square",), ("conv", 8, 3, 2, 0), ("square",), ("conv", 8, 3, 1, 1),
                               ("pool", 2), ("fc", 16), ("square",), ("fc", 2)]},
    # the layer list of the paper's Table 1 on 3x32x32 inputs: zero-padding rows merged into the layer that follows
    # them, the degree-2 polynomial of section 3.1 after every conv / fc layer but the last (whose sigmoid is applied
    # after decryption): 32 -> 22 -> 11 -> 7 -> 3 -> 3 -> 1 -> 1 -> 1 -> 4096 -> 4096 -> 1
    "table1": {"input": (3, 32, 32),
               "layers": [("conv", 96, 11, 1, 0), ("poly2",), ("pool", 2), ("conv", 256, 5, 1, 0), ("poly2",), ("pool", 2),
                          ("conv", 384, 3, 1, 1), ("poly2",), ("pool", 2), ("conv", 384, 3, 1, 1), ("poly2",), ("pool", 2, 1),
                          ("fc", 4096), ("poly2",), ("fc", 4096), ("poly2",), ("fc", 1)]},
    # the same sequence at reduced width and input size (first kernel 5x5): 16 -> 12 -> 6 -> 4 -> 2 -> 2 -> 1 -> 1 -> 1
    "table1_reduced": {"input": (3, 16, 16),
                       "layers": [("conv", 1, 5, 1, 0), ("poly2",), ("pool", 2), ("conv", 9, 3, 1, 0), ("poly2",), ("pool", 2),
                                  ("conv", 4, 3, 1, 1), ("poly2",), ("pool", 2), ("conv", 4, 3, 1, 1), ("poly2",), ("pool", 2, 1),
                                  ("fc", 6), ("poly2",), ("fc", 6), ("poly2",), ("fc", 1)]},
    # a few layers of the same kinds for slow (emulated) checks: 6 -> 4 -> 2 -> 2 -> 2 (padded pooling) -> 2
    "table1_tiny": {"input": (2, 6, 6),
                    "layers": [("conv", 4, 3, 1, 0), ("poly2",), ("pool", 2), ("conv", 3, 3, 1, 1), ("poly2",), ("pool", 2, 1), ("fc", 2)]},
    # one image in the rotation-packed layout: strided convolution, activation, pooling merged into the layer after it
    "single_image_tiny": {"input": (2, 8, 8),
                          "layers": [("conv", 3, 3, 2, 1), ("poly2",), ("pool", 2), ("fc", 4), ("poly2",), ("fc", 2)]},
    # the same with the layer kinds and order of Table 1 at reduced width: 3x16x16 -> 4x12x12 -> 4x6x6 -> 6x4x4 -> 6x2x2 -> 16 -> 2
    "single_image_reduced": {"input": (3, 16, 16),
                             "layers": [("conv", 4, 5, 1, 0), ("poly2",), ("pool", 2), ("conv", 6, 3, 1, 0), ("poly2",), ("pool", 2),
                                        ("fc", 16), ("poly2",), ("fc", 2)]},
    # a 3x32x32 image (the input size of Table 1) through its layer kinds at small width:
    # 3x32x32 -> 8x28x28 -> 8x14x14 -> 16x10x10 -> 16x5x5 -> 64 -> 10; the longest vector (6272) fills the 8192 slots of N = 2^14
    "single_image_cifar": {"input": (3, 32, 32),
                           "layers": [("conv", 8, 5, 1, 0), ("poly2",), ("pool", 2), ("conv", 16, 5, 1, 0), ("poly2",), ("pool", 2),
                                      ("fc", 64), ("poly2",), ("fc", 10)]},
    "cnn_tiny": {"input": (3, 16, 16),
                 "layers": [("conv", 4, 5, 2, 0), ("square",), ("conv", 4, 3, 2, 0), ("square",), ("conv", 4, 3, 1, 1),
                            ("pool", 2), ("fc", 6), ("square",), ("fc", 2)]},
}


def cnn_shapes(name):
    """[(layer, input shape (C,H,W), output shape (C,H,W))] for a topology."""
    topo = CNN_TOPOLOGIES[name]
    c, h, w = topo["input"]
    out = []
    for layer in topo["layers"]:
        kind = layer[0]
        if kind == "conv":
            _, o, k, s, p = layer
            nxt = (o, (h + 2 * p - k) // s + 1, (w + 2 * p - k) // s + 1)
        elif kind == "pool":
            pad = layer[2] if len(layer) > 2 else 0
            nxt = (c, (h + 2 * pad) // layer[1], (w + 2 * pad) // layer[1])
        elif kind == "fc":
            nxt = (layer[1], 1, 1)
        else:
            nxt = (c, h, w)
        out.append((layer, (c, h, w), nxt))
        c, h, w = nxt
    return out


def cnn_weights_float(name, seed, sigma=0.05):
    """Float weights per layer (None for layers without weights): conv [O][C][k][k], fc [O][C*H*W]."""
    ws = []
    for li, (layer, (c, h, w), _) in enumerate(cnn_shapes(name)):
        if layer[0] == "conv":
            ws.append(weights_float((layer[1], c, layer[2], layer[2]), seed, "cnn", li, sigma=sigma))
        elif layer[0] == "fc":
            ws.append(weights_float((layer[1], c * h * w), seed, "cnn", li, sigma=sigma))
        else:
            ws.append(None)
    return ws


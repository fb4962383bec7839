"""Feed-forward CNN over per-pixel ciphertexts as a sequence of library calls (argument marshalling only).

The paper's network (section 3.1, Table 1) is a stack of convolution, average-pooling, polynomial-activation and
fully connected layers evaluated on encrypted inputs.  With one ciphertext per pixel / feature (slot s = image s)
  conv / fc : integer-weight multiply-accumulate of ciphertexts, then a rescale of every output    level l -> l-1
              (weight = round(w * q_{l-1}), so the scale is unchanged by the layer)
  square    : x^2 with relinearisation and rescale                                                level l -> l-1
  poly2     : c2*x^2 + c1*x, the degree-2 polynomial that replaces ReLU (section 3.1)             level l -> l-2
  pool k    : sum of the k*k ciphertexts of a window of the (zero-padded) map; the 1/k^2 of the average is folded
              into the next conv / fc layer's weights                                             level unchanged
Layers whose activations do not fit in device memory are run in strips of output rows (`conv_rows`).
"""
from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import activation, ckksmi


@dataclass
class LayerPlan:
    kind: str                    # "conv" | "square" | "poly2" | "pool" | "fc"
    in_shape: tuple              # (C, H, W) ciphertexts
    out_shape: tuple
    level_in: int
    level_out: int
    w_int: Optional[np.ndarray]  # conv: [O][C][k][k] int64, fc: [O][C*H*W] int64
    kernel: int = 0
    stride: int = 1
    pad: int = 0
    consts: object = None        # poly2: activation.Poly2Constants


def plan(shapes, weights_float, q, level, scale):
    """shapes: [(layer tuple, in (C,H,W), out (C,H,W))], layer tuples ("conv", O, k, stride, pad) | ("square",) |
    ("poly2",) | ("pool", k[, pad]) | ("fc", O); weights_float: per layer float array or None; q: ciphertext primes; level, scale: of the
    input.  Returns ([LayerPlan], output level, output scale)."""
    plans = []
    fold = 1.0
    for (layer, ishape, oshape), wf in zip(shapes, weights_float):
        kind = layer[0]
        if kind in ("conv", "fc"):
            if level < 2:
                raise ValueError("not enough levels for the network")
            wi = np.rint(np.asarray(wf, dtype=np.float64) * fold * float(q[level - 1])).astype(np.int64)
            fold = 1.0
            if kind == "conv":
                plans.append(LayerPlan("conv", ishape, oshape, level, level - 1, wi, layer[2], layer[3], layer[4]))
            else:
                plans.append(LayerPlan("fc", ishape, oshape, level, level - 1, wi))
            level -= 1
        elif kind == "square":
            if level < 2:
                raise ValueError("not enough levels for the network")
            plans.append(LayerPlan("square", ishape, oshape, level, level - 1, None))
            scale = scale * scale / float(q[level - 1])
            level -= 1
        elif kind == "poly2":
            if level < 3:
                raise ValueError("not enough levels for the network")
            consts = activation.poly2_constants(q, level, scale)
            plans.append(LayerPlan("poly2", ishape, oshape, level, level - 2, None, consts=consts))
            scale = consts.out_scale
            level -= 2
        elif kind == "pool":
            plans.append(LayerPlan("pool", ishape, oshape, level, level, None, layer[1], pad=layer[2] if len(layer) > 2 else 0))
            fold = fold / float(layer[1] * layer[1])
        else:
            raise ValueError(kind)
    if fold != 1.0:
        raise ValueError("a pooling layer must be followed by a conv or fc layer that absorbs its 1/k^2")
    return plans, level, scale


def workspace_bytes(ctx, plans, max_items=64):
    """Scratch for `forward`: the largest need over the layers, with key-switching sweeps of at most max_items."""
    need = 0
    for p in plans:
        n_out = int(np.prod(p.out_shape))
        if p.kind in ("conv", "fc"):
            if p.kind == "conv":
                need = max(need, ctx.conv2d_workspace_bytes(p.in_shape[0], p.out_shape[0], p.kernel, p.kernel, p.level_in))
            else:
                need = max(need, ctx.conv2d_workspace_bytes(int(np.prod(p.in_shape)), n_out, 1, 1, p.level_in))
            need = max(need, ctx.workspace_bytes(ckksmi.OP_RESCALE, p.level_in, min(n_out, max_items)))
        elif p.kind == "square":
            need = max(need, ctx.workspace_bytes(ckksmi.OP_HMUL_RELIN_RESCALE, p.level_in, min(n_out, max_items)))
        elif p.kind == "poly2":
            need = max(need, activation.workspace_bytes(ctx, p.level_in, min(n_out, max_items)))
    return need


def conv_rows(ctx, p, x_strip, w_dev, in_row0, in_rows, out_row0, out_rows, mac_out, out, ws, stream=None):
    """Output rows out_row0 .. +out_rows of conv layer p from a strip of input rows, MAC then rescale.
    x_strip: [C][in_rows][W] cts at p.level_in; mac_out: [O][out_rows][Wo] at p.level_in (scratch);
    out: [O][out_rows][Wo] at p.level_out."""
    C, H, W = p.in_shape
    O, _, Wo = p.out_shape
    ctx.conv2d_mac_rows(x_strip, w_dev, C, H, W, O, p.kernel, p.kernel, p.stride, p.pad, in_row0, in_rows, out_row0, out_rows, mac_out,
                        p.level_in, ws, stream=stream)
    ctx.rescale(mac_out, out, p.level_in, O * out_rows * Wo, ws, stream=stream)


def poly2_batch(ctx, p, x, evk, y, n_ct, ws, max_items=64, stream=None):
    """Layer p ("poly2") on n_ct ciphertexts, max_items at a time (the schedule's temporaries are sized per sweep).
    x, y: flat device arrays of n_ct ciphertexts at p.level_in / p.level_out."""
    wi, wo = 2 * p.level_in * ctx.N, 2 * p.level_out * ctx.N
    xf, yf = x.reshape(-1), y.reshape(-1)
    for b0 in range(0, n_ct, max_items):
        n = min(max_items, n_ct - b0)
        activation.poly2(ctx, xf[b0 * wi:(b0 + n) * wi], evk, yf[b0 * wo:(b0 + n) * wo], p.level_in, n, p.consts, ws, stream=stream)


def forward(ctx, x, plans, evk, empty, to_dev, ws, stream=None, max_items=64):
    """Whole network with every activation resident.  x: device array of [C][H][W] ciphertexts at plans[0].level_in;
    empty(*shape) allocates a device array of 64-bit words, to_dev(int64 ndarray) uploads weights; ws as sized by
    workspace_bytes(ctx, plans, max_items).  Returns the device array of the last layer's ciphertexts."""
    N = ctx.N
    for p in plans:
        n_out = int(np.prod(p.out_shape))
        if p.kind == "conv":
            C, H, W = p.in_shape
            O, Ho, Wo = p.out_shape
            mac = empty(n_out, 2, p.level_in, N)
            y = empty(n_out, 2, p.level_out, N)
            conv_rows(ctx, p, x, to_dev(p.w_int), 0, H, 0, Ho, mac, y, ws, stream=stream)
        elif p.kind == "fc":
            F = int(np.prod(p.in_shape))
            mac = empty(n_out, 2, p.level_in, N)
            y = empty(n_out, 2, p.level_out, N)
            ctx.fc_mac(x, to_dev(p.w_int), F, n_out, mac, p.level_in, ws, stream=stream)
            ctx.rescale(mac, y, p.level_in, n_out, ws, stream=stream)
        elif p.kind == "square":
            y = empty(n_out, 2, p.level_out, N)
            ctx.hmul_relin_rescale(x, x, evk, y, p.level_in, n_out, ws, stream=stream)
        elif p.kind == "poly2":
            y = empty(n_out, 2, p.level_out, N)
            poly2_batch(ctx, p, x, evk, y, n_out, ws, max_items, stream=stream)
        elif p.kind == "pool":
            C, H, W = p.in_shape
            y = empty(n_out, 2, p.level_out, N)
            ctx.sum_pool2d(x, C, H, W, p.kernel, y, p.level_in, stream=stream, pad=p.pad)
        else:
            raise ValueError(p.kind)
        x = y
    return x

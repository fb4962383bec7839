"""Rotation-packed (single-image) layers as sequences of library calls.

The throughput layout of the network puts one image per slot and one ciphertext per pixel.  For ONE image with low
latency (the paper reports minutes per image, section 3.2) the whole activation vector sits in the slots of a single
ciphertext instead, and a convolution or fully connected layer (Table 1) becomes a matrix-vector product evaluated
through rotations:
    M z = sum_d diag_d * roll(z, -d),      diag_d[i] = M[i][(i + d) mod n],
with z repeated over the slots with period n (n a power of two dividing N/2).  On ciphertexts:
    out = RS( sum_d pt_d * Rot_d(x) ),
pt_d the d-th diagonal encoded at scale q_{level-1} (so the rescale restores the input scale), Rot_d taken for all
d at once from ONE shared ModUp (ckksmi_rotate_hoisted), the products by ckksmi_mul_plain, the sum by ckksmi_add in
a pairwise tree, then ckksmi_rescale.  Only non-zero diagonals cost a rotation: a k x k convolution on a C x H x W
image has far fewer of them than a dense layer.

This module only plans (host side: matrices, diagonals, encodings) and marshals arguments; every step on
ciphertexts runs in the library's kernels.
"""
from dataclasses import dataclass

import numpy as np

from . import ckksmi

MAX_ROTATIONS_PER_CALL = 64  # distinct keys one ckksmi_rotate_hoisted call can address


def square_pad(M):
    """zero-pad a matrix to n x n, n the next power of two"""
    M = np.asarray(M, dtype=np.float64)
    n = 1
    while n < max(M.shape):
        n *= 2
    out = np.zeros((n, n))
    out[: M.shape[0], : M.shape[1]] = M
    return out


def matrix_diagonals(M, n_slots):
    """{d: diag_d tiled over n_slots} for the non-zero generalised diagonals of a square power-of-two matrix"""
    M = np.asarray(M, dtype=np.float64)
    n = M.shape[0]
    if M.shape != (n, n) or n_slots % n:
        raise ValueError("matrix must be square with a size that divides the slot count")
    rows = np.arange(n)
    out = {}
    for d in range(n):
        diag = M[rows, (rows + d) % n]
        if np.any(diag):
            out[d] = np.tile(diag, n_slots // n)
    return out


def conv_matrix(w, H, W, pad):
    """stride-1 convolution of a channel-major C x H x W vector as a matrix [O*Ho*Wo][C*H*W]"""
    w = np.asarray(w, dtype=np.float64)
    O, C, kh, kw = w.shape
    Ho, Wo = H + 2 * pad - kh + 1, W + 2 * pad - kw + 1
    M = np.zeros((O, Ho, Wo, C, H, W))
    ys, xs = np.arange(Ho), np.arange(Wo)
    for u in range(kh):
        iy = ys + u - pad
        vy = (iy >= 0) & (iy < H)
        for v in range(kw):
            ix = xs + v - pad
            vx = (ix >= 0) & (ix < W)
            for o in range(O):
                for c in range(C):
                    M[o, ys[vy][:, None], xs[vx][None, :], c, iy[vy][:, None], ix[vx][None, :]] += w[o, c, u, v]
    return M.reshape(O * Ho * Wo, C * H * W)


@dataclass
class LinearPlan:
    """a matrix prepared for one level: rotation offsets (non-zero diagonals) and their encoded plaintexts on the device"""
    level: int
    n: int
    rotations: list        # offsets d != 0, ascending
    pts: object            # device [len(rotations)][level][N], in the order of `rotations`
    pt0: object            # device [level][N] for d = 0, or None


def plan_linear(ctx, M, level, to_dev, encode=None):
    """Encode the diagonals of M (padded to a power of two) at scale q_{level-1}.  `encode(values, scale, level)` returns
    the plaintext [level][N] (default: the library's host encoder); `to_dev` uploads a uint64 array."""
    Msq = square_pad(M)
    diags = matrix_diagonals(Msq, ctx.N // 2)
    enc = encode or (lambda v, s, l: ctx.encode(v, s, l))
    scale = float(ctx.q[level - 1])
    rots = sorted(d for d in diags if d)
    pts = to_dev(np.stack([enc(diags[d].astype(np.complex128), scale, level) for d in rots])) if rots else None
    pt0 = to_dev(enc(diags[0].astype(np.complex128), scale, level)) if 0 in diags else None
    return LinearPlan(level, Msq.shape[0], rots, pts, pt0)


def workspace_bytes(ctx, plan, max_rotations=MAX_ROTATIONS_PER_CALL):
    """bytes for the `ws` argument of linear_transform (device scratch for the rotated copies, the rotations' own
    workspace, the running sum and the rescale)"""
    L, N = plan.level, ctx.N
    R = min(len(plan.rotations), max_rotations)
    ct = 2 * L * N * 8
    rot_ws = ctx.rotate_hoisted_workspace_bytes(L, 1, R) if R else 0
    return (R + 1) * ct + max(rot_ws, ctx.workspace_bytes(ckksmi.OP_RESCALE, L, 1))


def linear_transform(ctx, x, plan, out, ws, stream=None, max_rotations=MAX_ROTATIONS_PER_CALL):
    """out [2][level-1][N] = RS(sum_d pt_d * Rot_d(x)) for one ciphertext x [2][level][N] (device, torch-like buffers that
    support flat slicing).  The Galois keys of plan.rotations must be registered.  ws: workspace_bytes(ctx, plan).
    max_rotations: rotations per ckksmi_rotate_hoisted call (less workspace for a smaller value, more calls)."""
    if not 1 <= max_rotations <= MAX_ROTATIONS_PER_CALL:
        raise ValueError("max_rotations out of range")
    L, N = plan.level, ctx.N
    ct = 2 * L * N
    R_max = min(len(plan.rotations), max_rotations)
    flat = ws.reshape(-1) if hasattr(ws, "reshape") else ws
    rotated = flat[: R_max * ct]
    acc = flat[R_max * ct: (R_max + 1) * ct]
    rest = flat[(R_max + 1) * ct:]
    have_acc = False
    if plan.pt0 is not None:
        ctx.mul_plain(x, plan.pt0, 0, acc, L, 1, stream=stream)
        have_acc = True
    for c0 in range(0, len(plan.rotations), max_rotations):
        rots = plan.rotations[c0: c0 + max_rotations]
        R = len(rots)
        ctx.rotate_hoisted(x, rots, rotated, L, 1, rest, stream=stream)
        # every rotated copy times its diagonal: R items, plaintext r for item r
        pts = plan.pts.reshape(-1)[c0 * L * N: (c0 + R) * L * N]
        ctx.mul_plain(rotated, pts, L * N, rotated, L, R, stream=stream)
        # pairwise tree over the R products (modular addition: any order gives the same words)
        n = R
        while n > 1:
            h = n // 2
            ctx.add(rotated[: h * ct], rotated[(n - h) * ct: n * ct], rotated[: h * ct], L, h, stream=stream)
            n -= h
        if have_acc:
            ctx.add(acc, rotated[:ct], acc, L, 1, stream=stream)
        else:
            ctx.mul_scalar(rotated[:ct], 1, acc, L, 1, stream=stream)  # start of the running sum (a copy)
            have_acc = True
    if not have_acc:
        raise ValueError("the matrix has no non-zero diagonal")
    ctx.rescale(acc, out, L, 1, rest, stream=stream)

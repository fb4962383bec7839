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

Baby steps and giant steps (plan_bsgs, linear_transform_bsgs): with d = g*B + b,
    sum_d diag_d * Rot_d(x) = sum_g Rot_(g*B)( sum_b roll(diag_(g*B+b), +g*B) * Rot_b(x) ),
so a layer needs the keys of the baby offsets b < B (hoisted from one ModUp) and of the giant offsets g*B (one ordinary
rotation per inner sum, all in one batched call) -- about 2 sqrt(n) keys read per layer instead of n -- and its inner
sums are one launch of ckksmi_plain_mac over tables the plan uploads once.

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


def conv_matrix(w, H, W, pad, stride=1):
    """convolution (zero padding `pad`, stride `stride`) of a channel-major C x H x W vector as a matrix [O*Ho*Wo][C*H*W]"""
    w = np.asarray(w, dtype=np.float64)
    O, C, kh, kw = w.shape
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    M = np.zeros((O, Ho, Wo, C, H, W))
    ys, xs = np.arange(Ho), np.arange(Wo)
    for u in range(kh):
        iy = ys * stride + u - pad
        vy = (iy >= 0) & (iy < H)
        for v in range(kw):
            ix = xs * stride + v - pad
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


# ---------------------------------------------------------------------------------------------------------------------
# whole networks on one image: vectors that may span several ciphertexts, pooling and strided layers as matrices
# ---------------------------------------------------------------------------------------------------------------------
def pool_matrix(C, H, W, k, pad=0):
    """k x k average pooling of a channel-major C x H x W vector padded with `pad` zero rows / columns on every side, as a
    matrix [C*Ho*Wo][C*H*W] with entries 1/k^2, Ho = (H + 2 pad) // k"""
    Ho, Wo = (H + 2 * pad) // k, (W + 2 * pad) // k
    M = np.zeros((C, Ho, Wo, C, H, W))
    for u in range(k):
        iy = np.arange(Ho) * k + u - pad
        vy = (iy >= 0) & (iy < H)
        for v in range(k):
            ix = np.arange(Wo) * k + v - pad
            vx = (ix >= 0) & (ix < W)
            for c in range(C):
                M[c, np.arange(Ho)[vy][:, None], np.arange(Wo)[vx][None, :], c, iy[vy][:, None], ix[vx][None, :]] = 1.0 / (k * k)
    return M.reshape(C * Ho * Wo, C * H * W)


def stage_matrices(layer_shapes, weights):
    """[("linear", M) | ("poly2",)] for a layer list as workloads.cnn_shapes gives it: the linear layers between two
    activations (convolutions, poolings, fully connected layers) multiplied into one matrix each"""
    stages, pending = [], None
    for (layer, (c, h, w), _), wt in zip(layer_shapes, weights):
        kind = layer[0]
        if kind == "poly2":
            stages += [("linear", pending), ("poly2",)]
            pending = None
            continue
        if kind == "conv":
            M = conv_matrix(wt, h, w, layer[4], layer[3])
        elif kind == "pool":
            M = pool_matrix(c, h, w, layer[1], layer[2] if len(layer) > 2 else 0)
        elif kind == "fc":
            M = np.asarray(wt, dtype=np.float64)
        else:
            raise ValueError("layer kind %r has no matrix" % (kind,))
        pending = M if pending is None else M @ pending
    if pending is not None:
        stages.append(("linear", pending))
    return stages


def block_diagonals(M, n, n_slots):
    """{(i, j): {d: diagonal d of the n x n block (i, j) of M, tiled over the slots}}; M zero-padded to multiples of n"""
    M = np.asarray(M, dtype=np.float64)
    bo, bi = -(-M.shape[0] // n), -(-M.shape[1] // n)
    if n_slots % n or not (n == n_slots or (bo == 1 and bi == 1)):
        raise ValueError("several blocks need a block size equal to the slot count")
    P = np.zeros((bo * n, bi * n))
    P[: M.shape[0], : M.shape[1]] = M
    out = {}
    for i in range(bo):
        for j in range(bi):
            dg = matrix_diagonals(P[i * n:(i + 1) * n, j * n:(j + 1) * n], n_slots)
            if dg:
                out[(i, j)] = dg
    return out


@dataclass
class BlockPlan:
    """a matrix cut into blocks, prepared for one level"""
    level: int
    n_in: int
    n_out: int
    rotations: dict     # input block j -> ascending non-zero offsets any output block needs of it
    offsets: dict       # (i, j) -> ascending offsets (0 included) of that block
    pts: dict           # (i, j) -> device [len(offsets)][level][N] in that order


def plan_blocks(ctx, M, n, level, to_dev, encode=None):
    """encode the diagonals of every block of M at scale q_{level-1}"""
    dg = block_diagonals(M, n, ctx.N // 2)
    enc = encode or (lambda v, s, l: ctx.encode(v, s, l))
    scale = float(ctx.q[level - 1])
    n_out, n_in = 1 + max(i for i, _ in dg), -(-np.asarray(M).shape[1] // n)
    if sorted({i for i, _ in dg}) != list(range(n_out)):
        raise ValueError("an output block receives nothing")
    rots = {j: sorted({d for (_, jj), dd in dg.items() if jj == j for d in dd if d}) for j in range(n_in)}
    offsets = {ij: sorted(dd) for ij, dd in dg.items()}
    pts = {ij: to_dev(np.stack([enc(dg[ij][d].astype(np.complex128), scale, level) for d in offsets[ij]])) for ij in dg}
    return BlockPlan(level, n_in, n_out, rots, offsets, pts)


def blocks_workspace_bytes(ctx, plan, max_rotations=MAX_ROTATIONS_PER_CALL):
    L, N = plan.level, ctx.N
    R = max([min(len(r), max_rotations) for r in plan.rotations.values()] + [1])
    ct = 2 * L * N * 8
    rot_ws = ctx.rotate_hoisted_workspace_bytes(L, 1, R)
    return (2 * R + plan.n_out) * ct + max(rot_ws, ctx.workspace_bytes(ckksmi.OP_RESCALE, L, plan.n_out))


def linear_transform_blocks(ctx, xs, plan, out, ws, stream=None, max_rotations=MAX_ROTATIONS_PER_CALL):
    """out [n_out][2][level-1][N] = RS(sum_j sum_d pt_(i,j),d * Rot_d(xs[j])) for the input blocks xs [n_in][2][level][N].
    Every input block is rotated once (in calls of at most max_rotations offsets) for all output blocks."""
    L, N = plan.level, ctx.N
    ct = 2 * L * N
    flat = ws.reshape(-1) if hasattr(ws, "reshape") else ws
    xflat = xs.reshape(-1) if hasattr(xs, "reshape") else xs
    R_max = max([min(len(r), max_rotations) for r in plan.rotations.values()] + [1])
    rotated = flat[: R_max * ct]
    prod = flat[R_max * ct: 2 * R_max * ct]
    acc = flat[2 * R_max * ct: (2 * R_max + plan.n_out) * ct]
    rest = flat[(2 * R_max + plan.n_out) * ct:]
    started = [False] * plan.n_out

    def accumulate(i, src):
        a = acc[i * ct:(i + 1) * ct]
        if started[i]:
            ctx.add(a, src, a, L, 1, stream=stream)
        else:
            ctx.mul_scalar(src, 1, a, L, 1, stream=stream)  # start of the running sum (a copy)
            started[i] = True

    for j in range(plan.n_in):
        x = xflat[j * ct:(j + 1) * ct]
        for (i, jj), offs in sorted(plan.offsets.items()):
            if jj == j and offs and offs[0] == 0:
                ctx.mul_plain(x, plan.pts[(i, j)].reshape(-1)[: L * N], 0, prod[:ct], L, 1, stream=stream)
                accumulate(i, prod[:ct])
        rots_j = plan.rotations[j]
        for c0 in range(0, len(rots_j), max_rotations):
            chunk = rots_j[c0: c0 + max_rotations]
            ctx.rotate_hoisted(x, chunk, rotated, L, 1, rest, stream=stream)
            for (i, jj), offs in sorted(plan.offsets.items()):
                if jj != j:
                    continue
                # runs of consecutive rotated copies whose offsets this block has: one batched product per run
                m, k = 0, 0
                while k < len(chunk):
                    if chunk[k] not in offs:
                        k += 1
                        continue
                    k1 = k
                    p0 = offs.index(chunk[k])
                    while k1 + 1 < len(chunk) and p0 + (k1 + 1 - k) < len(offs) and offs[p0 + (k1 + 1 - k)] == chunk[k1 + 1]:
                        k1 += 1
                    run = k1 - k + 1
                    ctx.mul_plain(rotated[k * ct:(k1 + 1) * ct], plan.pts[(i, j)].reshape(-1)[p0 * L * N:(p0 + run) * L * N], L * N,
                                  prod[m * ct:(m + run) * ct], L, run, stream=stream)
                    m += run
                    k = k1 + 1
                if m == 0:
                    continue
                while m > 1:  # pairwise tree (modular addition: any order gives the same words)
                    h = m // 2
                    ctx.add(prod[: h * ct], prod[(m - h) * ct: m * ct], prod[: h * ct], L, h, stream=stream)
                    m -= h
                accumulate(i, prod[:ct])
    ctx.rescale(acc, out, L, plan.n_out, rest, stream=stream)


# ---------------------------------------------------------------- baby steps and giant steps
def bsgs_baby(n):
    """baby-step count for a matrix of period n: the power of two next to sqrt(n) from above"""
    return 1 << ((int(n - 1).bit_length() + 1) // 2)


@dataclass
class BsgsPlan:
    """a matrix cut into blocks, its offsets split as d = g*baby + b: every input block is rotated by its baby offsets
    from one shared ModUp, the products are summed per (output block, g), each such sum with g != 0 is rotated by g*baby,
    and the sums over g are rescaled.  About 2 sqrt(n) rotation keys (and key reads per image) instead of n."""
    level: int
    n_in: int
    n_out: int
    baby: int
    babies: dict        # input block j -> ascending non-zero baby offsets
    slot: dict          # (j, b) -> position of Rot_b(x_j) among the rotated copies (b = 0: the block itself)
    n_ct: int           # rotated copies in all
    groups: list        # [(i, g)] in table order: the groups with g = 0 first, then those that are rotated
    n_plain: int        # number of groups with g = 0
    terms: list         # [(i, j, g, b)] in table order
    pts: object         # device [len(terms)][level][N]: the encoded diagonals, rolled by g*baby slots
    term: object        # device int32 [len(groups)][n_ct]: the plaintext that multiplies rotated copy s in group k, -1 = none
    ones: object        # device [level][N] of ones: the plaintext 1 in evaluation form (summing groups = products with it)
    member: object      # device int32 [n_out][len(groups)]: 0 where group k belongs to output block i, -1 elsewhere

    def rotation_offsets(self):
        return sorted({b for bb in self.babies.values() for b in bb} | {g * self.baby for _, g in self.groups if g})


def _i32_table(values, to_dev):
    """an int32 table as a device buffer (carried in whole 64-bit words)"""
    a = np.zeros((len(values) + 1) // 2 * 2 + 2, dtype=np.int32)
    a[: len(values)] = values
    return to_dev(a.view(np.uint64))


def plan_bsgs(ctx, M, n, level, to_dev, encode=None, baby=None, encode_batch=None):
    """encode the diagonals of every block of M at scale q_{level-1} in baby-step / giant-step form.  encode_batch(vectors
    [T][N/2] of real slot values, scale, level) -> device [T][level][N], if given, encodes all of them at once (e.g. on
    the device, ckksmi_encode_device) instead of one host call per diagonal."""
    dg = block_diagonals(M, n, ctx.N // 2)
    baby = baby or bsgs_baby(n)
    enc = encode or (lambda v, s, l: ctx.encode(v, s, l))
    scale = float(ctx.q[level - 1])
    n_out, n_in = 1 + max(i for i, _ in dg), -(-np.asarray(M).shape[1] // n)
    if sorted({i for i, _ in dg}) != list(range(n_out)):
        raise ValueError("an output block receives nothing")
    babies = {j: sorted({d % baby for (_, jj), dd in dg.items() if jj == j for d in dd if d % baby}) for j in range(n_in)}
    slot, n_ct = {}, 0
    for j in range(n_in):
        for b in [0] + babies[j]:
            slot[(j, b)] = n_ct
            n_ct += 1
    keys = sorted({(i, d // baby) for (i, _), dd in dg.items() for d in dd})
    groups = [k for k in keys if k[1] == 0] + [k for k in keys if k[1] != 0]
    terms, vecs = [], []
    table = np.full((len(groups), n_ct), -1, dtype=np.int32)
    for k, (i, g) in enumerate(groups):
        for (ii, j), dd in sorted(dg.items()):
            if ii != i:
                continue
            for d in sorted(dd):
                if d // baby != g:
                    continue
                table[k, slot[(j, d % baby)]] = len(terms)
                terms.append((i, j, g, d % baby))
                vecs.append(np.roll(dd[d], g * baby) if encode_batch else enc(np.roll(dd[d], g * baby).astype(np.complex128), scale, level))
    member = np.full((n_out, len(groups)), -1, dtype=np.int32)
    for k, (i, g) in enumerate(groups):
        member[i, k] = 0
    return BsgsPlan(level, n_in, n_out, baby, babies, slot, n_ct, groups, sum(1 for _, g in groups if g == 0), terms,
                    encode_batch(np.stack(vecs), scale, level) if encode_batch else to_dev(np.stack(vecs)),
                    _i32_table(table.reshape(-1), to_dev), to_dev(np.ones((level, ctx.N), dtype=np.uint64)),
                    _i32_table(member.reshape(-1), to_dev))


def bsgs_workspace_bytes(ctx, plan, max_rotations=MAX_ROTATIONS_PER_CALL):
    L, N = plan.level, ctx.N
    ct = 2 * L * N * 8
    n_giant = len(plan.groups) - plan.n_plain
    R = max([min(len(b), max_rotations) for b in plan.babies.values()] + [1])
    aux = max(ctx.rotate_hoisted_workspace_bytes(L, 1, R), ctx.workspace_bytes(ckksmi.OP_ROTATE, L, max(n_giant, 1)),
              ctx.workspace_bytes(ckksmi.OP_RESCALE, L, plan.n_out))
    return (plan.n_ct + 2 * len(plan.groups) + plan.n_out) * ct + aux


def linear_transform_bsgs(ctx, xs, plan, out, ws, stream=None, max_rotations=MAX_ROTATIONS_PER_CALL):
    """out [n_out][2][level-1][N] = RS(sum_g Rot_(g*baby)(sum_j sum_b pt * Rot_b(xs[j]))) for the input blocks
    xs [n_in][2][level][N]"""
    L, N = plan.level, ctx.N
    ct = 2 * L * N
    flat = ws.reshape(-1) if hasattr(ws, "reshape") else ws
    xflat = xs.reshape(-1) if hasattr(xs, "reshape") else xs
    n_groups, n_giant = len(plan.groups), len(plan.groups) - plan.n_plain
    rotated = flat[: plan.n_ct * ct]
    inner = flat[plan.n_ct * ct: (plan.n_ct + n_groups) * ct]
    turned = flat[(plan.n_ct + n_groups) * ct: (plan.n_ct + 2 * n_groups) * ct]
    acc = flat[(plan.n_ct + 2 * n_groups) * ct: (plan.n_ct + 2 * n_groups + plan.n_out) * ct]
    rest = flat[(plan.n_ct + 2 * n_groups + plan.n_out) * ct:]
    # 1. the rotated copies of every input block: the block itself, then its baby offsets from one shared ModUp
    for j in range(plan.n_in):
        x = xflat[j * ct:(j + 1) * ct]
        s0 = plan.slot[(j, 0)]
        ctx.mul_scalar(x, 1, rotated[s0 * ct:(s0 + 1) * ct], L, 1, stream=stream)  # a copy
        bb = plan.babies[j]
        for c0 in range(0, len(bb), max_rotations):
            chunk = bb[c0: c0 + max_rotations]
            s1 = plan.slot[(j, chunk[0])]
            ctx.rotate_hoisted(x, chunk, rotated[s1 * ct:(s1 + len(chunk)) * ct], L, 1, rest, stream=stream)
    # 2. every inner sum in one launch
    ctx.plain_mac(rotated, plan.n_ct, plan.pts, len(plan.terms), plan.term, n_groups, inner, L, stream=stream)
    # 3. the sums with g = 0 as they are, those with g != 0 rotated by g*baby (one batch of ordinary rotations)
    if plan.n_plain:
        ctx.mul_scalar(inner[: plan.n_plain * ct], 1, turned[: plan.n_plain * ct], L, plan.n_plain, stream=stream)
    if n_giant:
        ctx.rotate(inner[plan.n_plain * ct:], [g * plan.baby for _, g in plan.groups[plan.n_plain:]], turned[plan.n_plain * ct:], L, n_giant, rest,
                   stream=stream)
    # 4. per output block the sum over g, as products with the plaintext 1 (modular additions: the same words in any
    #    order), then the rescale
    ctx.plain_mac(turned, n_groups, plan.ones, 1, plan.member, plan.n_out, acc, L, stream=stream)
    ctx.rescale(acc, out, L, plan.n_out, rest, stream=stream)


def network_period(stages, n_slots):
    longest = max(max(st[1].shape) for st in stages if st[0] == "linear")
    n = 1
    while n < longest:
        n *= 2
    return min(n, n_slots)


def plan_network(ctx, layer_shapes, weights, level, scale, to_dev, encode=None, bsgs=False, encode_batch=None):
    """plans of every stage of a network on one image (BlockPlan, or BsgsPlan with bsgs=True, or
    activation.Poly2Constants), the packing period, the output level and scale"""
    from . import activation
    stages = stage_matrices(layer_shapes, weights)
    n = network_period(stages, ctx.N // 2)
    plans = []
    for st in stages:
        if st[0] == "linear":
            plans.append(plan_bsgs(ctx, st[1], n, level, to_dev, encode, encode_batch=encode_batch) if bsgs else plan_blocks(ctx, st[1], n, level, to_dev, encode))
            level -= 1
        else:
            k = activation.poly2_constants(ctx.q, level, scale)
            plans.append(k)
            scale = k.out_scale
            level -= 2
    return plans, n, level, scale


def network_workspace_bytes(ctx, plans, level, max_rotations=MAX_ROTATIONS_PER_CALL):
    from . import activation
    need, blocks, N = 0, 1, ctx.N
    for pl in plans:
        if isinstance(pl, (BlockPlan, BsgsPlan)):
            need = max(need, bsgs_workspace_bytes(ctx, pl, max_rotations) if isinstance(pl, BsgsPlan) else blocks_workspace_bytes(ctx, pl, max_rotations))
            blocks = pl.n_out
            level -= 1
        else:
            need = max(need, activation.workspace_bytes(ctx, level, blocks))
            level -= 2
    # two ping-pong buffers for the activations between stages
    widest = max([pl.n_in for pl in plans if isinstance(pl, (BlockPlan, BsgsPlan))] + [pl.n_out for pl in plans if isinstance(pl, (BlockPlan, BsgsPlan))])
    return need + 2 * widest * 2 * ctx.n_q * N * 8


def run_network(ctx, xs, plans, evk, level, ws, stream=None, max_rotations=MAX_ROTATIONS_PER_CALL):
    """one image through the planned stages; xs [n_in][2][level][N]; returns (flat device view of the output blocks
    [n_out][2][level_out][N] inside ws, n_out, level_out)"""
    from . import activation
    N = ctx.N
    flat = ws.reshape(-1) if hasattr(ws, "reshape") else ws
    widest = max([pl.n_in for pl in plans if isinstance(pl, (BlockPlan, BsgsPlan))] + [pl.n_out for pl in plans if isinstance(pl, (BlockPlan, BsgsPlan))])
    half = widest * 2 * ctx.n_q * N
    bufs = [flat[:half], flat[half: 2 * half]]
    rest = flat[2 * half:]
    cur, which = xs, 0
    blocks = None
    for pl in plans:
        dst = bufs[which]
        if isinstance(pl, (BlockPlan, BsgsPlan)):
            fn = linear_transform_bsgs if isinstance(pl, BsgsPlan) else linear_transform_blocks
            fn(ctx, cur, pl, dst[: pl.n_out * 2 * (level - 1) * N], rest, stream=stream, max_rotations=max_rotations)
            blocks = pl.n_out
            level -= 1
            cur = dst[: blocks * 2 * level * N]
        else:
            activation.poly2(ctx, cur, evk, dst[: blocks * 2 * (level - 2) * N], level, blocks, pl, rest, stream=stream)
            level -= 2
            cur = dst[: blocks * 2 * level * N]
        which ^= 1
    return cur, blocks, level

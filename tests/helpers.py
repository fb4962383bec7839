"""Shared test scaffolding: builds seeded key material and ciphertexts with the
CPU oracle from the draws of the neutral input module."""
import numpy as np

from oracle import oracle as orc
from paper_1911_11377_amd import workloads as wl


class Material:
    """Oracle-side parameter set + keys for one seeded instance."""

    def __init__(self, logN, n_q, q_bits, k, special_bits, alpha, seed, rotations=()):
        self.O = orc.Oracle(logN, n_q, q_bits, k, special_bits, alpha)
        O = self.O
        self.seed = seed
        self.logN, self.N = logN, 1 << logN
        T = n_q + k
        self.s = wl.ternary(O.N, seed, "s")
        a = wl.uniform_limbs(O.q, O.N, seed, "pk.a")
        e = wl.gaussian_error(O.N, seed, "pk.e")
        self.pk = O.keygen_public(self.s, a, e)
        self.rlk = None
        self.gk = {}
        if k > 0:
            self.rlk_a = wl.uniform_limbs(O.moduli, O.N, seed, "rlk.a", lead=(O.beta_top,))
            self.rlk_e = wl.gaussian_error((O.beta_top, O.N), seed, "rlk.e")
            self.rlk = O.keygen_relin(self.s, self.rlk_a, self.rlk_e)
            for r in rotations:
                ga = wl.uniform_limbs(O.moduli, O.N, seed, "gk.a", r, lead=(O.beta_top,))
                ge = wl.gaussian_error((O.beta_top, O.N), seed, "gk.e", r)
                self.gk[r] = O.keygen_galois(self.s, orc.galois_element(logN, r), ga, ge)

    def encode(self, z, scale, level):
        coeffs = orc.encode(z, scale, self.logN)
        rns = orc.to_rns(coeffs, self.O.q[:level])
        return self.O.ntt_limbs(rns, list(range(level)))

    def encrypt(self, z, scale, level, tag):
        pt = self.encode(z, scale, level)
        r = wl.ternary(self.N, self.seed, "enc.r", tag)
        e0 = wl.gaussian_error(self.N, self.seed, "enc.e0", tag)
        e1 = wl.gaussian_error(self.N, self.seed, "enc.e1", tag)
        return self.O.encrypt(self.pk, pt, r, e0, e1, level)

    def decrypt_poly(self, ct, level):
        """centred big-integer coefficients of c0 + c1*s (+ c2*s^2)"""
        m = self.O.decrypt(self.s, ct, level)
        return orc.crt_reconstruct(m, self.O.q[:level])

    def decrypt(self, ct, scale, level):
        return orc.decode(self.decrypt_poly(ct, level), scale, self.logN)


def poly_mul_negacyclic_int(a, b):
    """exact integer negacyclic product of two lists of Python ints (tiny N only)"""
    n = len(a)
    out = [0] * n
    for i in range(n):
        if a[i] == 0:
            continue
        for j in range(n):
            k = i + j
            if k < n:
                out[k] += a[i] * b[j]
            else:
                out[k - n] -= a[i] * b[j]
    return out


# ---------------------------------------------------------------------------
# single-image (rotation-packed) networks: test-side planning from the oracle's definitions
# ---------------------------------------------------------------------------
PAPER_C2, PAPER_C1 = 0.000469841857369822, 0.500000000000008  # section 3.1, tests/golden/activation_poly_deg2.txt


def network_stage_matrices(topology, weights):
    """[("linear", M) | ("poly2",)]: the linear layers between two activations multiplied into one matrix (convolution and
    pooling matrices from the oracle's definitions, fully connected layers as they are)"""
    stages, pending = [], None
    for (layer, (c, h, w), _), wt in zip(wl.cnn_shapes(topology), weights):
        kind = layer[0]
        if kind == "poly2":
            stages += [("linear", pending), ("poly2",)]
            pending = None
            continue
        if kind == "conv":
            M = orc.conv_as_matrix(wt, h, w, layer[4], layer[3])
        elif kind == "pool":
            M = orc.pool_as_matrix(c, h, w, layer[1], layer[2] if len(layer) > 2 else 0)
        elif kind == "fc":
            M = np.asarray(wt, dtype=np.float64)
        else:
            raise ValueError(kind)
        pending = M if pending is None else M @ pending
    if pending is not None:
        stages.append(("linear", pending))
    return stages


def network_float(stages, z):
    """the same stages on a plain float vector"""
    for st in stages:
        z = st[1] @ z if st[0] == "linear" else PAPER_C2 * z * z + PAPER_C1 * z
    return z


def network_period(stages, n_slots):
    """the slot period of the packing: the next power of two above every vector length, at most the slot count"""
    longest = max(max(st[1].shape) for st in stages if st[0] == "linear")
    n = 1
    while n < longest:
        n *= 2
    return min(n, n_slots)


def bsgs_baby(n):
    """baby-step count for a matrix of period n: the power of two next to sqrt(n) from above"""
    return 1 << ((int(n - 1).bit_length() + 1) // 2)


def network_integer_stages(stages, q, level, scale, n, n_slots, encode, bsgs=False):
    """the stages as the oracle's packed_network takes them: encoded diagonals (scale q_{level-1}, so that the rescale
    restores the scale) and the integer constants of the degree-2 activation from the tracked scale; bsgs: the linear
    stages in baby-step / giant-step form (pre-rotated diagonals, baby = bsgs_baby(n)).  Returns
    (stages, rotation offsets used, output level, output scale)."""
    out, rots = [], set()
    for st in stages:
        if st[0] == "linear":
            dg = orc.block_diagonals(st[1], n, n_slots)
            if bsgs:
                baby = bsgs_baby(n)
                bs = orc.bsgs_diagonals(dg, baby)
                out.append(("linear_bsgs", {ij: {gb: encode(v.astype(np.complex128), float(q[level - 1]), level) for gb, v in dd.items()} for ij, dd in bs.items()}, baby))
                rots |= {b for dd in bs.values() for (_, b) in dd if b} | {g * baby for dd in bs.values() for (g, _) in dd if g}
            else:
                out.append(("linear", {ij: {d: encode(v.astype(np.complex128), float(q[level - 1]), level) for d, v in dd.items()} for ij, dd in dg.items()}))
                rots |= {d for dd in dg.values() for d in dd if d}
            level -= 1
        else:
            s2 = scale * scale / float(q[level - 1])
            out.append(("poly2", round(PAPER_C2 * float(q[level - 2])), round(PAPER_C1 * (s2 / scale) * float(q[level - 2]))))
            scale = s2
            level -= 2
    return out, sorted(rots), level, scale

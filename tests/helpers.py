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

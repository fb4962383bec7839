"""Python face of the CPU oracle.  TEST INFRASTRUCTURE ONLY (see ckks_oracle.c).

Two layers:
  * ctypes bindings to the plain-C oracle (``libckks_oracle.so``) for everything
    that is integer arithmetic mod q_i;
  * pure Python / numpy pieces that need big integers or floating point:
    CRT reconstruction, the CKKS encoding map of the paper's section 2.1
    (m = round(scale * phi^-1(z)), phi = evaluation at the primitive roots
    zeta^(5^k), zeta = exp(i*pi/N)), decoding, and the activation schedules
    (compositions of the C operations).

Nothing here imports the GPU package.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

u64p = C.POINTER(C.c_uint64)
i64p = C.POINTER(C.c_int64)
intp = C.POINTER(C.c_int)


def lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.orc_addmod.restype = C.c_uint64
        L.orc_addmod.argtypes = [C.c_uint64] * 3
        L.orc_submod.restype = C.c_uint64
        L.orc_submod.argtypes = [C.c_uint64] * 3
        L.orc_mulmod.restype = C.c_uint64
        L.orc_mulmod.argtypes = [C.c_uint64] * 3
        L.orc_powmod.restype = C.c_uint64
        L.orc_powmod.argtypes = [C.c_uint64] * 3
        L.orc_invmod.restype = C.c_uint64
        L.orc_invmod.argtypes = [C.c_uint64] * 2
        L.orc_signed_mod.restype = C.c_uint64
        L.orc_signed_mod.argtypes = [C.c_int64, C.c_uint64]
        L.orc_is_prime.restype = C.c_int
        L.orc_is_prime.argtypes = [C.c_uint64]
        L.orc_find_primes.restype = C.c_int
        L.orc_find_primes.argtypes = [C.c_int, C.c_int, C.c_int, u64p, C.c_int, u64p]
        L.orc_find_psi.restype = C.c_uint64
        L.orc_find_psi.argtypes = [C.c_uint64, C.c_int]
        L.orc_brev.restype = C.c_uint64
        L.orc_brev.argtypes = [C.c_uint64, C.c_int]
        L.orc_galois_element.restype = C.c_uint64
        L.orc_galois_element.argtypes = [C.c_int, C.c_int64]
        L.orc_params_new.restype = C.c_void_p
        L.orc_params_new.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, u64p, u64p]
        L.orc_params_free.restype = None
        L.orc_params_free.argtypes = [C.c_void_p]
        for name in ("orc_ntt_direct", "orc_intt_direct"):
            getattr(L, name).restype = None
            getattr(L, name).argtypes = [u64p, C.c_int, C.c_uint64, C.c_uint64, u64p]
        L.orc_negacyclic_schoolbook.restype = None
        L.orc_negacyclic_schoolbook.argtypes = [u64p, u64p, C.c_int, C.c_uint64, u64p]
        for name in ("orc_ntt", "orc_intt"):
            getattr(L, name).restype = None
            getattr(L, name).argtypes = [u64p, C.c_int, C.c_uint64, C.c_uint64]
        _LIB = L
    return _LIB


def _p64(a):
    assert a.dtype == np.uint64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(u64p)


def _pi64(a):
    assert a.dtype == np.int64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(i64p)


def _pint(a):
    assert a.dtype == np.int32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(intp)


def _u64(a):
    return np.ascontiguousarray(a, dtype=np.uint64)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


# --------------------------------------------------------------------------
# scalar helpers
# --------------------------------------------------------------------------
def mulmod(a, b, q):
    return int(lib().orc_mulmod(int(a), int(b), int(q)))


def powmod(a, e, q):
    return int(lib().orc_powmod(int(a), int(e), int(q)))


def invmod(a, q):
    return int(lib().orc_invmod(int(a), int(q)))


def is_prime(n):
    return bool(lib().orc_is_prime(int(n)))


def brev(x, bits):
    return int(lib().orc_brev(int(x), int(bits)))


def find_primes(bits, logN, count, exclude=()):
    out = np.zeros(max(count, 1), dtype=np.uint64)
    ex = _u64(list(exclude) if len(exclude) else [0])
    n = lib().orc_find_primes(bits, logN, count, _p64(ex), len(exclude), _p64(out))
    if n != count:
        raise ValueError("only %d primes of %d bits found" % (n, bits))
    return [int(x) for x in out[:count]]


def find_psi(q, logN):
    return int(lib().orc_find_psi(int(q), logN))


def galois_element(logN, r):
    return int(lib().orc_galois_element(logN, int(r)))


# --------------------------------------------------------------------------
# single-limb transforms and the definitions they are pinned to
# --------------------------------------------------------------------------
def ntt_direct(a, logN, q, psi):
    a = _u64(a)
    out = np.empty_like(a)
    lib().orc_ntt_direct(_p64(a), logN, q, psi, _p64(out))
    return out


def intt_direct(a, logN, q, psi):
    a = _u64(a)
    out = np.empty_like(a)
    lib().orc_intt_direct(_p64(a), logN, q, psi, _p64(out))
    return out


def negacyclic_schoolbook(a, b, logN, q):
    a, b = _u64(a), _u64(b)
    out = np.empty_like(a)
    lib().orc_negacyclic_schoolbook(_p64(a), _p64(b), logN, q, _p64(out))
    return out


def ntt(a, logN, q, psi):
    a = _u64(a).copy()
    lib().orc_ntt(_p64(a), logN, q, psi)
    return a


def intt(a, logN, q, psi):
    a = _u64(a).copy()
    lib().orc_intt(_p64(a), logN, q, psi)
    return a


# --------------------------------------------------------------------------
# parameter set + ciphertext arithmetic
# --------------------------------------------------------------------------
class Oracle:
    """One RNS-CKKS parameter set; every method is a thin call into the C oracle.

    Primes: the n_q largest q_bits-bit primes = 1 mod 2N (descending), then the k
    largest special_bits-bit ones; psi_i = first x >= 2 with x^((q-1)/2N) of
    order exactly 2N.  `moduli`/`psis` may be given instead to force a basis.
    """

    def __init__(self, logN, n_q, q_bits, k, special_bits, alpha, moduli=None, psis=None):
        L = lib()
        self.logN, self.N = logN, 1 << logN
        self.n_q, self.k, self.alpha = n_q, k, max(alpha, 1)
        if moduli is None:
            q = find_primes(q_bits, logN, n_q)
            p = find_primes(special_bits, logN, k, exclude=q) if k else []
            moduli = q + p
        if psis is None:
            psis = [find_psi(m, logN) for m in moduli]
        self.moduli = [int(m) for m in moduli]
        self.psis = [int(x) for x in psis]
        self.q = self.moduli[:n_q]
        self.p = self.moduli[n_q:]
        self.beta_top = (n_q + self.alpha - 1) // self.alpha
        m = _u64(self.moduli)
        s = _u64(self.psis)
        self._h = C.c_void_p(L.orc_params_new(logN, n_q, k, self.alpha, _p64(m), _p64(s)))
        self._L = L
        V = C.c_void_p
        I = C.c_int
        sig = {
            "orc_ntt_limb": [V, I, u64p],
            "orc_intt_limb": [V, I, u64p],
            "orc_small_to_eval": [V, i64p, intp, I, u64p],
            "orc_keygen_public": [V, i64p, u64p, i64p, u64p],
            "orc_keygen_switch": [V, i64p, u64p, u64p, i64p, u64p],
            "orc_encrypt": [V, u64p, u64p, i64p, i64p, i64p, I, u64p],
            "orc_decrypt": [V, i64p, u64p, I, I, u64p],
            "orc_tensor": [V, u64p, u64p, I, u64p],
            "orc_modup": [V, u64p, I, I, u64p],
            "orc_divround_coef": [V, u64p, intp, I, intp, I, u64p],
            "orc_divround_exact_coef": [V, u64p, intp, I, intp, I, u64p],
            "orc_keyswitch": [V, u64p, u64p, I, u64p],
            "orc_relin": [V, u64p, u64p, I, u64p],
            "orc_rescale": [V, u64p, I, u64p],
            "orc_hmul_relin_rescale": [V, u64p, u64p, u64p, I, u64p],
            "orc_hmul_relin_rescale_merged": [V, u64p, u64p, u64p, I, u64p],
            "orc_hmul_sum_relin_rescale": [V, u64p, u64p, I, u64p, I, u64p],
            "orc_rotate": [V, u64p, C.c_uint64, u64p, I, u64p],
            "orc_rotate_hoisted": [V, u64p, I, I, u64p, u64p, u64p],
            "orc_add": [V, u64p, u64p, I, u64p],
            "orc_sub": [V, u64p, u64p, I, u64p],
            "orc_mul_plain": [V, u64p, u64p, I, u64p],
            "orc_mul_scalar": [V, u64p, C.c_int64, I, u64p],
            "orc_add_const": [V, u64p, C.c_int64, I, u64p],
            "orc_conv2d_mac": [V, u64p, i64p] + [I] * 8 + [I, u64p],
            "orc_fc_mac": [V, u64p, i64p, I, I, I, u64p],
            "orc_sum_pool2d": [V, u64p, I, I, I, I, I, I, u64p],
        }
        for name, args in sig.items():
            f = getattr(L, name)
            f.restype = None
            f.argtypes = args
        L.orc_automorphism_small.restype = None
        L.orc_automorphism_small.argtypes = [i64p, I, C.c_uint64, i64p]
        L.orc_automorphism_coef.restype = None
        L.orc_automorphism_coef.argtypes = [u64p, I, C.c_uint64, C.c_uint64, u64p]
        L.orc_automorphism_eval.restype = None
        L.orc_automorphism_eval.argtypes = [u64p, I, C.c_uint64, u64p]

    def __del__(self):
        try:
            self._L.orc_params_free(self._h)
        except Exception:
            pass

    # ---- basis bookkeeping ----
    def ext_moduli(self, level):
        return self.q[:level] + self.p

    def beta(self, level):
        return (level + self.alpha - 1) // self.alpha

    # ---- transforms on [.., N] arrays whose limb t uses modulus index idx[t] ----
    def ntt_limbs(self, a, idx):
        a = _u64(a).copy().reshape(len(idx), self.N)
        for r, t in enumerate(idx):
            self._L.orc_ntt_limb(self._h, int(t), _p64(a[r]))
        return a

    def intt_limbs(self, a, idx):
        a = _u64(a).copy().reshape(len(idx), self.N)
        for r, t in enumerate(idx):
            self._L.orc_intt_limb(self._h, int(t), _p64(a[r]))
        return a

    def small_to_eval(self, coef, idx):
        coef = _i64(coef)
        ix = np.ascontiguousarray(idx, dtype=np.int32)
        out = np.empty((len(ix), self.N), dtype=np.uint64)
        self._L.orc_small_to_eval(self._h, _pi64(coef), _pint(ix), len(ix), _p64(out))
        return out

    # ---- host crypto ----
    def keygen_public(self, s, a_eval, e):
        pk = np.empty((2, self.n_q, self.N), dtype=np.uint64)
        self._L.orc_keygen_public(self._h, _pi64(_i64(s)), _p64(_u64(a_eval)), _pi64(_i64(e)), _p64(pk))
        return pk

    def keygen_switch(self, s, sprime_eval, a, e):
        T = self.n_q + self.k
        key = np.empty((self.beta_top, 2, T, self.N), dtype=np.uint64)
        a = _u64(a)
        assert a.shape == (self.beta_top, T, self.N)
        e = _i64(e)
        assert e.shape == (self.beta_top, self.N)
        sp = _u64(sprime_eval)
        assert sp.shape == (T, self.N)
        self._L.orc_keygen_switch(self._h, _pi64(_i64(s)), _p64(sp), _p64(a), _pi64(e), _p64(key))
        return key

    def s_squared_eval(self, s):
        """s^2 over the full basis, evaluation form (pointwise square of s)."""
        T = self.n_q + self.k
        sh = self.small_to_eval(s, list(range(T)))
        out = np.empty_like(sh)
        for t in range(T):
            q = self.moduli[t]
            out[t] = np.array([(int(v) * int(v)) % q for v in sh[t]], dtype=np.uint64)
        return out

    def s_galois_eval(self, s, g):
        """sigma_g(s) over the full basis, evaluation form, via the coefficient definition."""
        T = self.n_q + self.k
        sg = np.empty(self.N, dtype=np.int64)
        self._L.orc_automorphism_small(_pi64(_i64(s)), self.logN, g, _pi64(sg))
        return self.small_to_eval(sg, list(range(T)))

    def keygen_relin(self, s, a, e):
        return self.keygen_switch(s, self.s_squared_eval(s), a, e)

    def keygen_galois(self, s, g, a, e):
        return self.keygen_switch(s, self.s_galois_eval(s, g), a, e)

    def encrypt(self, pk, m_eval, r, e0, e1, level):
        ct = np.empty((2, level, self.N), dtype=np.uint64)
        m_eval = _u64(m_eval)
        assert m_eval.shape == (level, self.N)
        self._L.orc_encrypt(self._h, _p64(_u64(pk)), _p64(m_eval), _pi64(_i64(r)), _pi64(_i64(e0)), _pi64(_i64(e1)), level, _p64(ct))
        return ct

    def decrypt(self, s, ct, level):
        """c0 + c1*s (+ c2*s^2) per limb, coefficient form [level][N]."""
        ct = _u64(ct)
        n_comp = ct.shape[0]
        assert ct.shape == (n_comp, level, self.N)
        m = np.empty((level, self.N), dtype=np.uint64)
        self._L.orc_decrypt(self._h, _pi64(_i64(s)), _p64(ct), level, n_comp, _p64(m))
        return m

    # ---- ciphertext arithmetic ----
    def tensor(self, a, b, level):
        d = np.empty((3, level, self.N), dtype=np.uint64)
        self._L.orc_tensor(self._h, _p64(_u64(a)), _p64(_u64(b)), level, _p64(d))
        return d

    def modup(self, d_coef, level, j):
        out = np.empty((level + self.k, self.N), dtype=np.uint64)
        self._L.orc_modup(self._h, _p64(_u64(d_coef)), level, j, _p64(out))
        return out

    def divround_coef(self, x, cidx, bidx, exact=False):
        ci = np.ascontiguousarray(cidx, dtype=np.int32)
        bi = np.ascontiguousarray(bidx, dtype=np.int32)
        x = _u64(x)
        assert x.shape == (len(ci) + len(bi), self.N)
        out = np.empty((len(ci), self.N), dtype=np.uint64)
        fn = self._L.orc_divround_exact_coef if exact else self._L.orc_divround_coef
        fn(self._h, _p64(x), _pint(ci), len(ci), _pint(bi), len(bi), _p64(out))
        return out

    def keyswitch(self, d_eval, key, level):
        ks = np.empty((2, level, self.N), dtype=np.uint64)
        self._L.orc_keyswitch(self._h, _p64(_u64(d_eval)), _p64(_u64(key)), level, _p64(ks))
        return ks

    def relin(self, d, rlk, level):
        out = np.empty((2, level, self.N), dtype=np.uint64)
        self._L.orc_relin(self._h, _p64(_u64(d)), _p64(_u64(rlk)), level, _p64(out))
        return out

    def rescale(self, ct, level):
        out = np.empty((2, level - 1, self.N), dtype=np.uint64)
        self._L.orc_rescale(self._h, _p64(_u64(ct)), level, _p64(out))
        return out

    def hmul_relin_rescale(self, a, b, rlk, level):
        out = np.empty((2, level - 1, self.N), dtype=np.uint64)
        self._L.orc_hmul_relin_rescale(self._h, _p64(_u64(a)), _p64(_u64(b)), _p64(_u64(rlk)), level, _p64(out))
        return out

    def hmul_sum_relin_rescale(self, a, b, rlk, level):
        """sum over the leading axis of a, b ([terms][2][level][N]) of the products, relinearised and rescaled once"""
        a, b = np.ascontiguousarray(_u64(a)), np.ascontiguousarray(_u64(b))
        assert a.shape == b.shape and a.shape[1:] == (2, level, self.N)
        out = np.empty((2, level - 1, self.N), dtype=np.uint64)
        self._L.orc_hmul_sum_relin_rescale(self._h, _p64(a), _p64(b), a.shape[0], _p64(_u64(rlk)), level, _p64(out))
        return out

    def hmul_relin_rescale_merged(self, a, b, rlk, level):
        """The product with one division by P*q_{level-1} (different output bits, same message)."""
        out = np.empty((2, level - 1, self.N), dtype=np.uint64)
        self._L.orc_hmul_relin_rescale_merged(self._h, _p64(_u64(a)), _p64(_u64(b)), _p64(_u64(rlk)), level, _p64(out))
        return out

    def automorphism_coef(self, a, g, t):
        a = _u64(a)
        out = np.empty_like(a)
        self._L.orc_automorphism_coef(_p64(a), self.logN, g, self.moduli[t], _p64(out))
        return out

    def automorphism_eval(self, a, g):
        a = _u64(a)
        out = np.empty_like(a)
        self._L.orc_automorphism_eval(_p64(a), self.logN, g, _p64(out))
        return out

    def rotate(self, ct, r, gk, level):
        """Left rotation of the slot vector by r (Galois element 5^r mod 2N)."""
        g = galois_element(self.logN, r)
        out = np.empty((2, level, self.N), dtype=np.uint64)
        self._L.orc_rotate(self._h, _p64(_u64(ct)), g, _p64(_u64(gk)), level, _p64(out))
        return out

    def rotate_hoisted(self, ct, rots, gks, level):
        """Left rotations of one ciphertext by every r in rots with one shared ModUp; gks: their keys, in order."""
        g = np.array([galois_element(self.logN, r) for r in rots], dtype=np.uint64)
        keys = np.ascontiguousarray(np.stack([_u64(k) for k in gks]))
        out = np.empty((len(rots), 2, level, self.N), dtype=np.uint64)
        self._L.orc_rotate_hoisted(self._h, _p64(_u64(ct)), level, len(rots), _p64(g), _p64(keys), _p64(out))
        return out

    def linear_transform(self, x, diag_pts, gks, level):
        """One ciphertext whose slots hold a vector z (the single-image, rotation-packed layout), times a matrix given by
        its generalised diagonals: out = Rescale( sum_d pt_d * Rot_d(x) ), pt_d the encoded d-th diagonal ([level][N],
        evaluation form) and Rot_d the rotation by d slots taken from ONE shared ModUp (rotate_hoisted); d = 0 needs no
        rotation.  Decrypts to sum_d diag_d * roll(z, -d) = M z at scale s * s_pt / q_{level-1}.  level -> level-1."""
        acc = None
        rots = sorted(d for d in diag_pts if d != 0)
        rotated = self.rotate_hoisted(x, rots, [gks[d] for d in rots], level) if rots else []
        for d in sorted(diag_pts):
            src = _u64(x) if d == 0 else rotated[rots.index(d)]
            term = self.mul_plain(src, diag_pts[d], level)
            acc = term if acc is None else self.add(acc, term, level)
        return self.rescale(acc, level)

    def linear_transform_blocks(self, xs, diag_pts, gks, level):
        """A matrix-vector product whose vectors span several ciphertexts (single-image packing of a layer wider than the
        slot count): xs[j] holds block j of the input vector, diag_pts[(i, j)] = {d: encoded diagonal d of block (i, j)},
        and output block i is  Rescale( sum_j sum_d pt_(i,j),d * Rot_d(xs[j]) ).  Every input block is rotated once for
        all the output blocks that need it, by all its offsets from ONE shared ModUp (rotate_hoisted); d = 0 needs no
        rotation.  Returns the list of output ciphertexts (level-1), blocks 0 .. max i; an output block that no input
        reaches would be an encryption of zero and is not allowed here."""
        n_out = 1 + max(i for i, _ in diag_pts)
        acc = [None] * n_out
        for j, x in enumerate(xs):
            rots = sorted({d for (i, jj), dg in diag_pts.items() if jj == j for d in dg if d != 0})
            rotated = self.rotate_hoisted(x, rots, [gks[d] for d in rots], level) if rots else []
            for (i, jj), dg in sorted(diag_pts.items()):
                if jj != j:
                    continue
                for d in sorted(dg):
                    src = _u64(x) if d == 0 else rotated[rots.index(d)]
                    term = self.mul_plain(src, dg[d], level)
                    acc[i] = term if acc[i] is None else self.add(acc[i], term, level)
        assert all(a is not None for a in acc), "an output block receives nothing"
        return [self.rescale(a, level) for a in acc]

    def linear_transform_bsgs(self, xs, bsgs_pts, gks, level, baby):
        """The block matrix-vector product of linear_transform_blocks with the rotations split into baby and giant steps
        (the standard way to apply an n-diagonal matrix with about 2 sqrt(n) rotation keys instead of n): offset
        d = g * baby + b, and
            sum_d diag_d * Rot_d(x) = sum_g Rot_(g*baby)( sum_b roll(diag_(g*baby+b), +g*baby) * Rot_b(x) ).
        bsgs_pts[(i, j)] = {(g, b): the encoded, pre-rotated diagonal roll(diag_(g*baby+b), g*baby)} (see bsgs_diagonals).
        Steps: every input block x_j is rotated by its baby offsets b != 0 from ONE shared ModUp (rotate_hoisted); for
        every output block i and giant index g the inner sum over j and b (plaintext products and additions); each inner
        sum with g != 0 is rotated by g*baby with an ordinary rotation (its own ModUp); the sum over g is rescaled.
        Returns the list of output ciphertexts at level-1.  Other bits than linear_transform_blocks (other rotations, other
        key-switching noise), the same decrypted product."""
        n_out = 1 + max(i for i, _ in bsgs_pts)
        rotated = []
        for j, x in enumerate(xs):
            babies = sorted({b for (i, jj), dg in bsgs_pts.items() if jj == j for (_, b) in dg if b != 0})
            rot = self.rotate_hoisted(x, babies, [gks[b] for b in babies], level) if babies else []
            rotated.append({0: _u64(x), **{b: rot[k] for k, b in enumerate(babies)}})
        outs = []
        for i in range(n_out):
            giants = sorted({g for (ii, _), dg in bsgs_pts.items() if ii == i for (g, _) in dg})
            assert giants, "an output block receives nothing"
            total = None
            for g in giants:
                inner = None
                for (ii, j), dg in sorted(bsgs_pts.items()):
                    if ii != i:
                        continue
                    for (gg, b) in sorted(dg):
                        if gg != g:
                            continue
                        term = self.mul_plain(rotated[j][b], dg[(gg, b)], level)
                        inner = term if inner is None else self.add(inner, term, level)
                if g != 0:
                    inner = self.rotate(inner, g * baby, gks[g * baby], level)
                total = inner if total is None else self.add(total, inner, level)
            outs.append(self.rescale(total, level))
        return outs

    def packed_network(self, xs, stages, rlk, gks, level):
        """One image through a network in the single-image packing: xs = the ciphertexts holding the input vector's
        blocks; stages = [("linear", diag_pts) | ("linear_bsgs", bsgs_pts, baby) | ("poly2", k2, k1)], a linear stage being any product of the network's
        linear layers between two activations (convolution, pooling and fully connected layers are all matrices, and a
        pooling layer is merged with the layer after it), poly2 the degree-2 activation of section 3.1 applied to every
        block.  Returns (list of output ciphertexts, their level)."""
        for st in stages:
            if st[0] == "linear":
                xs = self.linear_transform_blocks(xs, st[1], gks, level)
                level -= 1
            elif st[0] == "linear_bsgs":
                xs = self.linear_transform_bsgs(xs, st[1], gks, level, st[2])
                level -= 1
            elif st[0] == "poly2":
                xs = [self.poly2(x, rlk, level, st[1], st[2]) for x in xs]
                level -= 2
            else:
                raise ValueError(st[0])
        return xs, level

    def add(self, a, b, level):
        out = np.empty((2, level, self.N), dtype=np.uint64)
        self._L.orc_add(self._h, _p64(_u64(a)), _p64(_u64(b)), level, _p64(out))
        return out

    def sub(self, a, b, level):
        out = np.empty((2, level, self.N), dtype=np.uint64)
        self._L.orc_sub(self._h, _p64(_u64(a)), _p64(_u64(b)), level, _p64(out))
        return out

    def mul_plain(self, a, pt, level):
        out = np.empty((2, level, self.N), dtype=np.uint64)
        self._L.orc_mul_plain(self._h, _p64(_u64(a)), _p64(_u64(pt)), level, _p64(out))
        return out

    def mul_scalar(self, a, c, level):
        out = np.empty((2, level, self.N), dtype=np.uint64)
        self._L.orc_mul_scalar(self._h, _p64(_u64(a)), int(c), level, _p64(out))
        return out

    def add_const(self, a, c, level):
        out = np.empty((2, level, self.N), dtype=np.uint64)
        self._L.orc_add_const(self._h, _p64(_u64(a)), int(c), level, _p64(out))
        return out

    def mod_drop(self, a, level_in, level_out):
        a = _u64(a).reshape(2, level_in, self.N)
        return np.ascontiguousarray(a[:, :level_out, :])

    def conv2d_mac(self, x, w, stride, pad, level):
        x = _u64(x)
        w = _i64(w)
        Cc, H, W = x.shape[:3]
        O, C2, kh, kw = w.shape
        assert C2 == Cc and x.shape[3:] == (2, level, self.N)
        Ho = (H + 2 * pad - kh) // stride + 1
        Wo = (W + 2 * pad - kw) // stride + 1
        out = np.empty((O, Ho, Wo, 2, level, self.N), dtype=np.uint64)
        self._L.orc_conv2d_mac(self._h, _p64(x), _pi64(w), Cc, H, W, O, kh, kw, stride, pad, level, _p64(out))
        return out

    def fc_mac(self, x, w, level):
        x = _u64(x)
        w = _i64(w)
        F = x.shape[0]
        O = w.shape[0]
        assert w.shape == (O, F) and x.shape[1:] == (2, level, self.N)
        out = np.empty((O, 2, level, self.N), dtype=np.uint64)
        self._L.orc_fc_mac(self._h, _p64(x), _pi64(w), F, O, level, _p64(out))
        return out

    def sum_pool2d(self, x, k, level, pad=0):
        """k x k pooling as a sum of ciphertexts (Table 1's zero padding + average pooling without the 1/k^2)."""
        x = _u64(x)
        Cc, H, W = x.shape[:3]
        assert x.shape[3:] == (2, level, self.N)
        out = np.empty((Cc, (H + 2 * pad) // k, (W + 2 * pad) // k, 2, level, self.N), dtype=np.uint64)
        self._L.orc_sum_pool2d(self._h, _p64(x), Cc, H, W, k, pad, level, _p64(out))
        return out

    def _map(self, fn, n, workers):
        """fn(b) for b < n; independent ciphertexts may be spread over threads (the C calls release the GIL)"""
        if workers <= 1:
            for b in range(n):
                fn(b)
        else:
            from concurrent.futures import ThreadPoolExecutor
            with ThreadPoolExecutor(workers) as ex:
                list(ex.map(fn, range(n)))

    def rescale_each(self, cts, level, workers=1):
        """Rescale every ciphertext of an array [...][2][level][N]."""
        cts = _u64(cts)
        lead = cts.shape[:-3]
        flat = cts.reshape((-1, 2, level, self.N))
        out = np.empty((flat.shape[0], 2, level - 1, self.N), dtype=np.uint64)

        def one(b):
            out[b] = self.rescale(flat[b], level)
        self._map(one, flat.shape[0], workers)
        return out.reshape(lead + (2, level - 1, self.N))

    def square_each(self, cts, rlk, level, workers=1):
        cts = _u64(cts)
        lead = cts.shape[:-3]
        flat = cts.reshape((-1, 2, level, self.N))
        out = np.empty((flat.shape[0], 2, level - 1, self.N), dtype=np.uint64)

        def one(b):
            out[b] = self.hmul_relin_rescale(flat[b], flat[b], rlk, level)
        self._map(one, flat.shape[0], workers)
        return out.reshape(lead + (2, level - 1, self.N))

    def poly2_each(self, cts, rlk, level, k2, k1, workers=1):
        cts = _u64(cts)
        lead = cts.shape[:-3]
        flat = cts.reshape((-1, 2, level, self.N))
        out = np.empty((flat.shape[0], 2, level - 2, self.N), dtype=np.uint64)

        def one(b):
            out[b] = self.poly2(flat[b], rlk, level, k2, k1)
        self._map(one, flat.shape[0], workers)
        return out.reshape(lead + (2, level - 2, self.N))

    def conv2d_mac_each(self, x, w, stride, pad, level, workers=1):
        """conv2d_mac, one output channel per call"""
        w = _i64(w)
        parts = [None] * w.shape[0]

        def one(o):
            parts[o] = self.conv2d_mac(x, w[o:o + 1], stride, pad, level)
        self._map(one, w.shape[0], workers)
        return np.concatenate(parts, axis=0)

    def cnn_forward(self, x, layers, rlk, level, workers=1):
        """A feed-forward network over per-pixel ciphertexts (section 3: convolution, pooling, polynomial activation
        and fully connected layers in sequence), slot s = image s.

        x: [C][H][W][2][level][N].  layers: a list of
          ("conv", w_int [O][C][kh][kw], stride, pad)  convolution MAC, then rescale of every output   level -> level-1
          ("square",)                                  activation x^2 with relinearisation and rescale  level -> level-1
          ("pool", k[, pad])                           k x k sum pooling of the zero-padded image       level unchanged
          ("poly2", k2, k1)                            activation c2*x^2 + c1*x (integer constants)     level -> level-2
          ("fc", w_int [O][F])                         flatten [C][H][W] in that order, MAC, rescale    level -> level-1
        Integer weights are prepared by the caller (round(w * dropped modulus)).  Returns (cts, level).
        workers > 1 only spreads independent ciphertexts over threads.
        """
        x = _u64(x)
        for layer in layers:
            kind = layer[0]
            if kind == "conv":
                _, w, stride, pad = layer
                x = self.rescale_each(self.conv2d_mac_each(x, w, stride, pad, level, workers), level, workers)
                level -= 1
            elif kind == "square":
                x = self.square_each(x, rlk, level, workers)
                level -= 1
            elif kind == "pool":
                x = self.sum_pool2d(x, layer[1], level, layer[2] if len(layer) > 2 else 0)
            elif kind == "poly2":
                x = self.poly2_each(x, rlk, level, layer[1], layer[2], workers)
                level -= 2
            elif kind == "fc":
                flat = x.reshape((-1, 2, level, self.N))
                x = self.rescale_each(self.fc_mac(flat, layer[1], level), level, workers)
                level -= 1
                x = x.reshape((x.shape[0], 1, 1, 2, level, self.N))
            else:
                raise ValueError(kind)
        return x, level

    # ---- activation schedules (compositions; constants are passed in) ----
    def square(self, x, rlk, level):
        """x^2 with relinearisation and rescale: level -> level-1."""
        return self.hmul_relin_rescale(x, x, rlk, level)

    def poly2(self, x, rlk, level, k2, k1):
        """c2*x^2 + c1*x (the degree-2 polynomial that replaces ReLU in section 3.1) on a ciphertext x at `level`
        with scale s, ending at level-2 with scale s2 = s^2/q_{level-1}.  The caller prepares the integer constants so
        that both addends carry that scale:
          x2  = RS(Relin(x*x))                    level-1, scale s2
          t2  = RS(x2 * k2)                       level-2   (k2 ~ c2 * q_{level-2})
          t1  = RS(drop(x -> level-1) * k1)       level-2   (k1 ~ c1 * (s2/s) * q_{level-2})
          out = t2 + t1
        """
        x2 = self.hmul_relin_rescale(x, x, rlk, level)
        t2 = self.rescale(self.mul_scalar(x2, k2, level - 1), level - 1)
        t1 = self.rescale(self.mul_scalar(self.mod_drop(x, level, level - 1), k1, level - 1), level - 1)
        return self.add(t2, t1, level - 2)

    def poly3(self, y, rlk, level, c_m002, c_025, c_05):
        """0.5 + 0.25*y - 0.02*y^3 on a ciphertext y at `level`, ending at level-2.

        The three integer constants are prepared by the caller from the tracked
        scales so that every addend has the same scale:
          y2 = RS(Relin(y*y))                       level-1
          t  = RS(y * c_m002)                       level-1   (c_m002 ~ -0.02*q_{level-1})
          y3 = RS(Relin(y2*t))                      level-2
          u  = RS(drop(y -> level-1) * c_025)       level-2   (c_025 ~ 0.25*scale(y2))
          out = y3 + u + c_05                       level-2   (c_05 ~ 0.5*scale(y3))
        """
        y2 = self.hmul_relin_rescale(y, y, rlk, level)
        t = self.rescale(self.mul_scalar(y, c_m002, level), level)
        y3 = self.hmul_relin_rescale(y2, t, rlk, level - 1)
        u = self.rescale(self.mul_scalar(self.mod_drop(y, level, level - 1), c_025, level - 1), level - 1)
        return self.add_const(self.add(y3, u, level - 2), c_05, level - 2)


# --------------------------------------------------------------------------
# big-integer CRT and the encoding map
# --------------------------------------------------------------------------
def crt_reconstruct(residues, moduli, centered=True):
    """[l][n] residues -> list of n Python ints, in (-Q/2, Q/2] if centered else [0, Q)."""
    residues = np.asarray(residues)
    Q = 1
    for q in moduli:
        Q *= int(q)
    coef = []
    for q in moduli:
        Qi = Q // int(q)
        coef.append(Qi * pow(Qi % int(q), -1, int(q)))
    out = []
    rows = [[int(v) for v in residues[i]] for i in range(len(moduli))]
    for n in range(residues.shape[1]):
        x = 0
        for i in range(len(moduli)):
            x += rows[i][n] * coef[i]
        x %= Q
        if centered and x > Q // 2:
            x -= Q
        out.append(x)
    return out


def to_rns(coeffs, moduli):
    """list of Python ints (any size, signed) -> [l][n] canonical residues."""
    n = len(coeffs)
    out = np.empty((len(moduli), n), dtype=np.uint64)
    small = all(-(1 << 62) < int(c) < (1 << 62) for c in coeffs)
    if small:
        arr = np.array([int(c) for c in coeffs], dtype=np.int64)
        for i, q in enumerate(moduli):
            out[i] = np.mod(arr, np.int64(q)).astype(np.uint64)
    else:
        for i, q in enumerate(moduli):
            out[i] = np.array([int(c) % int(q) for c in coeffs], dtype=np.uint64)
    return out


def slot_exponents(logN):
    """5^k mod 2N for k < N/2: slot k lives at the root zeta^(5^k)."""
    N = 1 << logN
    e, out = 1, []
    for _ in range(N // 2):
        out.append(e)
        e = (e * 5) % (2 * N)
    return out


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    o = (C.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def sample(kind, sigma, seed, first_index, rows, logN):
    """rows x N small coefficients from the counter-based sampler: kind 0 ternary, kind 1 rounded Gaussian"""
    out = np.empty((rows, 1 << logN), dtype=np.int64)
    f = lib().orc_sample
    f.argtypes = [C.c_int, C.c_double, C.c_uint64, C.c_uint64, C.c_int, C.c_int, C.POINTER(C.c_int64)]
    f.restype = None
    f(kind, float(sigma), seed, first_index, rows, logN, out.ctypes.data_as(C.POINTER(C.c_int64)))
    return out


def gauss_thresholds(sigma):
    T = np.empty(40, dtype=np.uint64)
    f = lib().orc_gauss_thresholds
    f.argtypes = [C.c_double, C.POINTER(C.c_uint64)]
    f.restype = None
    f(float(sigma), T.ctypes.data_as(C.POINTER(C.c_uint64)))
    return T


def matrix_diagonals(M, n_slots):
    """Generalised diagonals of a square matrix M (n x n, n dividing n_slots) for a slot vector that repeats z with
    period n: diag_d[i] = M[i mod n][(i + d) mod n], so that M z = sum_d diag_d * roll(z, -d).  Zero diagonals are
    left out.  Returns {d: vector of n_slots values}."""
    M = np.asarray(M, dtype=np.float64)
    n = M.shape[0]
    assert M.shape == (n, n) and n_slots % n == 0
    out = {}
    for d in range(n):
        diag = np.array([M[i][(i + d) % n] for i in range(n)])
        if np.any(diag != 0.0):
            out[d] = np.tile(diag, n_slots // n)
    return out


def conv_as_matrix(w, H, W, pad, stride=1):
    """The convolution of a C x H x W image (flattened channel-major) with weights w [O][C][kh][kw], zero padding `pad`
    and stride `stride`, output O x H' x W' with H' = (H + 2 pad - kh) / stride + 1, written as a dense matrix
    [O*H'*W'][C*H*W] straight from the definition (Table 1's convolution rows)."""
    w = np.asarray(w, dtype=np.float64)
    O, C, kh, kw = w.shape
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    M = np.zeros((O * Ho * Wo, C * H * W))
    for o in range(O):
        for y in range(Ho):
            for x in range(Wo):
                for c in range(C):
                    for u in range(kh):
                        for v in range(kw):
                            iy, ix = y * stride + u - pad, x * stride + v - pad
                            if 0 <= iy < H and 0 <= ix < W:
                                M[(o * Ho + y) * Wo + x][(c * H + iy) * W + ix] += w[o][c][u][v]
    return M


def pool_as_matrix(C, H, W, k, pad=0):
    """k x k average pooling (Table 1's pooling rows) of a C x H x W image padded with `pad` zero rows / columns on every
    side, windows at multiples of k, output C x floor((H + 2 pad)/k) x floor((W + 2 pad)/k), as a matrix [C*H'*W'][C*H*W]
    with entries 1/k^2 (positions on the padding contribute nothing)."""
    Ho, Wo = (H + 2 * pad) // k, (W + 2 * pad) // k
    M = np.zeros((C * Ho * Wo, C * H * W))
    for c in range(C):
        for y in range(Ho):
            for x in range(Wo):
                for u in range(k):
                    for v in range(k):
                        iy, ix = k * y + u - pad, k * x + v - pad
                        if 0 <= iy < H and 0 <= ix < W:
                            M[(c * Ho + y) * Wo + x][(c * H + iy) * W + ix] = 1.0 / (k * k)
    return M


def block_diagonals(M, n, n_slots):
    """A matrix of any shape cut into n x n blocks (zero-padded to multiples of n; n divides n_slots, and n = n_slots as
    soon as there is more than one block in a direction): {(i, j): {d: diagonal d of block (i, j) tiled over n_slots}},
    empty diagonals and empty blocks left out.  Output block i of M z is sum_j sum_d diag_(i,j),d * roll(z_j, -d)."""
    M = np.asarray(M, dtype=np.float64)
    bo, bi = -(-M.shape[0] // n), -(-M.shape[1] // n)
    assert n_slots % n == 0 and (n == n_slots or (bo == 1 and bi == 1))
    P = np.zeros((bo * n, bi * n))
    P[: M.shape[0], : M.shape[1]] = M
    out = {}
    for i in range(bo):
        for j in range(bi):
            dg = matrix_diagonals(P[i * n:(i + 1) * n, j * n:(j + 1) * n], n_slots)
            if dg:
                out[(i, j)] = dg
    return out


def bsgs_diagonals(diags, baby):
    """Baby-step / giant-step form of block diagonals {(i, j): {d: vector}} (block_diagonals): {(i, j): {(g, b): roll(vector,
    +g*baby)}} with d = g*baby + b, 0 <= b < baby.  Rotating a product left by g*baby slots rotates the diagonal back."""
    out = {}
    for key, dg in diags.items():
        out[key] = {(d // baby, d % baby): np.roll(v, (d // baby) * baby) for d, v in dg.items()}
    return out


def encode_direct(z, scale, logN):
    """Definition, O(N^2): m_t = round( (2/N) * Re( sum_k scale*z_k * zeta^(-5^k t) ) )."""
    N = 1 << logN
    z = np.asarray(z, dtype=np.complex128)
    assert z.shape == (N // 2,)
    ex = np.array(slot_exponents(logN), dtype=np.int64)
    out = []
    for t in range(N):
        ang = -np.pi * ((ex * t) % (2 * N)) / N
        v = np.sum(z * (np.cos(ang) + 1j * np.sin(ang)))
        out.append(int(np.rint(2.0 * scale * v.real / N)))
    return out


def decode_direct(coeffs, scale, logN):
    """Definition, O(N^2): z_k = m(zeta^(5^k)) / scale."""
    N = 1 << logN
    m = np.array([float(c) for c in coeffs], dtype=np.float64)
    t = np.arange(N, dtype=np.int64)
    out = np.empty(N // 2, dtype=np.complex128)
    for k, e in enumerate(slot_exponents(logN)):
        ang = np.pi * ((e * t) % (2 * N)) / N
        out[k] = np.sum(m * (np.cos(ang) + 1j * np.sin(ang))) / scale
    return out


def encode(z, scale, logN):
    """Same map through a length-N FFT: with b_t = m_t*zeta^t, the values at the
    odd powers are v[u] = m(zeta^(2u+1)) = sum_t b_t e^(2 pi i u t / N)."""
    N = 1 << logN
    z = np.asarray(z, dtype=np.complex128)
    assert z.shape == (N // 2,)
    v = np.zeros(N, dtype=np.complex128)
    ex = np.array(slot_exponents(logN), dtype=np.int64)
    v[(ex - 1) // 2] = z
    v[(2 * N - ex - 1) // 2] = np.conj(z)
    b = np.fft.fft(v) / N
    t = np.arange(N)
    m = (b * np.exp(-1j * np.pi * t / N)).real * scale
    return [int(x) for x in np.rint(m)]


def decode(coeffs, scale, logN):
    N = 1 << logN
    m = np.array([float(c) for c in coeffs], dtype=np.float64)
    t = np.arange(N)
    b = m * np.exp(1j * np.pi * t / N)
    v = np.fft.ifft(b) * N
    ex = np.array(slot_exponents(logN), dtype=np.int64)
    return v[(ex - 1) // 2] / scale

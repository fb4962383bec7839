"""Pins for the CPU oracle: every check here compares the oracle with something
other than itself -- Python big-integer arithmetic, closed forms, brute force on
tiny inputs, invariants of the scheme -- so that a dropped term, a wrong sign or
index, or a transposed operand in the oracle fails at least one of them.
CPU only."""
import math
import random

import numpy as np
import pytest

from oracle import oracle as orc
from paper_1911_11377_amd import workloads as wl
from helpers import Material, poly_mul_negacyclic_int

# (bits, logN of the workload shape the prime belongs to)
SHAPE_PRIMES = [(40, 12), (41, 12), (50, 14), (51, 14), (50, 15), (50, 16), (51, 16)]


# ---------------------------------------------------------------- arithmetic
def test_modular_arithmetic_matches_python_ints():
    rnd = random.Random(1)
    L = orc.lib()
    for _ in range(2000):
        q = rnd.randrange(3, 1 << rnd.choice([20, 40, 51, 62, 64]))
        a, b = rnd.randrange(q), rnd.randrange(q)
        assert L.orc_mulmod(a, b, q) == a * b % q
        assert L.orc_addmod(a, b, q) == (a + b) % q
        assert L.orc_submod(a, b, q) == (a - b) % q
        e = rnd.randrange(1 << 64)
        assert L.orc_powmod(a, e, q) == pow(a, e, q)
        v = rnd.randrange(-(1 << 63), 1 << 63)
        assert L.orc_signed_mod(v, q) == v % q
    assert L.orc_signed_mod(-(1 << 63), 1000003) == (-(1 << 63)) % 1000003


def _lucas_certificate(q, logN):
    """q is prime iff some g has g^(q-1) = 1 and g^((q-1)/r) != 1 for every prime r | q-1."""
    m = (q - 1) >> (logN + 1)
    fac = {2}
    r = 2
    while r * r <= m:
        while m % r == 0:
            fac.add(r)
            m //= r
        r += 1 if r == 2 else 2
    if m > 1:
        fac.add(m)
    for g in range(2, 200):
        if pow(g, q - 1, q) == 1 and all(pow(g, (q - 1) // r, q) != 1 for r in fac):
            return True
    return False


@pytest.mark.parametrize("bits,logN", SHAPE_PRIMES)
def test_prime_rule(bits, logN):
    count = 4
    ps = orc.find_primes(bits, logN, count)
    twoN = 2 << logN
    assert ps == sorted(ps, reverse=True) and len(set(ps)) == count
    for q in ps:
        assert (1 << (bits - 1)) < q < (1 << bits) and q % twoN == 1
        assert _lucas_certificate(q, logN)
    # nothing skipped: every candidate above the last prime that is not listed is composite
    c = (1 << bits) - twoN + 1
    while c > ps[-1]:
        if c not in ps:
            assert pow(2, c - 1, c) != 1 or not _lucas_certificate(c, logN)
        c -= twoN
    # exclusion list
    assert orc.find_primes(bits, logN, 2, exclude=[ps[0]]) == ps[1:3]


@pytest.mark.parametrize("bits,logN", SHAPE_PRIMES)
def test_psi_rule(bits, logN):
    q = orc.find_primes(bits, logN, 1)[0]
    N = 1 << logN
    psi = orc.find_psi(q, logN)
    assert pow(psi, N, q) == q - 1 and pow(psi, 2 * N, q) == 1
    x = 2
    while True:
        cand = pow(x, (q - 1) // (2 * N), q)
        if pow(cand, N, q) == q - 1:
            break
        x += 1
    assert cand == psi


# ---------------------------------------------------------------- transform
def test_direct_transform_is_polynomial_evaluation():
    """definition vs Horner evaluation with Python ints, N = 8"""
    logN, N = 3, 8
    q = orc.find_primes(40, 12, 1)[0]
    psi = pow(orc.find_psi(q, 12), (1 << 12) // N, q)
    rnd = random.Random(2)
    a = [rnd.randrange(q) for _ in range(N)]
    got = orc.ntt_direct(a, logN, q, psi)
    for j in range(N):
        br = int(format(j, "03b")[::-1], 2)
        x = pow(psi, 2 * br + 1, q)
        assert int(got[j]) == sum(a[t] * pow(x, t, q) for t in range(N)) % q
    assert [int(v) for v in orc.intt_direct(got, logN, q, psi)] == a


@pytest.mark.parametrize("bits,shape_logN", SHAPE_PRIMES)
@pytest.mark.parametrize("logN", [2, 5, 8])
def test_fast_transform_matches_definition(bits, shape_logN, logN):
    q = orc.find_primes(bits, shape_logN, 2)[1]
    psi = pow(orc.find_psi(q, shape_logN), (1 << shape_logN) >> logN, q)
    N = 1 << logN
    a = wl.uniform_limbs([q], N, 3, bits, logN)[0]
    f = orc.ntt(a, logN, q, psi)
    assert np.array_equal(f, orc.ntt_direct(a, logN, q, psi))
    assert np.array_equal(orc.intt(f, logN, q, psi), a)
    assert np.array_equal(orc.intt_direct(f, logN, q, psi), a)


def test_fast_transform_matches_definition_n1024():
    logN = 10
    q = orc.find_primes(50, 16, 1)[0]
    psi = pow(orc.find_psi(q, 16), 1 << 6, q)
    a = wl.uniform_limbs([q], 1 << logN, 4)[0]
    assert np.array_equal(orc.ntt(a, logN, q, psi), orc.ntt_direct(a, logN, q, psi))


def test_transform_closed_forms():
    logN, N = 12, 1 << 12
    q = orc.find_primes(40, logN, 1)[0]
    psi = orc.find_psi(q, logN)
    X = np.zeros(N, dtype=np.uint64)
    X[1] = 1
    want = [pow(psi, 2 * orc.brev(j, logN) + 1, q) for j in range(N)]
    assert [int(v) for v in orc.ntt(X, logN, q, psi)] == want
    c = np.zeros(N, dtype=np.uint64)
    c[0] = 12345
    assert (orc.ntt(c, logN, q, psi) == 12345).all()
    # linearity
    a = wl.uniform_limbs([q], N, 5, "a")[0]
    b = wl.uniform_limbs([q], N, 5, "b")[0]
    s = (a.astype(object) + b.astype(object)) % q
    fa, fb = orc.ntt(a, logN, q, psi), orc.ntt(b, logN, q, psi)
    assert np.array_equal(orc.ntt(s.astype(np.uint64), logN, q, psi), ((fa.astype(object) + fb.astype(object)) % q).astype(np.uint64))


def test_schoolbook_is_the_ring_product():
    """schoolbook negacyclic vs exact integer polynomial product, N = 16"""
    logN, N = 4, 16
    q = orc.find_primes(50, 14, 1)[0]
    rnd = random.Random(6)
    a = [rnd.randrange(q) for _ in range(N)]
    b = [rnd.randrange(q) for _ in range(N)]
    want = [v % q for v in poly_mul_negacyclic_int(a, b)]
    assert [int(v) for v in orc.negacyclic_schoolbook(a, b, logN, q)] == want
    # X^(N-1) * X = -1
    x1 = [0] * N
    x1[1] = 1
    xl = [0] * N
    xl[N - 1] = 1
    r = orc.negacyclic_schoolbook(x1, xl, logN, q)
    assert int(r[0]) == q - 1 and not r[1:].any()


@pytest.mark.parametrize("bits,special", [(40, False), (41, True)])
def test_convolution_theorem_at_tiny_shape_size(bits, special):
    """iNTT(NTT(a) * NTT(b)) equals the schoolbook negacyclic product at N = 2^12."""
    logN, N = 12, 1 << 12
    q = orc.find_primes(bits, logN, 3)[2 if not special else 0]
    psi = orc.find_psi(q, logN)
    a = wl.uniform_limbs([q], N, 7, "a", bits)[0]
    b = wl.uniform_limbs([q], N, 7, "b", bits)[0]
    fa, fb = orc.ntt(a, logN, q, psi), orc.ntt(b, logN, q, psi)
    prod = np.array([int(x) * int(y) % q for x, y in zip(fa, fb)], dtype=np.uint64)
    assert np.array_equal(orc.intt(prod, logN, q, psi), orc.negacyclic_schoolbook(a, b, logN, q))


# ---------------------------------------------------------------- RNS steps
def _small_oracle(alpha=2, k=2, n_q=5, logN=4):
    return orc.Oracle(logN, n_q, 20, k, 21, alpha)


@pytest.mark.parametrize("alpha,k,n_q,level", [(1, 1, 3, 3), (2, 2, 5, 5), (2, 2, 5, 3), (3, 3, 7, 7), (3, 3, 7, 5)])
def test_modup_is_d_plus_u_QD(alpha, k, n_q, level):
    O = _small_oracle(alpha, k, n_q)
    d = wl.uniform_limbs(O.q[:level], O.N, 8, alpha, level)
    for j in range(O.beta(level)):
        D = list(range(j * alpha, min(level, (j + 1) * alpha)))
        out = O.modup(d, level, j)
        QD = math.prod(O.q[i] for i in D)
        dint = orc.crt_reconstruct(d[D], [O.q[i] for i in D], centered=False)
        ext = O.ext_moduli(level)
        for n in range(O.N):
            # the integer the conversion represents, recomputed with big integers
            v = sum(((int(d[i][n]) * pow(QD // O.q[i], -1, O.q[i])) % O.q[i]) * (QD // O.q[i]) for i in D)
            u, rem = divmod(v - dint[n], QD)
            assert rem == 0 and 0 <= u < len(D)
            for x, t in enumerate(ext):
                if x in D:
                    assert int(out[x][n]) == int(d[x][n])
                else:
                    assert int(out[x][n]) == v % t


@pytest.mark.parametrize("nb", [1, 2, 3])
def test_divround_is_rounded_division(nb):
    O = _small_oracle(alpha=nb, k=nb, n_q=4)
    cidx = [0, 1, 2]
    for bidx in ([O.n_q + m for m in range(nb)], [3] if nb == 1 else None):
        if bidx is None:
            continue
        mods = [O.moduli[i] for i in cidx + bidx]
        B = math.prod(O.moduli[i] for i in bidx)
        h = B // 2
        x = wl.uniform_limbs(mods, O.N, 9, nb, bidx[0])
        xint = orc.crt_reconstruct(x, mods, centered=False)
        out = O.divround_coef(x, cidx, bidx)
        QC = math.prod(O.moduli[i] for i in cidx)
        seen = set()
        for n in range(O.N):
            exact = (xint[n] + h) // B
            cands = [u for u in range(nb) if all(int(out[i][n]) == (exact - u) % O.moduli[c] for i, c in enumerate(cidx))]
            assert cands, "no u in [0,|B|-1] explains the output"
            seen.add(cands[0])
            if nb == 1:
                assert cands == [0]
                # exact round-to-nearest: |x/B - out| < 1/2 (B odd, no ties)
                got = orc.crt_reconstruct(out[:, n : n + 1], [O.moduli[c] for c in cidx], centered=False)[0]
                assert got == exact % QC and abs(xint[n] - exact * B) <= B // 2


def test_switching_key_identity():
    """b_j + a_j*s - e_j = [t in digit j] * (P mod t) * s' exactly, by schoolbook products."""
    M = Material(4, 5, 20, 2, 21, 2, seed=10, rotations=(1,))
    O = M.O
    T = O.n_q + O.k
    P = math.prod(O.p)
    g = orc.galois_element(4, 1)
    s_int = [int(v) for v in M.s]
    s2 = poly_mul_negacyclic_int(s_int, s_int)
    sg = [0] * O.N
    for t in range(O.N):
        i = (t * g) % (2 * O.N)
        if i < O.N:
            sg[i] = s_int[t]
        else:
            sg[i - O.N] = -s_int[t]
    for key, sp, a_in in ((M.rlk, s2, M.rlk_a), (M.gk[1], sg, None)):
        for j in range(O.beta_top):
            for t in range(T):
                q = O.moduli[t]
                b = O.intt_limbs(key[j, 0, t : t + 1], [t])[0]
                a = O.intt_limbs(key[j, 1, t : t + 1], [t])[0]
                if a_in is not None:
                    assert np.array_equal(key[j, 1, t], a_in[j, t])
                as_ = orc.negacyclic_schoolbook(a, [v % q for v in s_int], 4, q)
                lhs = [(int(b[n]) + int(as_[n])) % q for n in range(O.N)]
                in_digit = t < O.n_q and t // O.alpha == j
                if a_in is not None:
                    e = M.rlk_e[j]
                    want = [(int(e[n]) + (P % q) * sp[n] * in_digit) % q for n in range(O.N)]
                    assert lhs == want
                else:
                    # error is small and centred; the gadget term is exact
                    diff = [(lhs[n] - (P % q) * sp[n] * in_digit) % q for n in range(O.N)]
                    assert all(min(v, q - v) <= 19 for v in diff)


def test_tensor_identity():
    """d0 + d1*s + d2*s^2 = (a0 + a1*s)(b0 + b1*s) exactly mod Q"""
    M = Material(4, 4, 20, 2, 21, 2, seed=11)
    O = M.O
    level = 4
    a = wl.uniform_limbs(O.q[:level], O.N, 11, "a", lead=(2,))
    b = wl.uniform_limbs(O.q[:level], O.N, 11, "b", lead=(2,))
    d = O.tensor(a, b, level)
    Q = math.prod(O.q[:level])
    ma, mb, md = M.decrypt_poly(a, level), M.decrypt_poly(b, level), M.decrypt_poly(d, level)
    prod = poly_mul_negacyclic_int(ma, mb)
    assert all((prod[n] - md[n]) % Q == 0 for n in range(O.N))
    # and the decryption helper itself: c0 + c1*s by schoolbook
    s_int = [int(v) for v in M.s]
    for i in range(level):
        q = O.q[i]
        c0 = O.intt_limbs(a[0, i : i + 1], [i])[0]
        c1 = O.intt_limbs(a[1, i : i + 1], [i])[0]
        want = [(int(c0[n]) + int(v)) % q for n, v in enumerate(orc.negacyclic_schoolbook(c1, [x % q for x in s_int], 4, q))]
        assert [x % q for x in ma] == want


@pytest.mark.parametrize("alpha,k,n_q,level", [(1, 1, 3, 3), (2, 2, 5, 5), (2, 2, 5, 4), (3, 3, 7, 7), (3, 3, 7, 2)])
def test_keyswitch_noise_is_small(alpha, k, n_q, level):
    M = Material(4, n_q, 20, k, 21, alpha, seed=12)
    O = M.O
    d = wl.uniform_limbs(O.q[:level], O.N, 12, "d", level)
    ks = O.keyswitch(d, M.rlk, level)
    Q = math.prod(O.q[:level])
    s_int = [int(v) for v in M.s]
    s2 = poly_mul_negacyclic_int(s_int, s_int)
    dint = orc.crt_reconstruct(O.intt_limbs(d, list(range(level))), O.q[:level])
    want = poly_mul_negacyclic_int(dint, s2)
    got = M.decrypt_poly(ks, level)
    err = [((got[n] - want[n] + Q // 2) % Q) - Q // 2 for n in range(O.N)]
    P = math.prod(O.p)
    maxQD = max(math.prod(O.q[j * alpha : min(level, (j + 1) * alpha)]) for j in range(O.beta(level)))
    bound = O.beta(level) * O.N * 19 * alpha * maxQD / P + (k + 0.5) * (1 + sum(abs(v) for v in s_int))
    assert max(abs(e) for e in err) <= bound
    assert max(abs(e) for e in err) < 2**12


def test_rescale_divides_message_by_last_prime():
    M = Material(4, 4, 20, 1, 21, 1, seed=13)
    O = M.O
    level = 4
    ct = wl.uniform_limbs(O.q[:level], O.N, 13, "ct", lead=(2,))
    out = O.rescale(ct, level)
    ql = O.q[level - 1]
    Qn = math.prod(O.q[: level - 1])
    for c in range(2):
        xin = orc.crt_reconstruct(O.intt_limbs(ct[c], list(range(level))), O.q[:level], centered=False)
        xo = orc.crt_reconstruct(O.intt_limbs(out[c], list(range(level - 1))), O.q[: level - 1], centered=False)
        for n in range(O.N):
            assert xo[n] == ((xin[n] + ql // 2) // ql) % Qn


# ---------------------------------------------------------------- encoding
def test_encode_closed_forms_and_direct_definition():
    logN, N = 5, 32
    scale = 2.0**30
    c = orc.encode(np.full(N // 2, 0.75 + 0j), scale, logN)
    assert c[0] == round(0.75 * scale) and not any(c[1:])
    zeta = np.exp(1j * np.pi / N)
    z = np.array([zeta**e for e in orc.slot_exponents(logN)])
    c = orc.encode(z, scale, logN)
    assert c[1] == round(scale) and not any(c[:1] + c[2:])
    z = wl.slots_complex(N // 2, 14)
    assert orc.encode(z, scale, logN) == orc.encode_direct(z, scale, logN)
    back = orc.decode(orc.encode(z, scale, logN), scale, logN)
    assert np.max(np.abs(back - z)) < N / scale
    assert np.max(np.abs(orc.decode_direct(orc.encode(z, scale, logN), scale, logN) - back)) < 1e-9
    # slot k sits at zeta^(5^k): conjugate-symmetric values give real coefficients by construction,
    # and rotating the slot vector left by one equals the automorphism X -> X^5 on coefficients
    m = orc.encode(z, scale, logN)
    rot = [0] * N
    for t in range(N):
        i = (t * 5) % (2 * N)
        if i < N:
            rot[i] = m[t]
        else:
            rot[i - N] = -m[t]
    assert np.max(np.abs(orc.decode(rot, scale, logN) - np.roll(z, -1))) < N / scale


# ---------------------------------------------------------------- encryption
def test_encryption_noise_is_exactly_r_e_plus_e0_plus_e1_s():
    M = Material(4, 3, 20, 1, 21, 1, seed=15)
    O = M.O
    level = 3
    z = wl.slots_complex(O.N // 2, 15)
    scale = 2.0**30
    m = orc.encode(z, scale, 4)
    pt = O.ntt_limbs(orc.to_rns(m, O.q[:level]), list(range(level)))
    r = wl.ternary(O.N, 15, "r")
    e0 = wl.gaussian_error(O.N, 15, "e0")
    e1 = wl.gaussian_error(O.N, 15, "e1")
    ct = O.encrypt(M.pk, pt, r, e0, e1, level)
    e = wl.gaussian_error(O.N, 15, "pk.e")  # the draw Material used for the public key
    s_int = [int(v) for v in M.s]
    noise = poly_mul_negacyclic_int([int(v) for v in r], [int(v) for v in e])
    e1s = poly_mul_negacyclic_int([int(v) for v in e1], s_int)
    want = [m[n] + noise[n] + int(e0[n]) + e1s[n] for n in range(O.N)]
    assert M.decrypt_poly(ct, level) == want


def test_decrypt_encrypt_roundtrip_config_sizes():
    """decrypt(encrypt(m)) recovers m within 1e-6 at scale 2^40 (N = 2^12 here)."""
    M = Material(12, 3, 50, 1, 51, 1, seed=16)
    z = wl.slots_complex(M.N // 2, 16)
    ct = M.encrypt(z, 2.0**40, 3, "x")
    assert np.max(np.abs(M.decrypt(ct, 2.0**40, 3) - z)) < 1e-6


# ---------------------------------------------------------------- end to end
def test_hmul_relin_rescale_decrypts_to_product_tiny_shape():
    """the tiny workload shape: N=2^12, 3x40-bit + 41-bit special, scale 2^30 -> 1e-2 (output scale ~2^20)"""
    p = wl.PRESETS["tiny"]
    M = Material(p.logN, p.n_q, p.q_bits, p.k, p.special_bits, p.alpha, seed=1)
    scale = 2.0**p.log_scale
    za, zb = wl.slots_complex(M.N // 2, 1, "a"), wl.slots_complex(M.N // 2, 1, "b")
    a, b = M.encrypt(za, scale, 3, "a"), M.encrypt(zb, scale, 3, "b")
    out = M.O.hmul_relin_rescale(a, b, M.rlk, 3)
    got = M.decrypt(out, scale * scale / M.O.q[2], 2)
    assert np.max(np.abs(got - za * zb)) < 1e-2
    # the composite is the strict sequence
    seq = M.O.rescale(M.O.relin(M.O.tensor(a, b, 3), M.rlk, 3), 3)
    assert np.array_equal(seq, out)


def test_hmul_at_scale_2e40_within_1e3():
    M = Material(11, 4, 50, 1, 51, 1, seed=17)
    scale = 2.0**40
    za, zb = wl.slots_real(M.N // 2, 17, "a"), wl.slots_real(M.N // 2, 17, "b")
    a, b = M.encrypt(za, scale, 4, "a"), M.encrypt(zb, scale, 4, "b")
    out = M.O.hmul_relin_rescale(a, b, M.rlk, 4)
    got = M.decrypt(out, scale * scale / M.O.q[3], 3)
    assert np.max(np.abs(got - za * zb)) < 1e-3
    assert np.max(np.abs(got - za * zb)) < 1e-5  # expected size of the error at this N


def test_divround_mixed_dropped_set():
    """DivRound over B = {last q, every special prime}: floor((x + h)/B) - u with 0 <= u <= |B|-1, from Python integers."""
    O = _small_oracle(alpha=2, k=2, n_q=4)
    cidx, bidx = [0, 1, 2], [3, O.n_q, O.n_q + 1]
    mods = [O.moduli[i] for i in cidx + bidx]
    B = math.prod(O.moduli[i] for i in bidx)
    x = wl.uniform_limbs(mods, O.N, 9, 33, 3)
    xint = orc.crt_reconstruct(x, mods, centered=False)
    out = O.divround_coef(x, cidx, bidx)
    out_exact = O.divround_coef(x, cidx, bidx, exact=True)
    us = set()
    for n in range(O.N):
        exact = (xint[n] + B // 2) // B
        u = [u for u in range(len(bidx)) if all(int(out[i][n]) == (exact - u) % O.moduli[c] for i, c in enumerate(cidx))]
        assert u
        us.add(u[0])
        assert all(int(out_exact[i][n]) == exact % O.moduli[c] for i, c in enumerate(cidx))
    assert len(us) > 1  # the plain form does overshoot on this input, the exact form never


@pytest.mark.parametrize("nb,bits", [(2, 20), (3, 20), (4, 20), (2, 50), (4, 50)])
def test_divround_exact_is_round_to_nearest(nb, bits):
    """the exact form of DivRound returns floor((x + h)/B) itself, |x/B - out| <= 1/2, for any number of dropped primes"""
    O = orc.Oracle(5, 3, bits, nb, bits + 1, nb)
    cidx, bidx = [0, 1, 2], [O.n_q + m for m in range(nb)]
    mods = [O.moduli[i] for i in cidx + bidx]
    B = math.prod(O.moduli[i] for i in bidx)
    x = wl.uniform_limbs(mods, O.N, 10, nb, bits)
    xint = orc.crt_reconstruct(x, mods, centered=False)
    out = O.divround_coef(x, cidx, bidx, exact=True)
    QC = math.prod(O.moduli[i] for i in cidx)
    got = orc.crt_reconstruct(out, [O.moduli[c] for c in cidx], centered=False)
    for n in range(O.N):
        exact = (xint[n] + B // 2) // B
        assert got[n] == exact % QC and abs(xint[n] - exact * B) <= B // 2


def _coef_centered(O, ct, level):
    """[2][level][N] evaluation form -> two lists of centered Python integers"""
    idx = list(range(level))
    return [orc.crt_reconstruct(O.intt_limbs(ct[c], idx), [O.q[i] for i in idx]) for c in range(2)]


@pytest.mark.parametrize("alpha,k,n_q,level", [(1, 1, 3, 3), (2, 2, 5, 5), (2, 2, 5, 4), (3, 3, 7, 5)])
def test_merged_division_with_zero_key_is_division_of_P_times_d(alpha, k, n_q, level):
    """With an all-zero switching key the accumulators vanish and the merged result is DivRound_{q_last, P}(P*d_c):
    floor((P*D + h)/(P*q_last)) exactly, with D the integer d_c in [0, Q_level) (Python integers)."""
    O = _small_oracle(alpha, k, n_q)
    a = np.stack([wl.uniform_limbs(O.q[:level], O.N, 40, c, level) for c in range(2)])
    b = np.stack([wl.uniform_limbs(O.q[:level], O.N, 41, c, level) for c in range(2)])
    zero_key = np.zeros((O.beta_top, 2, O.n_q + O.k, O.N), dtype=np.uint64)
    out = O.hmul_relin_rescale_merged(a, b, zero_key, level)
    d = O.tensor(a, b, level)
    idx = list(range(level))
    P = math.prod(O.p)
    B = P * O.q[level - 1]
    Qout = math.prod(O.q[: level - 1])
    for c in range(2):
        D = orc.crt_reconstruct(O.intt_limbs(d[c], idx), [O.q[i] for i in idx], centered=False)
        got = orc.crt_reconstruct(O.intt_limbs(out[c], idx[:-1]), [O.q[i] for i in idx[:-1]], centered=False)
        for n in range(O.N):
            exact = (P * D[n] + B // 2) // B
            assert got[n] == exact % Qout


@pytest.mark.parametrize("alpha,k,n_q,level", [(1, 1, 3, 3), (2, 2, 5, 5), (2, 2, 5, 4), (3, 3, 7, 6)])
def test_merged_division_differs_from_two_divisions_by_rounding_only(alpha, k, n_q, level):
    """round(round(acc/P + d)/q) against one division of acc + P*d by P*q: the two rounding rules differ by at most
    one unit per coefficient, and a wrong factor, basis or term would differ by about a whole modulus."""
    M = Material(5, n_q, 20, k, 21, alpha, seed=42)
    O = M.O
    a = np.stack([wl.uniform_limbs(O.q[:level], O.N, 42, c, level) for c in range(2)])
    b = np.stack([wl.uniform_limbs(O.q[:level], O.N, 43, c, level) for c in range(2)])
    strict = _coef_centered(O, O.hmul_relin_rescale(a, b, M.rlk, level), level - 1)
    merged = _coef_centered(O, O.hmul_relin_rescale_merged(a, b, M.rlk, level), level - 1)
    Qout = math.prod(O.q[: level - 1])
    worst = 0
    for c in range(2):
        for n in range(O.N):
            diff = (merged[c][n] - strict[c][n]) % Qout
            diff = diff - Qout if diff > Qout // 2 else diff
            worst = max(worst, abs(diff))
    assert worst <= 1


def test_merged_division_decrypts_to_product():
    M = Material(11, 4, 50, 1, 51, 1, seed=17)
    scale = 2.0**40
    za, zb = wl.slots_real(M.N // 2, 17, "a"), wl.slots_real(M.N // 2, 17, "b")
    a, b = M.encrypt(za, scale, 4, "a"), M.encrypt(zb, scale, 4, "b")
    got = M.decrypt(M.O.hmul_relin_rescale_merged(a, b, M.rlk, 4), scale * scale / M.O.q[3], 3)
    assert np.max(np.abs(got - za * zb)) < 1e-5
    M = Material(8, 6, 50, 3, 51, 3, seed=18)
    scale = 2.0**50
    za, zb = wl.slots_real(M.N // 2, 18, "a"), wl.slots_real(M.N // 2, 18, "b")
    for level in (6, 5, 4):
        a, b = M.encrypt(za, scale, level, "a"), M.encrypt(zb, scale, level, "b")
        got = M.decrypt(M.O.hmul_relin_rescale_merged(a, b, M.rlk, level), scale * scale / M.O.q[level - 1], level - 1)
        assert np.max(np.abs(got - za * zb)) < 1e-6


def test_lazy_relinearisation_decrypts_to_the_sum_of_products():
    """one relinearisation and one rescale for a sum of products: decrypts to sum_t a_t*b_t, has the noise of ONE key
    switch (not worse than the sum of separately relinearised products), and with one term is the plain product"""
    M = Material(8, 6, 50, 3, 51, 3, seed=45)
    O = M.O
    scale, level, terms = 2.0**50, 5, 4
    za = [wl.slots_real(M.N // 2, 45, ("a", t)) for t in range(terms)]
    zb = [wl.slots_real(M.N // 2, 45, ("b", t)) for t in range(terms)]
    a = np.stack([M.encrypt(za[t], scale, level, ("a", t)) for t in range(terms)])
    b = np.stack([M.encrypt(zb[t], scale, level, ("b", t)) for t in range(terms)])
    want = sum(x * y for x, y in zip(za, zb))
    out = O.hmul_sum_relin_rescale(a, b, M.rlk, level)
    s_out = scale * scale / O.q[level - 1]
    err_lazy = np.max(np.abs(M.decrypt(out, s_out, level - 1) - want))
    sep = O.hmul_relin_rescale(a[0], b[0], M.rlk, level)
    for t in range(1, terms):
        sep = O.add(sep, O.hmul_relin_rescale(a[t], b[t], M.rlk, level), level - 1)
    err_sep = np.max(np.abs(M.decrypt(sep, s_out, level - 1) - want))
    assert err_lazy < 1e-6 and err_lazy < 2 * err_sep + 1e-9
    assert not np.array_equal(out, sep)
    assert np.array_equal(O.hmul_sum_relin_rescale(a[:1], b[:1], M.rlk, level), O.hmul_relin_rescale(a[0], b[0], M.rlk, level))
    # the tensors add limb-wise: the decrypted polynomial of the summed tensor is the sum of the products' (mod Q)
    Q = math.prod(O.q[:level])
    d_sum = [0] * O.N
    for t in range(terms):
        d_sum = [(x + y) % Q for x, y in zip(d_sum, M.decrypt_poly(O.tensor(a[t], b[t], level), level))]
    lazy_unrescaled = O.relin(np.stack([O.tensor(a[t], b[t], level) for t in range(terms)]).astype(object).sum(axis=0) % np.array(O.q[:level], dtype=object)[None, :, None], M.rlk, level)
    got = M.decrypt_poly(lazy_unrescaled, level)
    worst = max(abs(((x - y + Q // 2) % Q) - Q // 2) for x, y in zip(got, d_sum))
    assert worst < 2**40  # key-switch noise only (Q is 250 bits)


def test_hybrid_keyswitch_alpha3_end_to_end():
    M = Material(8, 6, 50, 3, 51, 3, seed=18, rotations=(3,))
    scale = 2.0**50
    za, zb = wl.slots_real(M.N // 2, 18, "a"), wl.slots_real(M.N // 2, 18, "b")
    for level in (6, 5, 4):
        a, b = M.encrypt(za, scale, level, "a"), M.encrypt(zb, scale, level, "b")
        out = M.O.hmul_relin_rescale(a, b, M.rlk, level)
        got = M.decrypt(out, scale * scale / M.O.q[level - 1], level - 1)
        assert np.max(np.abs(got - za * zb)) < 1e-6
    r = M.O.rotate(a, 3, M.gk[3], 4)
    assert np.max(np.abs(M.decrypt(r, scale, 4) - np.roll(za, -3))) < 1e-6


def test_rotation_permutation_formula_and_direction():
    M = Material(6, 3, 30, 1, 31, 1, seed=19, rotations=(1, 5))
    O = M.O
    for r in (1, 5):
        g = orc.galois_element(6, r)
        assert g == pow(5, r, 2 * O.N)
        for t in range(3):
            a = wl.uniform_limbs([O.q[t]], O.N, 19, r, t)[0]
            via_coef = O.ntt_limbs(O.automorphism_coef(O.intt_limbs(a[None], [t])[0], g, t)[None], [t])[0]
            assert np.array_equal(O.automorphism_eval(a, g), via_coef)
        z = wl.slots_complex(O.N // 2, 19, r)
        ct = M.encrypt(z, 2.0**25, 3, r)
        out = O.rotate(ct, r, M.gk[r], 3)
        assert np.max(np.abs(M.decrypt(out, 2.0**25, 3) - np.roll(z, -r))) < 1e-3


@pytest.mark.parametrize("shape,level", [((6, 3, 30, 1, 31, 1), 3), ((6, 5, 30, 2, 31, 2), 5), ((6, 5, 30, 2, 31, 2), 4), ((5, 7, 30, 3, 31, 3), 5)])
def test_hoisted_rotations_decrypt_to_rotated_slots_with_keyswitch_noise_only(shape, level):
    """every rotation from the shared ModUp: the decrypted POLYNOMIAL is the automorphism of the input's (Python
    integers) up to key-switch noise as small as the plain rotation's, and the slots are the rotated slots"""
    rots = (1, 5, 7)
    M = Material(*shape, seed=44, rotations=rots)
    O = M.O
    z = wl.slots_complex(O.N // 2, 44, level)
    ct = M.encrypt(z, 2.0**25, level, "h")
    outs = O.rotate_hoisted(ct, rots, [M.gk[r] for r in rots], level)
    Q = math.prod(O.q[:level])
    m_in = M.decrypt_poly(ct, level)
    for idx, r in enumerate(rots):
        g = orc.galois_element(O.logN, r)
        want = [0] * O.N
        for t in range(O.N):
            i = (t * g) % (2 * O.N)
            if i < O.N:
                want[i] = m_in[t]
            else:
                want[i - O.N] = -m_in[t]
        worst = {}
        for name, out in (("hoisted", outs[idx]), ("plain", O.rotate(ct, r, M.gk[r], level))):
            got = M.decrypt_poly(out, level)
            noise = [((a - b + Q // 2) % Q) - Q // 2 for a, b in zip(got, want)]
            worst[name] = max(abs(v) for v in noise)
        assert worst["hoisted"] < 4 * max(worst["plain"], 64), worst
        assert np.max(np.abs(M.decrypt(outs[idx], 2.0**25, level) - np.roll(z, -r))) < 1e-3
        # a rotation does not depend on the others in the list
        assert np.array_equal(outs[idx], O.rotate_hoisted(ct, [r], [M.gk[r]], level)[0])
    assert not np.array_equal(outs[0], O.rotate(ct, rots[0], M.gk[rots[0]], level))  # a different lift: other bits


def _square_pad(M):
    n = 1
    while n < max(M.shape):
        n *= 2
    out = np.zeros((n, n))
    out[: M.shape[0], : M.shape[1]] = M
    return out


def _packed_layer(M_, shape, seed, scale_bits=30):
    """encrypt a vector replicated over the slots, apply the matrix through rotations, decrypt"""
    Mt = Material(*shape, seed=seed)
    O = Mt.O
    level, n_slots = O.n_q, O.N // 2
    Msq = _square_pad(np.asarray(M_, dtype=np.float64))
    n = Msq.shape[0]
    diags = orc.matrix_diagonals(Msq, n_slots)
    Mt = Material(*shape, seed=seed, rotations=tuple(d for d in diags if d))
    O = Mt.O
    z = np.zeros(n)
    z[: M_.shape[1]] = wl.slots_real(n, seed, "vec").real[: M_.shape[1]]
    scale = 2.0**scale_bits
    x = Mt.encrypt(np.tile(z, n_slots // n).astype(complex), scale, level, "vec")
    pts = {d: Mt.encode(v.astype(complex), float(O.q[level - 1]), level) for d, v in diags.items()}
    out = O.linear_transform(x, pts, Mt.gk, level)
    got = Mt.decrypt(out, scale, level - 1)
    return got.real[:n], Msq @ z, diags


def test_packed_fully_connected_layer_decrypts_to_matrix_vector_product():
    """single-image packing: a dense 16x16 layer on one ciphertext through 15 rotations from one shared ModUp"""
    W = wl.weights_float((16, 16), 46, "fc")
    got, want, diags = _packed_layer(W, (6, 4, 40, 2, 41, 2), 46)
    assert sorted(diags) == list(range(16))
    assert np.max(np.abs(got - want)) < 1e-4
    # a rectangular layer (10 outputs from 13 inputs) is the same thing zero-padded
    W2 = wl.weights_float((10, 13), 47, "fc")
    got, want, _ = _packed_layer(W2, (6, 4, 40, 2, 41, 2), 47)
    assert np.max(np.abs(got[:10] - want[:10])) < 1e-4 and np.max(np.abs(got[10:])) < 1e-4


def test_packed_convolution_decrypts_to_the_convolution():
    """single-image packing: 2 -> 2 channels, 3x3, zero padding 1 on a 4x4 image in 32 slots; the matrix is sparse, only
    its non-zero diagonals cost a rotation; checked against a direct convolution, not against the matrix"""
    w = wl.weights_float((2, 2, 3, 3), 48, "conv")
    Mc = orc.conv_as_matrix(w, 4, 4, 1)
    got, want, diags = _packed_layer(Mc, (7, 4, 40, 2, 41, 2), 48)
    assert len(diags) < 32
    z = np.zeros(32)
    z[:32] = wl.slots_real(32, 48, "vec").real
    img = z.reshape(2, 4, 4)
    padded = np.zeros((2, 6, 6))
    padded[:, 1:5, 1:5] = img
    direct = np.array([[[sum(w[o, c, u, v] * padded[c, y + u, x + v] for c in range(2) for u in range(3) for v in range(3))
                         for x in range(4)] for y in range(4)] for o in range(2)]).reshape(-1)
    assert np.max(np.abs(want - direct)) < 1e-12
    assert np.max(np.abs(got - direct)) < 1e-4


def test_strided_convolution_and_pooling_matrices_match_the_layer_definitions():
    """the matrices of the single-image packing against direct loops over the layer definitions: a stride-2 convolution
    with zero padding, and 2x2 average pooling (plain and with a padded border)"""
    g = wl.rng(60, "mat")
    C, H, W, O, k, stride, pad = 2, 7, 6, 3, 3, 2, 1
    w = g.normal(size=(O, C, k, k))
    img = g.normal(size=(C, H, W))
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    padded = np.zeros((C, H + 2 * pad, W + 2 * pad))
    padded[:, pad:pad + H, pad:pad + W] = img
    direct = np.array([[[sum(w[o, c, u, v] * padded[c, y * stride + u, x * stride + v] for c in range(C) for u in range(k) for v in range(k))
                         for x in range(Wo)] for y in range(Ho)] for o in range(O)])
    assert np.allclose(orc.conv_as_matrix(w, H, W, pad, stride) @ img.reshape(-1), direct.reshape(-1), atol=1e-12)
    # stride 1 is what the earlier single-layer pins use
    assert np.array_equal(orc.conv_as_matrix(w, H, W, pad, 1), orc.conv_as_matrix(w, H, W, pad))
    for pp in (0, 1):
        Hp, Wp = (H + 2 * pp) // 2, (W + 2 * pp) // 2
        padded = np.zeros((C, H + 2 * pp + 2, W + 2 * pp + 2))
        padded[:, pp:pp + H, pp:pp + W] = img
        pooled = np.array([[[padded[c, 2 * y:2 * y + 2, 2 * x:2 * x + 2].mean() for x in range(Wp)] for y in range(Hp)] for c in range(C)])
        assert np.allclose(orc.pool_as_matrix(C, H, W, 2, pp) @ img.reshape(-1), pooled.reshape(-1), atol=1e-12)


def _run_single_image(topology, shape, seed, sigma=0.25, bsgs=False):
    import helpers
    probe = orc.Oracle(*shape)
    n_slots, level, s = probe.N // 2, probe.n_q, 2.0 ** 50
    weights = wl.cnn_weights_float(topology, seed, sigma=sigma)
    stages = helpers.network_stage_matrices(topology, weights)
    n = helpers.network_period(stages, n_slots)
    # the rotation offsets are known from the matrices alone: keys first, then the encodings
    rots = sorted({d for st in stages if st[0] == "linear" for dd in orc.block_diagonals(st[1], n, n_slots).values() for d in dd if d})
    if bsgs:  # every offset d = g*baby + b needs the keys of b and of g*baby only
        baby = helpers.bsgs_baby(n)
        rots = sorted({d % baby for d in rots if d % baby} | {d - d % baby for d in rots if d >= baby})
    M = Material(*shape, seed=seed, rotations=tuple(rots))
    O = M.O
    ist, rots2, out_level, out_scale = helpers.network_integer_stages(stages, O.q, level, s, n, n_slots, M.encode, bsgs=bsgs)
    assert rots2 == rots
    C, H, W = wl.CNN_TOPOLOGIES[topology]["input"]
    img = wl.slots_real(C * H * W, seed, "image", lo=0.0, hi=1.0).real
    blocks = -(-img.size // n)
    zin = np.zeros(blocks * n)
    zin[: img.size] = img
    xs = [M.encrypt(np.tile(zin[j * n:(j + 1) * n], n_slots // n).astype(complex), s, level, ("img", j)) for j in range(blocks)]
    outs, lvl = O.packed_network(xs, ist, M.rlk, M.gk, level)
    assert lvl == out_level
    want = helpers.network_float(stages, img)
    got = np.concatenate([M.decrypt(o, out_scale, lvl).real[:n] for o in outs])
    return got, want, blocks, len(outs), len(rots)


def test_single_image_network_decrypts_to_the_float_network():
    """strided convolution, degree-2 activation, pooling merged into the fully connected layer after it, activation, fully
    connected: one image in ONE ciphertext (128 slots), against the float network"""
    got, want, n_in, n_out, n_rot = _run_single_image("single_image_tiny", (8, 8, 50, 2, 51, 2), 61)
    assert (n_in, n_out) == (1, 1) and n_rot > 20
    assert np.max(np.abs(want)) > 1e-3
    assert np.max(np.abs(got[: want.size] - want)) < 1e-4 and np.max(np.abs(got[want.size:])) < 1e-4


def test_single_image_network_with_baby_and_giant_steps():
    """the same network with every linear stage in baby-step / giant-step form: the same decrypted result from a third of
    the rotation keys (period 128: baby = 16, at most 15 + 7 offsets)"""
    got, want, n_in, n_out, n_rot = _run_single_image("single_image_tiny", (8, 8, 50, 2, 51, 2), 61, bsgs=True)
    _, _, _, _, n_rot_plain = _run_single_image("single_image_tiny", (8, 8, 50, 2, 51, 2), 61)
    assert (n_in, n_out) == (1, 1) and n_rot <= 22 and n_rot_plain > 3 * n_rot // 2
    assert np.max(np.abs(got[: want.size] - want)) < 1e-4 and np.max(np.abs(got[want.size:])) < 1e-4


def test_single_image_network_with_a_vector_that_spans_two_ciphertexts():
    """the same network with 64 slots per ciphertext: the 128 input values take two ciphertexts, the first layer is a
    1 x 2 block matrix, every input block rotated once for the output block"""
    got, want, n_in, n_out, _ = _run_single_image("single_image_tiny", (7, 8, 50, 2, 51, 2), 61)
    assert (n_in, n_out) == (2, 1)
    assert np.max(np.abs(got[: want.size] - want)) < 1e-4


def test_block_linear_transform_with_several_output_ciphertexts():
    """a 70 x 50 dense matrix with 32 slots per ciphertext: 2 input blocks, 3 output blocks"""
    import helpers
    shape = (6, 3, 50, 2, 51, 2)
    probe = orc.Oracle(*shape)
    n = probe.N // 2
    Wm = wl.weights_float((70, 50), 62, "blk", sigma=0.3)
    dg = orc.block_diagonals(Wm, n, n)
    assert sorted(dg) == [(i, j) for i in range(3) for j in range(2)]
    rots = sorted({d for dd in dg.values() for d in dd if d})
    M = Material(*shape, seed=62, rotations=tuple(rots))
    O = M.O
    z = np.zeros(2 * n)
    z[:50] = wl.slots_real(50, 62, "z").real
    s = 2.0 ** 40
    xs = [M.encrypt(z[j * n:(j + 1) * n].astype(complex), s, 3, ("z", j)) for j in range(2)]
    pts = {ij: {d: M.encode(v.astype(complex), float(O.q[2]), 3) for d, v in dd.items()} for ij, dd in dg.items()}
    outs = O.linear_transform_blocks(xs, pts, M.gk, 3)
    got = np.concatenate([M.decrypt(o, s, 2).real for o in outs])
    want = np.zeros(3 * n)
    want[:70] = Wm @ z[:50]
    assert np.max(np.abs(got - want)) < 1e-4
    # one block in each direction is the single-ciphertext transform, bit for bit
    W1 = wl.weights_float((20, 30), 63, "one", sigma=0.3)
    d1 = orc.block_diagonals(W1, n, n)
    assert list(d1) == [(0, 0)]
    M1 = Material(*shape, seed=63, rotations=tuple(d for d in d1[(0, 0)] if d))
    x = M1.encrypt(wl.slots_real(n, 63, "x"), s, 3, "x")
    p1 = {d: M1.encode(v.astype(complex), float(M1.O.q[2]), 3) for d, v in d1[(0, 0)].items()}
    assert np.array_equal(M1.O.linear_transform_blocks([x], {(0, 0): p1}, M1.gk, 3)[0], M1.O.linear_transform(x, p1, M1.gk, 3))


def test_baby_step_giant_step_transform_decrypts_to_the_same_product_with_fewer_keys():
    """the 70 x 50 matrix again (2 input blocks, 3 output blocks, 32 slots): with baby = 8 every offset d = 8 g + b needs
    only the keys of b = 1..7 and of 8, 16, 24 instead of all 31; the decrypted result is M z as before; one giant
    group only (baby >= every offset) rotates nothing after the sums and is linear_transform_blocks bit for bit; the
    pre-rotated diagonals are what the identity  diag_d * roll(z, -d) = roll(roll(diag_d, g*baby) * roll(z, -b), -g*baby)  asks"""
    shape = (6, 3, 50, 2, 51, 2)
    probe = orc.Oracle(*shape)
    n = probe.N // 2
    Wm = wl.weights_float((70, 50), 62, "blk", sigma=0.3)
    dg = orc.block_diagonals(Wm, n, n)
    baby = 8
    bs = orc.bsgs_diagonals(dg, baby)
    zt = wl.slots_real(n, 64, "zt").real
    for key in dg:  # the identity on plain vectors, every diagonal
        for d, v in dg[key].items():
            g, b = divmod(d, baby)
            assert np.allclose(v * np.roll(zt, -d), np.roll(bs[key][(g, b)] * np.roll(zt, -b), -g * baby))
    needed = sorted({b for dd in bs.values() for (_, b) in dd if b} | {g * baby for dd in bs.values() for (g, _) in dd if g})
    assert needed == [1, 2, 3, 4, 5, 6, 7, 8, 16, 24]
    M = Material(*shape, seed=62, rotations=tuple(needed))
    O = M.O
    z = np.zeros(2 * n)
    z[:50] = wl.slots_real(50, 62, "z").real
    s = 2.0 ** 40
    xs = [M.encrypt(z[j * n:(j + 1) * n].astype(complex), s, 3, ("z", j)) for j in range(2)]
    pts = {ij: {gb: M.encode(v.astype(complex), float(O.q[2]), 3) for gb, v in dd.items()} for ij, dd in bs.items()}
    outs = O.linear_transform_bsgs(xs, pts, M.gk, 3, baby)
    assert len(outs) == 3 and all(o.shape == (2, 2, O.N) for o in outs)
    got = np.concatenate([M.decrypt(o, s, 2).real for o in outs])
    want = np.zeros(3 * n)
    want[:70] = Wm @ z[:50]
    assert np.max(np.abs(got - want)) < 1e-4
    # a baby step that covers every offset: no giant rotation, the same sums in the same order as the plain block transform
    M2 = Material(*shape, seed=62, rotations=tuple(range(1, n)))
    pts_plain = {ij: {d: M2.encode(v.astype(complex), float(O.q[2]), 3) for d, v in dd.items()} for ij, dd in dg.items()}
    pts_one = {ij: {(0, d): pt for d, pt in dd.items()} for ij, dd in pts_plain.items()}
    xs2 = [M2.encrypt(z[j * n:(j + 1) * n].astype(complex), s, 3, ("z", j)) for j in range(2)]
    a = M2.O.linear_transform_bsgs(xs2, pts_one, M2.gk, 3, n)
    b_ = M2.O.linear_transform_blocks(xs2, pts_plain, M2.gk, 3)
    assert all(np.array_equal(x, y) for x, y in zip(a, b_))


def test_philox_known_answers():
    """Philox4x32-10 known-answer vectors published with the generator (zeros, all ones, digits of pi)"""
    assert orc.philox4x32_10([0] * 4, [0] * 2) == [0x6627E8D5, 0xE169C58D, 0xBC57AC4C, 0x9B00DBD8]
    assert orc.philox4x32_10([0xFFFFFFFF] * 4, [0xFFFFFFFF] * 2) == [0x408F276D, 0x41C83B0E, 0xA20BC7C6, 0x6D5451FD]
    assert orc.philox4x32_10([0x243F6A88, 0x85A308D3, 0x13198A2E, 0x03707344], [0xA4093822, 0x299F31D0]) == [
        0xD16CFE09, 0x94FDCCEB, 0x5001E420, 0x24126EA1]


def test_sampler_distributions_and_counter_structure():
    """ternary: each value a third of the time; Gaussian: the probabilities of round(N(0, sigma^2)) (chi-square against
    the exact masses from erf), thresholds equal to 2^64*erf(.) ; a coefficient depends only on (seed, polynomial, t)"""
    sigma, logN, rows = 3.2, 12, 64
    tern = orc.sample(0, sigma, 7, 100, rows, logN)
    n = tern.size
    assert set(np.unique(tern)) == {-1, 0, 1}
    for v in (-1, 0, 1):
        assert abs(np.mean(tern == v) - 1 / 3) < 4 * math.sqrt(2 / 9 / n)
    g = orc.sample(1, sigma, 7, 100, rows, logN)
    assert abs(np.mean(g)) < 5 * sigma / math.sqrt(n)
    assert abs(np.var(g) - (sigma**2 + 1 / 12)) < 0.1
    chi = 0.0
    for k in range(-12, 13):
        pk = 0.5 * (math.erf((k + 0.5) / (sigma * math.sqrt(2))) - math.erf((k - 0.5) / (sigma * math.sqrt(2))))
        chi += (np.sum(g == k) - n * pk) ** 2 / (n * pk)
    assert chi < 60  # 24 degrees of freedom: 60 is beyond the 99.99 % point
    T = orc.gauss_thresholds(sigma)
    for k in range(12):
        assert abs(int(T[k]) / 2.0**64 - math.erf((k + 0.5) / (sigma * math.sqrt(2)))) < 1e-14
    assert all(int(T[k]) <= int(T[k + 1]) for k in range(39)) and int(T[39]) == 2**64 - 1
    # counter structure: polynomial 103 drawn alone equals row 3 of the block; another seed gives other values
    assert np.array_equal(orc.sample(1, sigma, 7, 103, 1, logN)[0], g[3])
    assert np.array_equal(orc.sample(0, sigma, 7, 2**40 + 5, 2, 6)[1], orc.sample(0, sigma, 7, 2**40 + 6, 1, 6)[0])
    assert not np.array_equal(orc.sample(1, sigma, 8, 100, 1, logN)[0], g[0])


def test_elementwise_ops_on_decrypted_polynomials():
    M = Material(5, 3, 30, 1, 31, 1, seed=20)
    O = M.O
    level = 3
    Q = math.prod(O.q[:level])
    a = wl.uniform_limbs(O.q[:level], O.N, 20, "a", lead=(2,))
    b = wl.uniform_limbs(O.q[:level], O.N, 20, "b", lead=(2,))
    ma, mb = M.decrypt_poly(a, level), M.decrypt_poly(b, level)
    eq = lambda x, y: all((u - v) % Q == 0 for u, v in zip(x, y))
    assert eq(M.decrypt_poly(O.add(a, b, level), level), [u + v for u, v in zip(ma, mb)])
    assert eq(M.decrypt_poly(O.sub(a, b, level), level), [u - v for u, v in zip(ma, mb)])
    assert eq(M.decrypt_poly(O.mul_scalar(a, -12345678901, level), level), [-12345678901 * u for u in ma])
    assert eq(M.decrypt_poly(O.add_const(a, -77, level), level), [ma[0] - 77] + ma[1:])
    pt_coef = [int(v) for v in wl.gaussian_error(O.N, 20, "pt")]
    pt = O.ntt_limbs(orc.to_rns(pt_coef, O.q[:level]), list(range(level)))
    assert eq(M.decrypt_poly(O.mul_plain(a, pt, level), level), poly_mul_negacyclic_int(ma, pt_coef))
    dropped = O.mod_drop(a, 3, 2)
    assert np.array_equal(dropped, a[:, :2])


def _conv_reference(x, w, stride, pad):
    C_, H, W = x.shape[:3]
    O_, _, kh, kw = w.shape
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    out = np.zeros((O_, Ho, Wo) + x.shape[3:], dtype=x.dtype)
    for o in range(O_):
        for y in range(Ho):
            for xx in range(Wo):
                for c in range(C_):
                    for u in range(kh):
                        for v in range(kw):
                            iy, ix = y * stride + u - pad, xx * stride + v - pad
                            if 0 <= iy < H and 0 <= ix < W:
                                out[o, y, xx] = out[o, y, xx] + w[o, c, u, v] * x[c, iy, ix]
    return out


@pytest.mark.parametrize("stride,pad", [(2, 0), (1, 1)])
def test_conv_mac_is_linear_in_decrypted_polynomials(stride, pad):
    M = Material(4, 3, 30, 1, 31, 1, seed=21)
    O = M.O
    level = 3
    Q = math.prod(O.q[:level])
    Cc, H, W, Oc, kh = 2, 5, 5, 3, 3
    x = wl.uniform_limbs(O.q[:level], O.N, 21, "x", lead=(Cc, H, W, 2))
    w = wl.rng(21, "w").integers(-(2**29), 2**29, size=(Oc, Cc, kh, kh), dtype=np.int64)
    out = O.conv2d_mac(x, w, stride, pad, level)
    mx = np.array([[[M.decrypt_poly(x[c, y, xx], level) for xx in range(W)] for y in range(H)] for c in range(Cc)], dtype=object)
    want = _conv_reference(mx, w.astype(object), stride, pad)
    assert out.shape[:3] == want.shape[:3]
    for o in range(out.shape[0]):
        for y in range(out.shape[1]):
            for xx in range(out.shape[2]):
                got = M.decrypt_poly(out[o, y, xx], level)
                assert all((int(g) - int(v)) % Q == 0 for g, v in zip(got, want[o, y, xx]))
    # FC = flat 1x1 case
    f = x[:, 0, 0]
    wf = w[:, :, 0, 0]
    fc = O.fc_mac(f, wf, level)
    for o in range(Oc):
        got = M.decrypt_poly(fc[o], level)
        want_o = [sum(int(wf[o, c]) * mx[c, 0, 0][n] for c in range(Cc)) for n in range(O.N)]
        assert all((g - v) % Q == 0 for g, v in zip(got, want_o))


def test_conv_layer_decrypts_to_float_convolution():
    """slots-as-batch conv + rescale vs a float convolution of the slot values"""
    M = Material(6, 3, 40, 0, 41, 1, seed=22)
    O = M.O
    level = 3
    scale = 2.0**30
    Cc, H, W, Oc, kh, stride = 2, 6, 6, 2, 3, 2
    imgs = wl.rng(22, "img").uniform(0, 1, size=(Cc, H, W, O.N // 2))
    x = np.array([[[M.encrypt(imgs[c, y, xx].astype(np.complex128), scale, level, (c, y, xx)) for xx in range(W)] for y in range(H)] for c in range(Cc)])
    wf = wl.weights_float((Oc, Cc, kh, kh), 22)
    wi = np.rint(wf * O.q[level - 1]).astype(np.int64)
    out = O.conv2d_mac(x, wi, stride, 0, level)
    want = _conv_reference(imgs, wf, stride, 0)
    for o in range(Oc):
        for y in range(out.shape[1]):
            for xx in range(out.shape[2]):
                got = M.decrypt(O.rescale(out[o, y, xx], level), scale, level - 1)
                assert np.max(np.abs(got.real - want[o, y, xx])) < 1e-3


def test_activation_schedules_match_float_polynomials():
    M = Material(8, 6, 50, 3, 51, 3, seed=23)
    O = M.O
    level = 6
    s = 2.0**50
    z = wl.slots_real(O.N // 2, 23)
    x = M.encrypt(z, s, level, "x")
    y = O.square(x, M.rlk, level)  # level 5
    s_y = s * s / O.q[5]
    assert np.max(np.abs(M.decrypt(y, s_y, 5) - z * z)) < 1e-6
    s_2 = s_y * s_y / O.q[4]
    s_3 = s_2 * s_y / O.q[3]
    c_m002 = round(-0.02 * O.q[4])
    c_025 = round(0.25 * s_2)
    c_05 = round(0.5 * s_3)
    out = O.poly3(y, M.rlk, 5, c_m002, c_025, c_05)
    yv = (z * z).real
    want = 0.5 + 0.25 * yv - 0.02 * yv**3
    assert np.max(np.abs(M.decrypt(out, s_3, 3).real - want)) < 1e-5


def test_paper_degree2_activation_polynomial():
    """the degree-2 ReLU substitute printed in the paper's section 3.1, coefficients from tests/golden"""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "activation_poly_deg2.txt")
    vals = [float(l.split()[1]) for l in open(path) if l.strip() and not l.startswith("#")]
    c2, c1 = vals
    M = Material(8, 4, 50, 1, 51, 1, seed=24)
    O = M.O
    level = 4
    s = 2.0**40
    z = wl.slots_real(O.N // 2, 24, lo=-4.0, hi=4.0)
    x = M.encrypt(z, s, level, "x")
    # c2*x^2: RS(Relin(x*x)) then scalar (scale q_2 so the rescale restores the scale); c1*x likewise
    x2 = O.square(x, M.rlk, level)
    s2 = s * s / O.q[3]
    t2 = O.rescale(O.mul_scalar(x2, round(c2 * O.q[2]), 3), 3)  # level 2, scale s2
    t1 = O.rescale(O.mul_scalar(O.mod_drop(x, 4, 3), round(c1 * s2 / s * O.q[2]), 3), 3)  # level 2, scale s2
    out = O.add(t2, t1, 2)
    want = c2 * z.real**2 + c1 * z.real
    assert np.max(np.abs(M.decrypt(out, s2, 2).real - want)) < 1e-4


def test_sum_pool_is_sum_of_decrypted_polynomials():
    M = Material(4, 3, 30, 1, 31, 1, seed=25)
    O = M.O
    level = 3
    Q = math.prod(O.q[:level])
    x = wl.uniform_limbs(O.q[:level], O.N, 25, "x", lead=(2, 5, 4, 2))
    out = O.sum_pool2d(x, 2, level)
    assert out.shape[:3] == (2, 2, 2)
    for c in range(2):
        for y in range(2):
            for xx in range(2):
                got = M.decrypt_poly(out[c, y, xx], level)
                parts = [M.decrypt_poly(x[c, 2 * y + u, 2 * xx + v], level) for u in range(2) for v in range(2)]
                assert all((g - sum(p[n] for p in parts)) % Q == 0 for n, g in enumerate(got))


def _float_network(imgs, layers_f):
    """cleartext float network over arrays [C][H][W][images]; average pooling as in Table 1"""
    x = imgs
    for layer in layers_f:
        if layer[0] == "conv":
            x = _conv_reference(x, layer[1], layer[2], layer[3])
        elif layer[0] == "square":
            x = x * x
        elif layer[0] == "poly2":
            x = layer[1] * x * x + layer[2] * x
        elif layer[0] == "pool":
            k = layer[1]
            pad = layer[2] if len(layer) > 2 else 0
            x = np.pad(x, ((0, 0), (pad, pad), (pad, pad), (0, 0)))  # zero padding rows of Table 1
            Cc, H, W = x.shape[:3]
            x = x[:, : H // k * k, : W // k * k].reshape(Cc, H // k, k, W // k, k, -1).mean(axis=(2, 4))
        elif layer[0] == "fc":
            x = np.tensordot(layer[1], x.reshape(-1, x.shape[-1]), axes=1).reshape(layer[1].shape[0], 1, 1, -1)
    return x


def test_network_decrypts_to_float_network():
    """conv - square - conv - square - conv - pool - fc - square - fc over per-pixel ciphertexts against the same
    network on the slot values in floating point (section 3: the layer types of Table 1 with polynomial activations);
    the average pooling's 1/4 is folded into the next layer's integer weights"""
    name = "cnn_tiny"
    M = Material(6, 10, 50, 3, 51, 3, seed=26)
    O = M.O
    level = 10
    scale = 2.0**50
    Cc, H, W = wl.CNN_TOPOLOGIES[name]["input"]
    imgs = wl.rng(26, "img").uniform(0, 1, size=(Cc, H, W, O.N // 2))
    x = np.array([[[M.encrypt(imgs[c, y, xx].astype(np.complex128), scale, level, (c, y, xx)) for xx in range(W)] for y in range(H)] for c in range(Cc)])
    shapes = wl.cnn_shapes(name)
    wf = wl.cnn_weights_float(name, 26, sigma=1.0)
    layers_f, layers_i = [], []
    lvl, s, fold = level, scale, 1.0
    for (layer, (c, h, w), _), wt in zip(shapes, wf):
        if layer[0] in ("conv", "fc"):
            fan_in = wt[0].size
            wt = wt * (1.0 / math.sqrt(fan_in))  # keeps the activations of this random network near 0.1 .. 1
            wi = np.rint(wt * fold * O.q[lvl - 1]).astype(np.int64)
            fold = 1.0
            if layer[0] == "conv":
                layers_f.append(("conv", wt, layer[3], layer[4]))
                layers_i.append(("conv", wi, layer[3], layer[4]))
            else:
                layers_f.append(("fc", wt))
                layers_i.append(("fc", wi))
            lvl -= 1  # scale unchanged: the integer weight carries the dropped modulus
        elif layer[0] == "square":
            layers_f.append(layer)
            layers_i.append(layer)
            s = s * s / O.q[lvl - 1]
            lvl -= 1
        else:
            layers_f.append(layer)
            layers_i.append(layer)
            fold = 1.0 / (layer[1] * layer[1])
    out, out_level = O.cnn_forward(x, layers_i, M.rlk, level)
    assert out_level == lvl == 2 and out.shape[:3] == (2, 1, 1)
    want = _float_network(imgs, layers_f)
    assert 1e-3 < np.max(np.abs(want)) < 0.4  # a meaningful, decodable output at the last level
    for o in range(2):
        got = M.decrypt(out[o, 0, 0], s, out_level).real
        assert np.max(np.abs(got - want[o, 0, 0])) < 1e-6 * max(1.0, np.max(np.abs(want)))


def test_padded_sum_pool_counts_only_the_image():
    M = Material(4, 2, 30, 1, 31, 1, seed=27)
    O = M.O
    level = 2
    Q = math.prod(O.q[:level])
    x = wl.uniform_limbs(O.q[:level], O.N, 27, "x", lead=(1, 3, 3, 2))
    out = O.sum_pool2d(x, 2, level, pad=1)  # padded 5x5 -> 2x2 windows starting at -1
    assert out.shape[:3] == (1, 2, 2)
    mx = [[M.decrypt_poly(x[0, y, xx], level) for xx in range(3)] for y in range(3)]
    for y in range(2):
        for xx in range(2):
            want = [0] * O.N
            for u in range(2):
                for v in range(2):
                    iy, ix = 2 * y + u - 1, 2 * xx + v - 1
                    if 0 <= iy < 3 and 0 <= ix < 3:
                        want = [a + b for a, b in zip(want, mx[iy][ix])]
            got = M.decrypt_poly(out[0, y, xx], level)
            assert all((g - w) % Q == 0 for g, w in zip(got, want))
    # a 1x1 map padded by one and pooled 2x2 is the map itself (its one window holds three zeros)
    one = O.sum_pool2d(x[:, :1, :1], 2, level, pad=1)
    assert one.shape[:3] == (1, 1, 1) and np.array_equal(one[0, 0, 0], x[0, 0, 0])


def test_table1_topology_matches_the_paper():
    """the layer list used for the paper's network against Table 1 (rows with parameters, tests/golden)"""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "table1_layers.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    want = []
    pad = 0
    for _, kind, n, k, stride in rows:
        if kind == "zeropad":
            pad = int(k)
        elif kind == "conv":
            want.append(("conv", int(n), int(k), int(stride), pad)); pad = 0
        elif kind == "avgpool":
            want.append(("pool", int(k)) if pad == 0 else ("pool", int(k), pad)); pad = 0
        elif kind == "fc":
            want.append(("fc", int(n)))
    got = [l for l in wl.CNN_TOPOLOGIES["table1"]["layers"] if l[0] != "poly2"]
    assert got == want
    # an activation after every conv / fc layer except the last one (section 3.1)
    layers = wl.CNN_TOPOLOGIES["table1"]["layers"]
    for i, l in enumerate(layers[:-1]):
        if l[0] in ("conv", "fc"):
            assert layers[i + 1] == ("poly2",)
    assert layers[-1] == ("fc", 1)
    assert wl.cnn_shapes("table1")[-1][2] == (1, 1, 1) and wl.cnn_shapes("table1")[12][1] == (384, 1, 1)


def test_table1_like_network_with_degree2_activation_decrypts_to_float_network():
    """Table 1's layer sequence (reduced widths) with the paper's degree-2 activation polynomial (tests/golden)
    against the same network in floating point on the slot values"""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "activation_poly_deg2.txt")
    c2, c1 = [float(l.split()[1]) for l in open(path) if l.strip() and not l.startswith("#")]
    name = "table1_reduced"
    M = Material(6, 20, 50, 3, 51, 3, seed=28)
    O = M.O
    level = 20
    scale = 2.0**50
    Cc, H, W = wl.CNN_TOPOLOGIES[name]["input"]
    imgs = wl.rng(28, "img").uniform(0, 1, size=(Cc, H, W, O.N // 2))
    x = np.array([[[M.encrypt(imgs[c, y, xx].astype(np.complex128), scale, level, (c, y, xx)) for xx in range(W)] for y in range(H)] for c in range(Cc)])
    shapes = wl.cnn_shapes(name)
    wf = wl.cnn_weights_float(name, 28, sigma=1.0)
    layers_f, layers_i = [], []
    lvl, s, fold = level, scale, 1.0
    for (layer, (c, h, w), _), wt in zip(shapes, wf):
        if layer[0] in ("conv", "fc"):
            wt = wt * (3.0 / math.sqrt(wt[0].size))  # c1 = 0.5 halves the activations at every layer: keep them near 0.1 .. 1
            wi = np.rint(wt * fold * O.q[lvl - 1]).astype(np.int64)
            fold = 1.0
            layers_f.append(("conv", wt, layer[3], layer[4]) if layer[0] == "conv" else ("fc", wt))
            layers_i.append(("conv", wi, layer[3], layer[4]) if layer[0] == "conv" else ("fc", wi))
            lvl -= 1
        elif layer[0] == "poly2":
            s2 = s * s / O.q[lvl - 1]
            layers_f.append(("poly2", c2, c1))
            layers_i.append(("poly2", round(c2 * O.q[lvl - 2]), round(c1 * (s2 / s) * O.q[lvl - 2])))
            s = s2
            lvl -= 2
        else:
            layers_f.append(layer)
            layers_i.append(layer)
            fold = fold / (layer[1] * layer[1])
    out, out_level = O.cnn_forward(x, layers_i, M.rlk, level)
    assert out_level == lvl == 1 and out.shape[:3] == (1, 1, 1)
    want = _float_network(imgs, layers_f)
    assert 1e-3 < np.max(np.abs(want)) < 0.4
    got = M.decrypt(out[0, 0, 0], s, out_level).real
    assert np.max(np.abs(got - want[0, 0, 0])) < 1e-6 * max(1.0, np.max(np.abs(want)))


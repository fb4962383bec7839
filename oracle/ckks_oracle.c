/*
 * ckks_oracle.c -- plain, slow, obviously-correct CPU reference for the RNS-CKKS
 * ciphertext arithmetic behind encrypted CNN inference.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It exists only so that tests, the smoke
 * check and the benchmark's CPU-baseline leg can check and time the GPU library
 * against an independent implementation.  It shares no source, header, table or
 * constant generator with the GPU library and must never be called from the
 * product path.
 *
 * Scheme: the paper (section 2.1) fixes the public-key equations
 *     sk = (1, s),  pk = (b = -a*s + e, a),
 *     ct = (c0 = r*b + e0 + m, c1 = r*a + e1),   m ~ c0 + c1*s,
 * over R_q = Z_q[X]/(X^N + 1) (the printed exponent "n+1" is a typo for the
 * cyclotomic X^N + 1).  The paper names CKKS (its ref. [13]) as the scheme and
 * says that add and multiply are supported and that the scaling factor is
 * updated along the way (section 2.1); it gives no algorithm for either.  The
 * RNS realisation below (residue limbs, hybrid key switching with special
 * primes, rescale) is the standard public construction, written out step by
 * step in its plainest form:
 *   - every product is (unsigned __int128) a * b % q;
 *   - every residue is the canonical representative in [0, q);
 *   - polynomial products are defined by schoolbook negacyclic convolution and
 *     the transform by direct evaluation; the fast transform here (twist by
 *     psi^t, textbook radix-2 cyclic FFT, bit-reversal) is a different
 *     algorithm from the GPU's and is accepted only because tests pin it to
 *     those two definitions;
 *   - rescale / ModDown are done coefficient by coefficient in coefficient form
 *     (inverse-transform everything, divide-and-round, transform back).
 *
 * Layout everywhere: a "limb" is N uint64 words; a polynomial over l moduli is
 * [l][N]; a ciphertext is [2][l][N]; a degree-2 ciphertext is [3][l][N].
 * "Evaluation form": word j of limb i is the polynomial evaluated at
 * psi_i^(2*brev(j)+1) mod q_i, brev = log2(N)-bit reversal.
 * Modulus indices: 0..n_q-1 are the ciphertext primes q_i, n_q..n_q+k-1 the
 * special primes p_m.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef uint64_t u64;
typedef int64_t i64;
typedef unsigned __int128 u128;

/* ------------------------------------------------------------------ */
/* modular arithmetic: the definition                                  */
/* ------------------------------------------------------------------ */
u64 orc_addmod(u64 a, u64 b, u64 q) { return (u64)(((u128)a + b) % q); }
u64 orc_submod(u64 a, u64 b, u64 q) { return (u64)(((u128)a + q - (b % q)) % q); }
u64 orc_mulmod(u64 a, u64 b, u64 q) { return (u64)((u128)a * b % q); }
u64 orc_powmod(u64 a, u64 e, u64 q) {
    u64 r = 1 % q;
    a %= q;
    while (e) {
        if (e & 1) r = orc_mulmod(r, a, q);
        a = orc_mulmod(a, a, q);
        e >>= 1;
    }
    return r;
}
/* q prime */
u64 orc_invmod(u64 a, u64 q) { return orc_powmod(a, q - 2, q); }
/* signed integer -> canonical residue */
u64 orc_signed_mod(i64 v, u64 q) {
    if (v >= 0) return (u64)v % q;
    u64 m = ((u64)(-(v + 1)) + 1u) % q; /* |v| mod q without overflow at INT64_MIN */
    return m ? q - m : 0;
}

/* deterministic Miller-Rabin for 64-bit n (first twelve prime bases) */
int orc_is_prime(u64 n) {
    static const u64 bases[12] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    if (n < 2) return 0;
    for (int i = 0; i < 12; i++) {
        if (n == bases[i]) return 1;
        if (n % bases[i] == 0) return 0;
    }
    u64 d = n - 1;
    int r = 0;
    while ((d & 1) == 0) { d >>= 1; r++; }
    for (int i = 0; i < 12; i++) {
        u64 x = orc_powmod(bases[i], d, n);
        if (x == 1 || x == n - 1) continue;
        int comp = 1;
        for (int j = 1; j < r; j++) {
            x = orc_mulmod(x, x, n);
            if (x == n - 1) { comp = 0; break; }
        }
        if (comp) return 0;
    }
    return 1;
}

/*
 * Parameter rule: the `count` largest primes below 2^bits that are 1 mod 2N,
 * found by scanning 2^bits - t*2N + 1 for t = 1, 2, ...; out[0] is the largest.
 * Values listed in `exclude` are skipped.  Returns the number found.
 */
int orc_find_primes(int bits, int logN, int count, const u64 *exclude, int n_excl, u64 *out) {
    u64 twoN = (u64)2 << logN;
    u64 top = (u64)1 << bits;
    u64 floor_ = (u64)1 << (bits - 1);
    int found = 0;
    for (u64 t = 1; found < count; t++) {
        if (t * twoN >= top) break;
        u64 c = top - t * twoN + 1;
        if (c <= floor_) break;
        if (!orc_is_prime(c)) continue;
        int skip = 0;
        for (int i = 0; i < n_excl; i++) if (exclude[i] == c) skip = 1;
        if (skip) continue;
        out[found++] = c;
    }
    return found;
}

/* first x = 2, 3, ... such that psi = x^((q-1)/2N) has psi^N = -1 mod q */
u64 orc_find_psi(u64 q, int logN) {
    u64 N = (u64)1 << logN;
    for (u64 x = 2; x < q; x++) {
        u64 psi = orc_powmod(x, (q - 1) / (2 * N), q);
        if (orc_powmod(psi, N, q) == q - 1) return psi;
    }
    return 0;
}

static u64 brev(u64 x, int bits) {
    u64 r = 0;
    for (int i = 0; i < bits; i++) { r = (r << 1) | (x & 1); x >>= 1; }
    return r;
}
u64 orc_brev(u64 x, int bits) { return brev(x, bits); }

/* ------------------------------------------------------------------ */
/* the definitions: direct evaluation and schoolbook convolution       */
/* ------------------------------------------------------------------ */

/* out[j] = sum_t a[t] * psi^((2*brev(j)+1)*t) mod q      O(N^2) */
void orc_ntt_direct(const u64 *a, int logN, u64 q, u64 psi, u64 *out) {
    u64 N = (u64)1 << logN;
    for (u64 j = 0; j < N; j++) {
        u64 x = orc_powmod(psi, 2 * brev(j, logN) + 1, q);
        u64 acc = 0, xp = 1;
        for (u64 t = 0; t < N; t++) {
            acc = orc_addmod(acc, orc_mulmod(a[t] % q, xp, q), q);
            xp = orc_mulmod(xp, x, q);
        }
        out[j] = acc;
    }
}

/* a[t] = N^-1 * sum_j ahat[j] * psi^(-(2*brev(j)+1)*t) mod q      O(N^2) */
void orc_intt_direct(const u64 *ahat, int logN, u64 q, u64 psi, u64 *out) {
    u64 N = (u64)1 << logN;
    u64 ninv = orc_invmod(N % q, q), psinv = orc_invmod(psi, q);
    for (u64 t = 0; t < N; t++) {
        u64 acc = 0;
        for (u64 j = 0; j < N; j++) {
            u64 e = ((2 * brev(j, logN) + 1) * t) % (2 * N);
            acc = orc_addmod(acc, orc_mulmod(ahat[j] % q, orc_powmod(psinv, e, q), q), q);
        }
        out[t] = orc_mulmod(acc, ninv, q);
    }
}

/* c = a * b in Z_q[X]/(X^N+1), schoolbook: X^N = -1      O(N^2) */
void orc_negacyclic_schoolbook(const u64 *a, const u64 *b, int logN, u64 q, u64 *out) {
    u64 N = (u64)1 << logN;
    memset(out, 0, N * sizeof(u64));
    for (u64 i = 0; i < N; i++) {
        if (a[i] % q == 0) continue;
        for (u64 j = 0; j < N; j++) {
            u64 p = orc_mulmod(a[i] % q, b[j] % q, q);
            u64 k = i + j;
            if (k < N) out[k] = orc_addmod(out[k], p, q);
            else out[k - N] = orc_submod(out[k - N], p, q);
        }
    }
}

/* ------------------------------------------------------------------ */
/* the oracle's own O(N log N) transform                               */
/* twist by psi^t, textbook in-place radix-2 cyclic FFT (bit-reverse   */
/* the input, then butterflies of span 2, 4, ..., N giving natural     */
/* order), then read the result in bit-reversed order.                  */
/* ------------------------------------------------------------------ */
static void cyclic_fft(u64 *b, int logN, u64 q, u64 omega) {
    u64 N = (u64)1 << logN;
    for (u64 i = 0; i < N; i++) {
        u64 j = brev(i, logN);
        if (i < j) { u64 t = b[i]; b[i] = b[j]; b[j] = t; }
    }
    for (u64 len = 2; len <= N; len <<= 1) {
        u64 wlen = orc_powmod(omega, N / len, q);
        for (u64 s = 0; s < N; s += len) {
            u64 w = 1;
            for (u64 j = 0; j < len / 2; j++) {
                u64 u = b[s + j], v = orc_mulmod(b[s + j + len / 2], w, q);
                b[s + j] = orc_addmod(u, v, q);
                b[s + j + len / 2] = orc_submod(u, v, q);
                w = orc_mulmod(w, wlen, q);
            }
        }
    }
}

void orc_ntt(u64 *a, int logN, u64 q, u64 psi) {
    u64 N = (u64)1 << logN;
    u64 *b = (u64 *)malloc(N * sizeof(u64));
    u64 pw = 1;
    for (u64 t = 0; t < N; t++) { b[t] = orc_mulmod(a[t] % q, pw, q); pw = orc_mulmod(pw, psi, q); }
    cyclic_fft(b, logN, q, orc_mulmod(psi, psi, q));
    for (u64 j = 0; j < N; j++) a[j] = b[brev(j, logN)];
    free(b);
}

void orc_intt(u64 *a, int logN, u64 q, u64 psi) {
    u64 N = (u64)1 << logN;
    u64 *b = (u64 *)malloc(N * sizeof(u64));
    u64 psinv = orc_invmod(psi, q), ninv = orc_invmod(N % q, q);
    for (u64 u = 0; u < N; u++) b[u] = a[brev(u, logN)] % q;
    cyclic_fft(b, logN, q, orc_mulmod(psinv, psinv, q));
    u64 pw = 1;
    for (u64 t = 0; t < N; t++) {
        a[t] = orc_mulmod(orc_mulmod(b[t], ninv, q), pw, q);
        pw = orc_mulmod(pw, psinv, q);
    }
    free(b);
}

/* ------------------------------------------------------------------ */
/* parameter set                                                       */
/* ------------------------------------------------------------------ */
typedef struct {
    int logN, n_q, k, alpha;
    u64 N;
    u64 *mod; /* n_q + k */
    u64 *psi; /* n_q + k */
} orc_params;

orc_params *orc_params_new(int logN, int n_q, int k, int alpha, const u64 *mod, const u64 *psi) {
    orc_params *P = (orc_params *)calloc(1, sizeof(orc_params));
    P->logN = logN; P->n_q = n_q; P->k = k; P->alpha = alpha;
    P->N = (u64)1 << logN;
    P->mod = (u64 *)malloc((n_q + k) * sizeof(u64));
    P->psi = (u64 *)malloc((n_q + k) * sizeof(u64));
    memcpy(P->mod, mod, (n_q + k) * sizeof(u64));
    memcpy(P->psi, psi, (n_q + k) * sizeof(u64));
    return P;
}
void orc_params_free(orc_params *P) {
    if (!P) return;
    free(P->mod); free(P->psi); free(P);
}

void orc_ntt_limb(const orc_params *P, int t, u64 *a) { orc_ntt(a, P->logN, P->mod[t], P->psi[t]); }
void orc_intt_limb(const orc_params *P, int t, u64 *a) { orc_intt(a, P->logN, P->mod[t], P->psi[t]); }

/* index into the full basis of extended-basis position x at level l */
static int ext_index(const orc_params *P, int level, int x) { return x < level ? x : P->n_q + (x - level); }

/* small signed polynomial (coefficient form) -> evaluation form over the listed moduli */
void orc_small_to_eval(const orc_params *P, const i64 *coef, const int *idx, int n_idx, u64 *out) {
    for (int a = 0; a < n_idx; a++) {
        u64 q = P->mod[idx[a]];
        u64 *o = out + (size_t)a * P->N;
        for (u64 n = 0; n < P->N; n++) o[n] = orc_signed_mod(coef[n], q);
        orc_ntt_limb(P, idx[a], o);
    }
}

/* ------------------------------------------------------------------ */
/* host crypto (paper section 2.1 equations)                           */
/* ------------------------------------------------------------------ */

/* pk = (b, a), b = -a*s + e over q_0..q_{n_q-1}; a is given in evaluation form */
void orc_keygen_public(const orc_params *P, const i64 *s, const u64 *a_eval, const i64 *e, u64 *pk) {
    u64 N = P->N;
    u64 *sh = (u64 *)malloc(N * 8), *eh = (u64 *)malloc(N * 8);
    for (int i = 0; i < P->n_q; i++) {
        u64 q = P->mod[i];
        orc_small_to_eval(P, s, &i, 1, sh);
        orc_small_to_eval(P, e, &i, 1, eh);
        u64 *b = pk + (size_t)i * N, *a = pk + (size_t)(P->n_q + i) * N;
        for (u64 n = 0; n < N; n++) {
            u64 av = a_eval[(size_t)i * N + n] % q;
            a[n] = av;
            b[n] = orc_addmod(orc_submod(0, orc_mulmod(av, sh[n], q), q), eh[n], q);
        }
    }
    free(sh); free(eh);
}

/*
 * Switching key from s' to s, hybrid (digit) form.  For digit j and every
 * modulus t of the full basis:
 *     key[j][1][t] = a_j[t]                       (given, evaluation form)
 *     key[j][0][t] = -a_j[t]*s + e_j + [t = q_i, i in digit j] * (P mod q_i) * s'
 * with P the product of the special primes and digit j = {j*alpha, ...,
 * min(n_q,(j+1)*alpha)-1}.  s_coef and sprime_eval: s as signed coefficients,
 * s' in evaluation form over all n_q+k moduli.  a: [beta][n_q+k][N],
 * e: [beta][N] signed coefficients, key: [beta][2][n_q+k][N].
 */
void orc_keygen_switch(const orc_params *P, const i64 *s, const u64 *sprime_eval, const u64 *a, const i64 *e, u64 *key) {
    u64 N = P->N;
    int T = P->n_q + P->k;
    int beta = (P->n_q + P->alpha - 1) / P->alpha;
    u64 *sh = (u64 *)malloc(N * 8), *eh = (u64 *)malloc(N * 8);
    for (int j = 0; j < beta; j++) {
        for (int t = 0; t < T; t++) {
            u64 q = P->mod[t];
            orc_small_to_eval(P, s, &t, 1, sh);
            orc_small_to_eval(P, e + (size_t)j * N, &t, 1, eh);
            int in_digit = (t < P->n_q) && (t / P->alpha == j);
            u64 Pmod = 1;
            for (int m = 0; m < P->k; m++) Pmod = orc_mulmod(Pmod, P->mod[P->n_q + m] % q, q);
            const u64 *aj = a + ((size_t)j * T + t) * N;
            u64 *kb = key + (((size_t)j * 2 + 0) * T + t) * N;
            u64 *ka = key + (((size_t)j * 2 + 1) * T + t) * N;
            for (u64 n = 0; n < N; n++) {
                u64 av = aj[n] % q;
                u64 v = orc_addmod(orc_submod(0, orc_mulmod(av, sh[n], q), q), eh[n], q);
                if (in_digit) v = orc_addmod(v, orc_mulmod(Pmod, sprime_eval[(size_t)t * N + n] % q, q), q);
                kb[n] = v;
                ka[n] = av;
            }
        }
    }
    free(sh); free(eh);
}

/* ct = (r*b + e0 + m, r*a + e1) at `level` limbs; m: [level][N] evaluation form */
void orc_encrypt(const orc_params *P, const u64 *pk, const u64 *m, const i64 *r, const i64 *e0, const i64 *e1, int level, u64 *ct) {
    u64 N = P->N;
    u64 *rh = (u64 *)malloc(N * 8), *e0h = (u64 *)malloc(N * 8), *e1h = (u64 *)malloc(N * 8);
    for (int i = 0; i < level; i++) {
        u64 q = P->mod[i];
        orc_small_to_eval(P, r, &i, 1, rh);
        orc_small_to_eval(P, e0, &i, 1, e0h);
        orc_small_to_eval(P, e1, &i, 1, e1h);
        const u64 *b = pk + (size_t)i * N, *a = pk + (size_t)(P->n_q + i) * N;
        u64 *c0 = ct + (size_t)i * N, *c1 = ct + (size_t)(level + i) * N;
        for (u64 n = 0; n < N; n++) {
            c0[n] = orc_addmod(orc_addmod(orc_mulmod(rh[n], b[n], q), e0h[n], q), m[(size_t)i * N + n] % q, q);
            c1[n] = orc_addmod(orc_mulmod(rh[n], a[n], q), e1h[n], q);
        }
    }
    free(rh); free(e0h); free(e1h);
}

/* m' = c0 + c1*s per limb, returned in COEFFICIENT form [level][N]; works for a
 * degree-2 ciphertext too (n_comp = 3: m' = d0 + d1*s + d2*s^2) */
void orc_decrypt(const orc_params *P, const i64 *s, const u64 *ct, int level, int n_comp, u64 *m_coef) {
    u64 N = P->N;
    u64 *sh = (u64 *)malloc(N * 8);
    for (int i = 0; i < level; i++) {
        u64 q = P->mod[i];
        orc_small_to_eval(P, s, &i, 1, sh);
        u64 *o = m_coef + (size_t)i * N;
        for (u64 n = 0; n < N; n++) {
            u64 acc = 0, sp = 1;
            for (int c = 0; c < n_comp; c++) {
                acc = orc_addmod(acc, orc_mulmod(ct[((size_t)c * level + i) * N + n] % q, sp, q), q);
                sp = orc_mulmod(sp, sh[n], q);
            }
            o[n] = acc;
        }
        orc_intt_limb(P, i, o);
    }
    free(sh);
}

/* ------------------------------------------------------------------ */
/* ciphertext arithmetic                                               */
/* ------------------------------------------------------------------ */

/* ct x ct: (d0, d1, d2) = (a0*b0, a0*b1 + a1*b0, a1*b1), pointwise per limb */
void orc_tensor(const orc_params *P, const u64 *a, const u64 *b, int level, u64 *d) {
    u64 N = P->N;
    for (int i = 0; i < level; i++) {
        u64 q = P->mod[i];
        const u64 *a0 = a + (size_t)i * N, *a1 = a + (size_t)(level + i) * N;
        const u64 *b0 = b + (size_t)i * N, *b1 = b + (size_t)(level + i) * N;
        u64 *d0 = d + (size_t)i * N, *d1 = d + (size_t)(level + i) * N, *d2 = d + (size_t)(2 * level + i) * N;
        for (u64 n = 0; n < N; n++) {
            d0[n] = orc_mulmod(a0[n], b0[n], q);
            d1[n] = orc_addmod(orc_mulmod(a0[n], b1[n], q), orc_mulmod(a1[n], b0[n], q), q);
            d2[n] = orc_mulmod(a1[n], b1[n], q);
        }
    }
}

/*
 * ModUp of digit j at `level`: fast basis conversion of the limbs D = digit j
 * restricted to [0, level) onto every other modulus of the extended basis
 * (q_0..q_{level-1}, p_0..p_{k-1}).  d_coef [level][N] and out [level+k][N] are
 * in coefficient form.  With Q_D = prod_{i in D} q_i and qhat_i = Q_D / q_i:
 *     y_i    = d_i * (qhat_i^-1 mod q_i) mod q_i              in [0, q_i)
 *     out[t] = ( sum_{i in D} y_i * (qhat_i mod t) ) mod t    for t not in D
 *     out[i] = d_i                                            for i in D
 * i.e. the integer sum_i y_i*qhat_i = d + u*Q_D (0 <= u < |D|) reduced mod t;
 * no floating-point correction of u and no centring.
 */
void orc_modup(const orc_params *P, const u64 *d_coef, int level, int j, u64 *out) {
    u64 N = P->N;
    int lo = j * P->alpha, hi = lo + P->alpha;
    if (hi > level) hi = level;
    int nd = hi - lo;
    int E = level + P->k;
    u64 *y = (u64 *)malloc((size_t)nd * N * 8);
    for (int a = 0; a < nd; a++) {
        u64 qi = P->mod[lo + a];
        u64 qhat = 1;
        for (int b = 0; b < nd; b++) if (b != a) qhat = orc_mulmod(qhat, P->mod[lo + b] % qi, qi);
        u64 inv = orc_invmod(qhat, qi);
        for (u64 n = 0; n < N; n++) y[(size_t)a * N + n] = orc_mulmod(d_coef[(size_t)(lo + a) * N + n] % qi, inv, qi);
    }
    for (int x = 0; x < E; x++) {
        u64 *o = out + (size_t)x * N;
        if (x >= lo && x < hi) { memcpy(o, d_coef + (size_t)x * N, N * 8); continue; }
        u64 t = P->mod[ext_index(P, level, x)];
        for (u64 n = 0; n < N; n++) o[n] = 0;
        for (int a = 0; a < nd; a++) {
            u64 qhat_t = 1;
            for (int b = 0; b < nd; b++) if (b != a) qhat_t = orc_mulmod(qhat_t, P->mod[lo + b] % t, t);
            for (u64 n = 0; n < N; n++) o[n] = orc_addmod(o[n], orc_mulmod(y[(size_t)a * N + n] % t, qhat_t, t), t);
        }
    }
    free(y);
}

/*
 * DivRound_B, coefficient form.  x holds nc limbs over the kept moduli C
 * (indices cidx) followed by nb limbs over the dropped moduli B (indices bidx).
 * Bbar = prod B, h = floor(Bbar/2) = (Bbar-1)/2 (Bbar is odd), bhat_m = Bbar/b_m.
 *   x'_m  = (x_m + h) mod b_m
 *   y_m   = x'_m * (bhat_m^-1 mod b_m) mod b_m
 *   r_i   = ( sum_m y_m * (bhat_m mod c_i) ) mod c_i
 *   out_i = (x_i + h - r_i) * (Bbar^-1 mod c_i) mod c_i
 * As integers: out = floor((x + h)/Bbar) - u, u = 0 when |B| = 1 (exact
 * round-to-nearest), 0 <= u <= |B|-1 otherwise.  h mod t is obtained from
 * 2*h = Bbar - 1, i.e. h = (Bbar mod t - 1) * 2^-1 mod t (t odd).
 *
 * exact != 0 removes u: sum_m y_m * bhat_m = ((x + h) mod Bbar) + u*Bbar, hence
 * sum_m y_m / b_m = ((x + h) mod Bbar)/Bbar + u and u is the integer part of that
 * sum.  It is taken in double precision, v = floor(((y_0*i_0 + y_1*i_1) + y_2*i_2) + ...)
 * with i_m the double nearest to 1/b_m and every product and sum rounded to
 * nearest, and r_i loses v * (Bbar mod c_i).  v = u unless (x + h) mod Bbar lies
 * within about |B| * 2^-52 * Bbar of a multiple of Bbar; the order of the
 * floating-point operations is part of the definition.
 */
static void divround_coef(const orc_params *P, const u64 *x, const int *cidx, int nc, const int *bidx, int nb, int exact, u64 *out) {
    u64 N = P->N;
    u64 *y = (u64 *)malloc((size_t)nb * N * 8);
    u64 *v = (u64 *)calloc(N, 8);
    for (int m = 0; m < nb; m++) {
        u64 bm = P->mod[bidx[m]];
        u64 bhat = 1;
        for (int m2 = 0; m2 < nb; m2++) if (m2 != m) bhat = orc_mulmod(bhat, P->mod[bidx[m2]] % bm, bm);
        u64 inv = orc_invmod(bhat, bm);
        u64 h = (bm - 1) / 2; /* (0 - 1) * 2^-1 mod b_m */
        const u64 *xm = x + (size_t)(nc + m) * N;
        for (u64 n = 0; n < N; n++) y[(size_t)m * N + n] = orc_mulmod(orc_addmod(xm[n] % bm, h, bm), inv, bm);
    }
    if (exact)
        for (u64 n = 0; n < N; n++) {
            volatile double sum = 0.0; /* volatile: every operation rounded to double, none contracted */
            for (int m = 0; m < nb; m++) {
                volatile double inv_b = 1.0 / (double)P->mod[bidx[m]];
                volatile double term = (double)y[(size_t)m * N + n] * inv_b;
                sum = m == 0 ? term : sum + term;
            }
            v[n] = (u64)floor(sum);
        }
    for (int i = 0; i < nc; i++) {
        u64 c = P->mod[cidx[i]];
        u64 Bbar = 1;
        for (int m = 0; m < nb; m++) Bbar = orc_mulmod(Bbar, P->mod[bidx[m]] % c, c);
        u64 h = orc_mulmod(orc_submod(Bbar, 1, c), orc_invmod(2, c), c);
        u64 Binv = orc_invmod(Bbar, c);
        const u64 *xi = x + (size_t)i * N;
        u64 *o = out + (size_t)i * N;
        u64 *bhat_c = (u64 *)malloc(sizeof(u64) * nb);
        for (int m = 0; m < nb; m++) {
            bhat_c[m] = 1;
            for (int m2 = 0; m2 < nb; m2++) if (m2 != m) bhat_c[m] = orc_mulmod(bhat_c[m], P->mod[bidx[m2]] % c, c);
        }
        for (u64 n = 0; n < N; n++) {
            u64 r = 0;
            for (int m = 0; m < nb; m++) r = orc_addmod(r, orc_mulmod(y[(size_t)m * N + n] % c, bhat_c[m], c), c);
            r = orc_submod(r, orc_mulmod(v[n] % c, Bbar, c), c);
            o[n] = orc_mulmod(orc_submod(orc_addmod(xi[n] % c, h, c), r, c), Binv, c);
        }
        free(bhat_c);
    }
    free(y); free(v);
}

void orc_divround_coef(const orc_params *P, const u64 *x, const int *cidx, int nc, const int *bidx, int nb, u64 *out) {
    divround_coef(P, x, cidx, nc, bidx, nb, 0, out);
}

void orc_divround_exact_coef(const orc_params *P, const u64 *x, const int *cidx, int nc, const int *bidx, int nb, u64 *out) {
    divround_coef(P, x, cidx, nc, bidx, nb, 1, out);
}

/*
 * Inner-product stage of the key switch of one polynomial d (evaluation form,
 * [level][N]) with a switching key [beta][2][n_q+k][N]: inverse transform, ModUp
 * each digit, transform, multiply-accumulate with the key over the extended
 * basis.  acc: [2][level+k][N], evaluation form, zeroed here.
 */
static void ks_accumulate(const orc_params *P, const u64 *d_eval, const u64 *key, int level, u64 *acc) {
    u64 N = P->N;
    int E = level + P->k, T = P->n_q + P->k;
    int beta = (level + P->alpha - 1) / P->alpha;
    u64 *dc = (u64 *)malloc((size_t)level * N * 8);
    u64 *dt = (u64 *)malloc((size_t)E * N * 8);
    memset(acc, 0, (size_t)2 * E * N * 8);
    memcpy(dc, d_eval, (size_t)level * N * 8);
    for (int i = 0; i < level; i++) orc_intt_limb(P, i, dc + (size_t)i * N);
    for (int j = 0; j < beta; j++) {
        orc_modup(P, dc, level, j, dt);
        for (int x = 0; x < E; x++) {
            int t = ext_index(P, level, x);
            u64 q = P->mod[t];
            u64 *v = dt + (size_t)x * N;
            orc_ntt_limb(P, t, v);
            for (int c = 0; c < 2; c++) {
                const u64 *kk = key + (((size_t)j * 2 + c) * T + t) * N;
                u64 *ac = acc + ((size_t)c * E + x) * N;
                for (u64 n = 0; n < N; n++) ac[n] = orc_addmod(ac[n], orc_mulmod(v[n], kk[n] % q, q), q);
            }
        }
    }
    free(dc); free(dt);
}

/*
 * Key switch: the inner-product stage above, then DivRound_P of both
 * accumulators.  ks: [2][level][N] evaluation form.
 */
void orc_keyswitch(const orc_params *P, const u64 *d_eval, const u64 *key, int level, u64 *ks) {
    u64 N = P->N;
    int E = level + P->k;
    u64 *acc = (u64 *)malloc((size_t)2 * E * N * 8);
    ks_accumulate(P, d_eval, key, level, acc);
    int *cidx = (int *)malloc(sizeof(int) * level), *bidx = (int *)malloc(sizeof(int) * (P->k ? P->k : 1));
    for (int i = 0; i < level; i++) cidx[i] = i;
    for (int m = 0; m < P->k; m++) bidx[m] = P->n_q + m;
    for (int c = 0; c < 2; c++) {
        u64 *ac = acc + (size_t)c * E * N;
        for (int x = 0; x < E; x++) orc_intt_limb(P, ext_index(P, level, x), ac + (size_t)x * N);
        u64 *o = ks + (size_t)c * level * N;
        orc_divround_coef(P, ac, cidx, level, bidx, P->k, o);
        for (int i = 0; i < level; i++) orc_ntt_limb(P, i, o + (size_t)i * N);
    }
    free(cidx); free(bidx); free(acc);
}

/* relinearise: (d0 + ks0, d1 + ks1), ks = KeySwitch(d2) with the key for s' = s^2 */
void orc_relin(const orc_params *P, const u64 *d, const u64 *rlk, int level, u64 *out) {
    u64 N = P->N;
    orc_keyswitch(P, d + (size_t)2 * level * N, rlk, level, out);
    for (int c = 0; c < 2; c++)
        for (int i = 0; i < level; i++) {
            u64 q = P->mod[i];
            u64 *o = out + ((size_t)c * level + i) * N;
            const u64 *dd = d + ((size_t)c * level + i) * N;
            for (u64 n = 0; n < N; n++) o[n] = orc_addmod(o[n], dd[n] % q, q);
        }
}

/* rescale: DivRound by the last modulus q_{level-1} on both components */
void orc_rescale(const orc_params *P, const u64 *ct, int level, u64 *out) {
    u64 N = P->N;
    int *cidx = (int *)malloc(sizeof(int) * level);
    for (int i = 0; i < level; i++) cidx[i] = i;
    int b = level - 1;
    u64 *tmp = (u64 *)malloc((size_t)level * N * 8);
    for (int c = 0; c < 2; c++) {
        memcpy(tmp, ct + (size_t)c * level * N, (size_t)level * N * 8);
        for (int i = 0; i < level; i++) orc_intt_limb(P, i, tmp + (size_t)i * N);
        u64 *o = out + (size_t)c * (level - 1) * N;
        orc_divround_coef(P, tmp, cidx, level - 1, &b, 1, o);
        for (int i = 0; i < level - 1; i++) orc_ntt_limb(P, i, o + (size_t)i * N);
    }
    free(cidx); free(tmp);
}

/* the strict sequence tensor -> key switch -> add -> rescale */
void orc_hmul_relin_rescale(const orc_params *P, const u64 *a, const u64 *b, const u64 *rlk, int level, u64 *out) {
    u64 N = P->N;
    u64 *d = (u64 *)malloc((size_t)3 * level * N * 8);
    u64 *r = (u64 *)malloc((size_t)2 * level * N * 8);
    orc_tensor(P, a, b, level, d);
    orc_relin(P, d, rlk, level, r);
    orc_rescale(P, r, level, out);
    free(d); free(r);
}

/*
 * Lazy relinearisation: the sum of `terms` products is relinearised and rescaled
 * ONCE, out = Rescale(Relin(sum_t Tensor(a_t, b_t))), the three-component tensors
 * added limb-wise mod q_i.  a, b: [terms][2][level][N]; out: [2][level-1][N].
 * Not the bits of summing separately relinearised products (one key-switch and one
 * rounding error instead of `terms` of each); with terms = 1 it is
 * orc_hmul_relin_rescale.
 */
void orc_hmul_sum_relin_rescale(const orc_params *P, const u64 *a, const u64 *b, int terms, const u64 *rlk, int level, u64 *out) {
    u64 N = P->N;
    size_t ct_words = (size_t)2 * level * N;
    u64 *d = (u64 *)calloc((size_t)3 * level * N, 8);
    u64 *dt = (u64 *)malloc((size_t)3 * level * N * 8);
    u64 *r = (u64 *)malloc((size_t)2 * level * N * 8);
    for (int t = 0; t < terms; t++) {
        orc_tensor(P, a + (size_t)t * ct_words, b + (size_t)t * ct_words, level, dt);
        for (int c = 0; c < 3; c++)
            for (int i = 0; i < level; i++) {
                u64 q = P->mod[i];
                size_t o = ((size_t)c * level + i) * N;
                for (u64 n = 0; n < N; n++) d[o + n] = orc_addmod(d[o + n], dt[o + n], q);
            }
    }
    orc_relin(P, d, rlk, level, r);
    orc_rescale(P, r, level, out);
    free(d); free(dt); free(r);
}

/*
 * The same product with ONE division: the key-switch accumulators stay over the
 * extended basis, P*(d0, d1) is added there (zero on the special limbs), and both
 * components are divided by P*q_{level-1} in a single DivRound over
 * B = {q_{level-1}, p_0 .. p_{k-1}}:
 *     out_c = DivRound_B(acc_c + P*d_c),   c = 0, 1,
 * with the exact form of DivRound: the conversion's overshoot u would otherwise
 * sit at the scale of the output (in the strict sequence the rescale divides it
 * by q_{level-1}) and, being one-sided, would add up over the coefficients.
 * The integer divided is the one the strict sequence divides in two steps, so the
 * two results differ only by the rounding of those steps (one unit per
 * coefficient); the output bits are NOT those of orc_hmul_relin_rescale.
 * out: [2][level-1][N] evaluation form.
 */
void orc_hmul_relin_rescale_merged(const orc_params *P, const u64 *a, const u64 *b, const u64 *rlk, int level, u64 *out) {
    u64 N = P->N;
    int E = level + P->k, nb = P->k + 1;
    u64 *d = (u64 *)malloc((size_t)3 * level * N * 8);
    u64 *acc = (u64 *)malloc((size_t)2 * E * N * 8);
    orc_tensor(P, a, b, level, d);
    ks_accumulate(P, d + (size_t)2 * level * N, rlk, level, acc);
    int *cidx = (int *)malloc(sizeof(int) * level), *bidx = (int *)malloc(sizeof(int) * nb);
    for (int i = 0; i < level - 1; i++) cidx[i] = i;
    bidx[0] = level - 1;
    for (int m = 0; m < P->k; m++) bidx[1 + m] = P->n_q + m;
    for (int c = 0; c < 2; c++) {
        u64 *ac = acc + (size_t)c * E * N;
        for (int i = 0; i < level; i++) {
            u64 q = P->mod[i];
            u64 Pq = 1;
            for (int m = 0; m < P->k; m++) Pq = orc_mulmod(Pq, P->mod[P->n_q + m] % q, q);
            const u64 *dd = d + ((size_t)c * level + i) * N;
            u64 *x = ac + (size_t)i * N;
            for (u64 n = 0; n < N; n++) x[n] = orc_addmod(x[n], orc_mulmod(dd[n] % q, Pq, q), q);
        }
        /* extended layout [q_0 .. q_{level-1}, p_0 .. p_{k-1}] = kept limbs followed by the limbs of B */
        for (int x = 0; x < E; x++) orc_intt_limb(P, ext_index(P, level, x), ac + (size_t)x * N);
        u64 *o = out + (size_t)c * (level - 1) * N;
        orc_divround_exact_coef(P, ac, cidx, level - 1, bidx, nb, o);
        for (int i = 0; i < level - 1; i++) orc_ntt_limb(P, i, o + (size_t)i * N);
    }
    free(cidx); free(bidx); free(d); free(acc);
}

/* automorphism X -> X^g on signed coefficients (used for sigma_g(s)) */
void orc_automorphism_small(const i64 *a, int logN, u64 g, i64 *out) {
    u64 N = (u64)1 << logN;
    for (u64 t = 0; t < N; t++) {
        u64 idx = (t * g) % (2 * N);
        if (idx < N) out[idx] = a[t]; else out[idx - N] = -a[t];
    }
}

/* automorphism X -> X^g on one limb in coefficient form: coefficient t moves to
 * index t*g mod 2N, negated when that index is >= N */
void orc_automorphism_coef(const u64 *a, int logN, u64 g, u64 q, u64 *out) {
    u64 N = (u64)1 << logN;
    for (u64 t = 0; t < N; t++) {
        u64 idx = (t * g) % (2 * N);
        if (idx < N) out[idx] = a[t] % q; else out[idx - N] = orc_submod(0, a[t] % q, q);
    }
}

/* the same automorphism in evaluation form: out[j] = in[pi(j)],
 * pi(j) = brev(((2*brev(j)+1)*g mod 2N - 1)/2) */
void orc_automorphism_eval(const u64 *a, int logN, u64 g, u64 *out) {
    u64 N = (u64)1 << logN;
    for (u64 j = 0; j < N; j++) {
        u64 e = ((2 * brev(j, logN) + 1) * g) % (2 * N);
        out[j] = a[brev((e - 1) / 2, logN)];
    }
}

/* g = 5^r mod 2N */
u64 orc_galois_element(int logN, i64 r) {
    u64 N = (u64)1 << logN, half = N / 2;
    u64 rr = (u64)(((r % (i64)half) + (i64)half) % (i64)half);
    return orc_powmod(5, rr, 2 * N);
}

/*
 * Rotation with Galois element g: automorphism first (by its coefficient-form
 * definition), then key switch of the second component with the key whose
 * s' = sigma_g(s):  out = (sigma_g(c0) + ks0, ks1).
 */
void orc_rotate(const orc_params *P, const u64 *ct, u64 g, const u64 *gk, int level, u64 *out) {
    u64 N = P->N;
    u64 *sg = (u64 *)malloc((size_t)2 * level * N * 8);
    u64 *tmp = (u64 *)malloc(N * 8);
    for (int c = 0; c < 2; c++)
        for (int i = 0; i < level; i++) {
            u64 *o = sg + ((size_t)c * level + i) * N;
            memcpy(tmp, ct + ((size_t)c * level + i) * N, N * 8);
            orc_intt_limb(P, i, tmp);
            orc_automorphism_coef(tmp, P->logN, g, P->mod[i], o);
            orc_ntt_limb(P, i, o);
        }
    orc_keyswitch(P, sg + (size_t)level * N, gk, level, out);
    for (int i = 0; i < level; i++) {
        u64 q = P->mod[i];
        u64 *o = out + (size_t)i * N;
        const u64 *a = sg + (size_t)i * N;
        for (u64 n = 0; n < N; n++) o[n] = orc_addmod(o[n], a[n], q);
    }
    free(sg); free(tmp);
}

/*
 * R rotations of ONE ciphertext with a shared ModUp ("hoisting"): the second
 * component is decomposed and lifted once,
 *     dt_j = NTT(ModUp_j(INTT(c1))),  j < beta,   over the extended basis,
 * and every rotation applies its automorphism to those lifted digits (limb-wise,
 * evaluation form) before the inner product with its own key:
 *     acc_c = sum_j sigma_g(dt_j) * gk_g[j][c],   ks = DivRound_P(acc),
 *     out_g = (sigma_g(c0) + ks0, ks1).
 * sigma_g(ModUp_j(d)) = sigma_g(d) + sigma_g(u)*Q_j is as good a lift of
 * sigma_g(d) as ModUp_j(sigma_g(d)) but not the same one, so out_g decrypts like
 * orc_rotate's result and is NOT bit-identical to it.
 * g: R Galois elements; gk: R keys [beta][2][n_q+k][N] back to back;
 * out: [R][2][level][N].
 */
void orc_rotate_hoisted(const orc_params *P, const u64 *ct, int level, int R, const u64 *g, const u64 *gk, u64 *out) {
    u64 N = P->N;
    int E = level + P->k, T = P->n_q + P->k;
    int beta = (level + P->alpha - 1) / P->alpha;
    size_t key_words = (size_t)((P->n_q + P->alpha - 1) / P->alpha) * 2 * T * N; /* digits are fixed at the top level */
    u64 *dc = (u64 *)malloc((size_t)level * N * 8);
    u64 *dt = (u64 *)malloc((size_t)beta * E * N * 8);
    u64 *acc = (u64 *)malloc((size_t)2 * E * N * 8);
    u64 *v = (u64 *)malloc(N * 8);
    int *cidx = (int *)malloc(sizeof(int) * level), *bidx = (int *)malloc(sizeof(int) * (P->k ? P->k : 1));
    for (int i = 0; i < level; i++) cidx[i] = i;
    for (int m = 0; m < P->k; m++) bidx[m] = P->n_q + m;
    memcpy(dc, ct + (size_t)level * N, (size_t)level * N * 8);
    for (int i = 0; i < level; i++) orc_intt_limb(P, i, dc + (size_t)i * N);
    for (int j = 0; j < beta; j++) {
        u64 *dj = dt + (size_t)j * E * N;
        orc_modup(P, dc, level, j, dj);
        for (int x = 0; x < E; x++) orc_ntt_limb(P, ext_index(P, level, x), dj + (size_t)x * N);
    }
    for (int r = 0; r < R; r++) {
        const u64 *key = gk + (size_t)r * key_words;
        u64 *o = out + (size_t)r * 2 * level * N;
        memset(acc, 0, (size_t)2 * E * N * 8);
        for (int j = 0; j < beta; j++)
            for (int x = 0; x < E; x++) {
                int t = ext_index(P, level, x);
                u64 q = P->mod[t];
                orc_automorphism_eval(dt + ((size_t)j * E + x) * N, P->logN, g[r], v);
                for (int c = 0; c < 2; c++) {
                    const u64 *kk = key + (((size_t)j * 2 + c) * T + t) * N;
                    u64 *ac = acc + ((size_t)c * E + x) * N;
                    for (u64 n = 0; n < N; n++) ac[n] = orc_addmod(ac[n], orc_mulmod(v[n] % q, kk[n] % q, q), q);
                }
            }
        for (int c = 0; c < 2; c++) {
            u64 *ac = acc + (size_t)c * E * N;
            for (int x = 0; x < E; x++) orc_intt_limb(P, ext_index(P, level, x), ac + (size_t)x * N);
            orc_divround_coef(P, ac, cidx, level, bidx, P->k, o + (size_t)c * level * N);
            for (int i = 0; i < level; i++) orc_ntt_limb(P, i, o + ((size_t)c * level + i) * N);
        }
        for (int i = 0; i < level; i++) {
            u64 q = P->mod[i];
            orc_automorphism_eval(ct + (size_t)i * N, P->logN, g[r], v);
            for (u64 n = 0; n < N; n++) o[(size_t)i * N + n] = orc_addmod(o[(size_t)i * N + n], v[n] % q, q);
        }
    }
    free(cidx); free(bidx); free(dc); free(dt); free(acc); free(v);
}

/* ---- sampling (the distributions of section 2.1's key generation and encryption; the paper names none) ----
 * Counter-based, so that any coefficient can be drawn anywhere: Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel
 * random numbers: as easy as 1, 2, 3", 2011).  One round: with the 32x32->64 products p0 = M0*c0, p1 = M1*c2,
 * (c0, c1, c2, c3) <- (hi(p1) ^ c1 ^ k0, lo(p1), hi(p0) ^ c3 ^ k1, lo(p0)); the key advances by (W0, W1) between
 * rounds; ten rounds. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; r++) {
        if (r) { k0 += W0; k1 += W1; }
        uint64_t p0 = M0 * c0, p1 = M1 * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1, n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* thresholds of the rounded Gaussian's magnitude: T_k = floor(2^64 * P(|X| <= k)), P(|X| <= k) = erf((k + 1/2)/(sigma*sqrt 2)),
 * taken from the complementary function so that the tail keeps its relative accuracy */
#define ORC_GAUSS_K 40
static void gauss_thresholds(double sigma, u64 T[ORC_GAUSS_K]) {
    for (int k = 0; k < ORC_GAUSS_K; k++) {
        long double tail = erfcl(((long double)k + 0.5L) / ((long double)sigma * sqrtl(2.0L))) * 18446744073709551616.0L; /* 2^64 */
        T[k] = tail >= 1.0L ? (u64)0 - (u64)ceill(tail) : ~(u64)0;
    }
}

/*
 * rows polynomials of N coefficients.  Coefficient t of polynomial p = first_index + row uses the Philox block with
 * counter (t, kind, lo32(p), hi32(p)) and key (lo32(seed), hi32(seed)); its words w0..w3 give
 *   kind 0, ternary : ((w0 * 3) >> 32) - 1                    in {-1, 0, 1}
 *   kind 1, Gaussian: magnitude = #{k : u >= T_k}, u = w1*2^32 + w0, negative when w2 is odd   (round(N(0, sigma^2)))
 */
void orc_sample(int kind, double sigma, u64 seed, u64 first_index, int rows, int logN, i64 *out) {
    u64 N = (u64)1 << logN;
    u64 T[ORC_GAUSS_K];
    if (kind == 1) gauss_thresholds(sigma, T);
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (int row = 0; row < rows; row++) {
        u64 p = first_index + (u64)row;
        for (u64 t = 0; t < N; t++) {
            uint32_t ctr[4] = {(uint32_t)t, (uint32_t)kind, (uint32_t)p, (uint32_t)(p >> 32)}, w[4];
            orc_philox4x32_10(ctr, key, w);
            i64 v;
            if (kind == 0) {
                v = (i64)(((u64)w[0] * 3) >> 32) - 1;
            } else {
                u64 u = ((u64)w[1] << 32) | w[0];
                int mag = 0;
                for (int k = 0; k < ORC_GAUSS_K; k++) mag += (u >= T[k]);
                v = (w[2] & 1u) ? -(i64)mag : (i64)mag;
            }
            out[(size_t)row * N + t] = v;
        }
    }
}

void orc_gauss_thresholds(double sigma, u64 *T) { gauss_thresholds(sigma, T); }

/* ---- limb-wise operations ---- */
void orc_add(const orc_params *P, const u64 *a, const u64 *b, int level, u64 *out) {
    for (int c = 0; c < 2; c++) for (int i = 0; i < level; i++) {
        u64 q = P->mod[i]; size_t o = ((size_t)c * level + i) * P->N;
        for (u64 n = 0; n < P->N; n++) out[o + n] = orc_addmod(a[o + n] % q, b[o + n] % q, q);
    }
}
void orc_sub(const orc_params *P, const u64 *a, const u64 *b, int level, u64 *out) {
    for (int c = 0; c < 2; c++) for (int i = 0; i < level; i++) {
        u64 q = P->mod[i]; size_t o = ((size_t)c * level + i) * P->N;
        for (u64 n = 0; n < P->N; n++) out[o + n] = orc_submod(a[o + n] % q, b[o + n] % q, q);
    }
}
/* pointwise product of both components with a plaintext [level][N] in evaluation form */
void orc_mul_plain(const orc_params *P, const u64 *a, const u64 *pt, int level, u64 *out) {
    for (int c = 0; c < 2; c++) for (int i = 0; i < level; i++) {
        u64 q = P->mod[i]; size_t o = ((size_t)c * level + i) * P->N;
        for (u64 n = 0; n < P->N; n++) out[o + n] = orc_mulmod(a[o + n] % q, pt[(size_t)i * P->N + n] % q, q);
    }
}
/* multiply every word of both components by the signed integer c */
void orc_mul_scalar(const orc_params *P, const u64 *a, i64 cst, int level, u64 *out) {
    for (int c = 0; c < 2; c++) for (int i = 0; i < level; i++) {
        u64 q = P->mod[i]; size_t o = ((size_t)c * level + i) * P->N;
        u64 w = orc_signed_mod(cst, q);
        for (u64 n = 0; n < P->N; n++) out[o + n] = orc_mulmod(a[o + n] % q, w, q);
    }
}
/* add the constant polynomial c (every slot += c/scale): in evaluation form a
 * constant polynomial is the same constant in every word of component 0 */
void orc_add_const(const orc_params *P, const u64 *a, i64 cst, int level, u64 *out) {
    for (int c = 0; c < 2; c++) for (int i = 0; i < level; i++) {
        u64 q = P->mod[i]; size_t o = ((size_t)c * level + i) * P->N;
        u64 w = c == 0 ? orc_signed_mod(cst, q) : 0;
        for (u64 n = 0; n < P->N; n++) out[o + n] = orc_addmod(a[o + n] % q, w, q);
    }
}

/*
 * conv layer over per-pixel ciphertexts (slots-as-batch packing, plaintext
 * integer weights):  out[o,y,x] = sum_{c,u,v} W[o,c,u,v] * in[c, y*stride+u-pad,
 * x*stride+v-pad] as ciphertext-word arithmetic mod q_i, taps outside the image
 * skipped.  in: [C][H][W] ciphertexts, out: [O][Ho][Wo] ciphertexts, each
 * [2][level][N].  The layer types are those of the paper's Table 1 network
 * (convolution, fully connected); FC is the 1x1 case over a flat feature list.
 */
void orc_conv2d_mac(const orc_params *P, const u64 *in, const i64 *w, int C, int H, int W, int O, int kh, int kw,
                    int stride, int pad, int level, u64 *out) {
    u64 N = P->N;
    size_t ctw = (size_t)2 * level * N;
    int Ho = (H + 2 * pad - kh) / stride + 1, Wo = (W + 2 * pad - kw) / stride + 1;
    for (int o = 0; o < O; o++) for (int y = 0; y < Ho; y++) for (int x = 0; x < Wo; x++) {
        u64 *dst = out + (((size_t)o * Ho + y) * Wo + x) * ctw;
        memset(dst, 0, ctw * 8);
        for (int c = 0; c < C; c++) for (int u = 0; u < kh; u++) for (int v = 0; v < kw; v++) {
            int iy = y * stride + u - pad, ix = x * stride + v - pad;
            if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
            i64 wt = w[(((size_t)o * C + c) * kh + u) * kw + v];
            const u64 *src = in + (((size_t)c * H + iy) * W + ix) * ctw;
            for (int comp = 0; comp < 2; comp++) for (int i = 0; i < level; i++) {
                u64 q = P->mod[i];
                u64 wm = orc_signed_mod(wt, q);
                size_t off = ((size_t)comp * level + i) * N;
                for (u64 n = 0; n < N; n++) dst[off + n] = orc_addmod(dst[off + n], orc_mulmod(src[off + n] % q, wm, q), q);
            }
        }
    }
}
void orc_fc_mac(const orc_params *P, const u64 *in, const i64 *w, int F, int O, int level, u64 *out) {
    orc_conv2d_mac(P, in, w, F, 1, 1, O, 1, 1, 1, 0, level, out);
}

/*
 * k x k pooling of per-pixel ciphertexts (the zero-padding and average-pooling
 * rows of the paper's Table 1) as a plain sum of ciphertexts over windows of
 * the image padded with `pad` rows / columns of zeros on every side:
 * out[c,y,x] = sum_{u,v<k} in[c, k*y+u-pad, k*x+v-pad], positions outside the
 * image contribute nothing; the 1/k^2 of the average is a plaintext constant
 * that the caller folds into the next layer's weights.  in: [C][H][W]
 * ciphertexts, out: [C][(H+2*pad)/k][(W+2*pad)/k] (rows/columns beyond the last
 * full window are ignored).
 */
void orc_sum_pool2d(const orc_params *P, const u64 *in, int C, int H, int W, int k, int pad, int level, u64 *out) {
    u64 N = P->N;
    size_t ctw = (size_t)2 * level * N;
    int Ho = (H + 2 * pad) / k, Wo = (W + 2 * pad) / k;
    for (int c = 0; c < C; c++) for (int y = 0; y < Ho; y++) for (int x = 0; x < Wo; x++) {
        u64 *dst = out + (((size_t)c * Ho + y) * Wo + x) * ctw;
        memset(dst, 0, ctw * 8);
        for (int u = 0; u < k; u++) for (int v = 0; v < k; v++) {
            int iy = k * y + u - pad, ix = k * x + v - pad;
            if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
            const u64 *src = in + (((size_t)c * H + iy) * W + ix) * ctw;
            for (int comp = 0; comp < 2; comp++) for (int i = 0; i < level; i++) {
                u64 q = P->mod[i];
                size_t off = ((size_t)comp * level + i) * N;
                for (u64 n = 0; n < N; n++) dst[off + n] = orc_addmod(dst[off + n], src[off + n] % q, q);
            }
        }
    }
}

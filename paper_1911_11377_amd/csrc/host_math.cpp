// Host-side number theory and constant tables for the GPU library: prime and root
// search, the library's own integer transform (used by encode/decode/keygen on the
// host), and the floating-point multiplicand tables the kernels consume.
#include "ckksmi_internal.h"

namespace hm {

u64 powmod(u64 a, u64 e, u64 q) {
    u64 r = 1 % q;
    a %= q;
    for (; e; e >>= 1) {
        if (e & 1) r = mulmod(r, a, q);
        a = mulmod(a, a, q);
    }
    return r;
}

u64 invmod(u64 a, u64 q) { return powmod(a, q - 2, q); }

u64 signed_mod(i64 v, u64 q) {
    if (v >= 0) return (u64)v % q;
    u64 mag = (u64)0 - (u64)v;  // two's complement magnitude, fine at INT64_MIN
    u64 r = mag % q;
    return r ? q - r : 0;
}

// Miller-Rabin, deterministic below 2^64 with the first twelve primes as bases.
bool is_prime(u64 n) {
    static const u64 small[12] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    if (n < 2) return false;
    for (u64 p : small) {
        if (n == p) return true;
        if (n % p == 0) return false;
    }
    int r = __builtin_ctzll(n - 1);
    u64 d = (n - 1) >> r;
    for (u64 a : small) {
        u64 x = powmod(a, d, n);
        if (x == 1 || x == n - 1) continue;
        bool witness = true;
        for (int i = 1; i < r && witness; i++) {
            x = mulmod(x, x, n);
            if (x == n - 1) witness = false;
        }
        if (witness) return false;
    }
    return true;
}

// Largest `count` primes below 2^bits congruent to 1 mod 2N, descending, skipping `taken`.
bool find_primes(int bits, int logN, int count, const std::vector<u64> &taken, std::vector<u64> &out) {
    const u64 step = (u64)2 << logN, hi = (u64)1 << bits, lo = (u64)1 << (bits - 1);
    if (step >= hi) return count == 0;
    for (u64 c = hi - step + 1; (int)out.size() < count && c > lo; c -= step) {
        if (!is_prime(c)) continue;
        bool dup = false;
        for (u64 t : taken) dup |= (t == c);
        if (!dup) out.push_back(c);
        if (c < step) break;
    }
    return (int)out.size() == count;
}

u64 find_psi(u64 q, int logN) {
    const u64 N = (u64)1 << logN;
    for (u64 x = 2; x < q; x++) {
        u64 cand = powmod(x, (q - 1) / (2 * N), q);
        if (powmod(cand, N, q) == q - 1) return cand;
    }
    return 0;
}

}  // namespace hm

WMul make_wmul(u64 w, u64 p) {
    // balanced representative; both conversions are exact (|w| < 2^51), the division
    // is the correctly rounded IEEE quotient
    double wb = (w > p / 2) ? -(double)(p - w) : (double)w;
    return WMul{wb, wb / (double)p};
}

void build_host_tables(ckksmi_ctx *c) {
    const int L = c->logN;
    const u64 N = c->N;
    c->h_fwd.assign(c->T, std::vector<u64>(N));
    c->h_inv.assign(c->T, std::vector<u64>(N));
    c->h_ninv.resize(c->T);
    for (int t = 0; t < c->T; t++) {
        const u64 q = c->mod[t], psi = c->psi[t], psi_inv = hm::invmod(psi, q);
        std::vector<u64> pw(N), pwi(N);
        pw[0] = pwi[0] = 1;
        for (u64 e = 1; e < N; e++) {
            pw[e] = hm::mulmod(pw[e - 1], psi, q);
            pwi[e] = hm::mulmod(pwi[e - 1], psi_inv, q);
        }
        for (u64 x = 0; x < N; x++) {
            u64 e = hm::brev(x, L);
            c->h_fwd[t][x] = pw[e];
            c->h_inv[t][x] = pwi[e];
        }
        c->h_ninv[t] = hm::invmod(N % q, q);
        c->h_modc[t] = ModConst{(double)q, 1.0 / (double)q};
    }
}

// In-place decimation-in-time transform with the twist merged into the twiddles:
// natural order in, evaluation (bit-reversed exponent) order out.
void host_ntt(const ckksmi_ctx *c, int t, u64 *a) {
    const u64 q = c->mod[t], N = c->N;
    const u64 *tw = c->h_fwd[t].data();
    u64 span = N;
    for (u64 m = 1; m < N; m <<= 1) {
        span >>= 1;
        for (u64 i = 0; i < m; i++) {
            const u64 w = tw[m + i], base = 2 * i * span;
            for (u64 j = base; j < base + span; j++) {
                u64 u = a[j], v = hm::mulmod(a[j + span], w, q);
                a[j] = hm::addmod(u, v, q);
                a[j + span] = hm::submod(u, v, q);
            }
        }
    }
}

void host_intt(const ckksmi_ctx *c, int t, u64 *a) {
    const u64 q = c->mod[t], N = c->N;
    const u64 *tw = c->h_inv[t].data();
    u64 span = 1;
    for (u64 m = N >> 1; m >= 1; m >>= 1) {
        for (u64 i = 0; i < m; i++) {
            const u64 w = tw[m + i], base = 2 * i * span;
            for (u64 j = base; j < base + span; j++) {
                u64 u = a[j], v = a[j + span];
                a[j] = hm::addmod(u, v, q);
                a[j + span] = hm::mulmod(hm::submod(u, v, q), w, q);
            }
        }
        span <<= 1;
    }
    const u64 ninv = c->h_ninv[t];
    for (u64 j = 0; j < N; j++) a[j] = hm::mulmod(a[j], ninv, q);
}

// Constants of DivRound over the dropped moduli `bidx`: with Bbar their product,
// h = (Bbar-1)/2 and bhat_m = Bbar/b_m.  h mod t follows from 2h = Bbar - 1.
DivRoundHost make_divround(const ckksmi_ctx *c, const std::vector<int> &bidx) {
    DivRoundHost d;
    d.nb = (int)bidx.size();
    const int T = c->T;
    d.hb.resize(d.nb);
    d.invb.resize(d.nb);
    d.conv.assign((size_t)d.nb * T, WMul{0, 0});
    d.hc.assign(T, 0.0);
    d.Binv.assign(T, WMul{0, 0});
    d.Bmod.assign(T, 0.0);
    for (int m = 0; m < d.nb; m++) {
        d.b_idx[m] = bidx[m];
        const u64 bm = c->mod[bidx[m]];
        u64 bhat = 1;
        for (int m2 = 0; m2 < d.nb; m2++)
            if (m2 != m) bhat = hm::mulmod(bhat, c->mod[bidx[m2]] % bm, bm);
        d.hb[m] = (double)((bm - 1) / 2);
        d.invb[m] = make_wmul(hm::invmod(bhat, bm), bm);
    }
    for (int t = 0; t < T; t++) {
        bool dropped = false;
        for (int m = 0; m < d.nb; m++) dropped |= (bidx[m] == t);
        if (dropped) continue;
        const u64 q = c->mod[t];
        u64 B = 1;
        for (int m = 0; m < d.nb; m++) B = hm::mulmod(B, c->mod[bidx[m]] % q, q);
        d.hc[t] = (double)hm::mulmod(hm::submod(B, 1, q), hm::invmod(2, q), q);
        d.Binv[t] = make_wmul(hm::invmod(B, q), q);
        d.Bmod[t] = (double)B;
        for (int m = 0; m < d.nb; m++) {
            u64 bhat = 1;
            for (int m2 = 0; m2 < d.nb; m2++)
                if (m2 != m) bhat = hm::mulmod(bhat, c->mod[bidx[m2]] % q, q);
            d.conv[(size_t)m * T + t] = make_wmul(bhat, q);
        }
    }
    return d;
}

// ModUp constants.  Digit j holds q_{j*alpha} .. ; at a lower level only its first
// nd limbs exist, so the constants are tabulated per (j, nd).
//   inv[(j*alpha + nd-1)*alpha + a]        = (prod_{b != a} q_{lo+b})^-1 mod q_{lo+a}
//   cc [((j*alpha + nd-1)*alpha + a)*T + t] = (prod_{b != a} q_{lo+b}) mod modulus t
void make_modup_tables(const ckksmi_ctx *c, std::vector<WMul> &inv, std::vector<WMul> &cc) {
    const int A = c->alpha, T = c->T;
    inv.assign((size_t)c->beta_top * A * A, WMul{0, 0});
    cc.assign((size_t)c->beta_top * A * A * T, WMul{0, 0});
    for (int j = 0; j < c->beta_top; j++) {
        const int lo = j * A;
        for (int nd = 1; nd <= A && lo + nd <= c->n_q; nd++) {
            for (int a = 0; a < nd; a++) {
                const size_t row = ((size_t)j * A + (nd - 1)) * A + a;
                const u64 qa = c->mod[lo + a];
                u64 hat = 1;
                for (int b = 0; b < nd; b++)
                    if (b != a) hat = hm::mulmod(hat, c->mod[lo + b] % qa, qa);
                inv[row] = make_wmul(hm::invmod(hat, qa), qa);
                for (int t = 0; t < T; t++) {
                    const u64 qt = c->mod[t];
                    u64 h2 = 1;
                    for (int b = 0; b < nd; b++)
                        if (b != a) h2 = hm::mulmod(h2, c->mod[lo + b] % qt, qt);
                    cc[row * T + t] = make_wmul(h2, qt);
                }
            }
        }
    }
}

// Host side of the C ABI: context life cycle, samplers, the CKKS encoding map and
// the public-key equations of the paper's section 2.1 (keygen, encrypt, decrypt).
#include <cmath>
#include <complex>
#include <cstdlib>
#include <cstring>
#include <new>

#include "ckksmi_internal.h"

typedef long double ld;
typedef std::complex<ld> cld;

static bool level_ok(const ckksmi_ctx *c, int level) { return level >= 1 && level <= c->n_q; }

extern "C" const char *ckksmi_strerror(int code) {
    switch (code) {
        case CKKSMI_OK: return "ok";
        case CKKSMI_EINVAL: return "invalid argument";
        case CKKSMI_ELEVEL: return "level out of range for this operation";
        case CKKSMI_ENOKEY: return "no Galois key registered for that rotation";
        case CKKSMI_EWORKSPACE: return "workspace too small";
        case CKKSMI_EDEVICE: return "device error or host-only context";
        case CKKSMI_EUNSUPPORTED: return "unsupported";
    }
    return "unknown error code";
}

extern "C" int ckksmi_ctx_create(const ckksmi_params *p, ckksmi_ctx **out) {
    if (!p || !out) return CKKSMI_EINVAL;
    *out = nullptr;
    if (p->logN < 2 || p->logN > 17) return CKKSMI_EINVAL;
    if (p->n_q < 1 || p->n_q > 62 || p->n_special < 0 || p->n_special > CKKSMI_MAX_SPECIAL) return CKKSMI_EINVAL;
    if (p->n_q + p->n_special > CKKSMI_MAX_MODULI) return CKKSMI_EINVAL;
    const int alpha = p->alpha < 1 ? 1 : p->alpha;
    if (alpha > CKKSMI_MAX_ALPHA || (p->n_special > 0 && alpha > p->n_special)) return CKKSMI_EINVAL;
    if (!p->moduli_override) {
        if (p->q_bits > 51 || p->q_bits < p->logN + 3) return CKKSMI_EINVAL;
        if (p->n_special && (p->special_bits > 51 || p->special_bits < p->logN + 3)) return CKKSMI_EINVAL;
    }
    ckksmi_ctx *c = new (std::nothrow) ckksmi_ctx();
    if (!c) return CKKSMI_EINVAL;
    c->logN = p->logN;
    c->N = (u64)1 << p->logN;
    c->n_q = p->n_q;
    c->k = p->n_special;
    c->alpha = alpha;
    c->T = c->n_q + c->k;
    c->beta_top = (c->n_q + alpha - 1) / alpha;
    c->device = p->device;
    if (p->moduli_override) {
        for (int t = 0; t < c->T; t++) {
            u64 m = p->moduli_override[t];
            bool ok = m < ((u64)1 << 51) && m % (2 * c->N) == 1 && hm::is_prime(m);
            for (u64 prev : c->mod) ok = ok && prev != m;
            if (!ok) { delete c; return CKKSMI_EINVAL; }
            c->mod.push_back(m);
        }
    } else {
        std::vector<u64> q, sp;
        if (!hm::find_primes(p->q_bits, p->logN, c->n_q, {}, q)) { delete c; return CKKSMI_EINVAL; }
        if (c->k && !hm::find_primes(p->special_bits, p->logN, c->k, q, sp)) { delete c; return CKKSMI_EINVAL; }
        c->mod = q;
        c->mod.insert(c->mod.end(), sp.begin(), sp.end());
    }
    for (int t = 0; t < c->T; t++) {
        u64 psi = (p->moduli_override && p->psi_override) ? p->psi_override[t] : hm::find_psi(c->mod[t], c->logN);
        if (psi == 0 || hm::powmod(psi, c->N, c->mod[t]) != c->mod[t] - 1) { delete c; return CKKSMI_EINVAL; }
        c->psi.push_back(psi);
    }
    build_host_tables(c);
    if (c->device >= 0) {
        int rc = dev_upload_tables(c);
        if (rc != CKKSMI_OK) {
            dev_free_tables(c);
            delete c;
            return rc;
        }
    }
    *out = c;
    return CKKSMI_OK;
}

extern "C" void ckksmi_ctx_destroy(ckksmi_ctx *c) {
    if (!c) return;
    if (c->device >= 0) dev_free_tables(c);
    delete c;
}

extern "C" int ckksmi_get_moduli(const ckksmi_ctx *c, uint64_t *moduli, uint64_t *psi) {
    if (!c) return CKKSMI_EINVAL;
    if (moduli) memcpy(moduli, c->mod.data(), c->T * sizeof(u64));
    if (psi) memcpy(psi, c->psi.data(), c->T * sizeof(u64));
    return CKKSMI_OK;
}

extern "C" int ckksmi_last_device_error(const ckksmi_ctx *c) { return c ? c->last_hip_error : 0; }

// ------------------------------------------------------------------ samplers
// Counter-based stream: word i of stream `seed` is the SplitMix64 finaliser applied
// to seed + (i+1)*golden-ratio increment.
namespace {
struct Stream {
    u64 state;
    explicit Stream(u64 seed) : state(seed) {}
    u64 next() {
        u64 z = (state += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    double unit() { return ((next() >> 11) + 0.5) * (1.0 / 9007199254740992.0); }  // (0,1)
};
}  // namespace

extern "C" int ckksmi_sample_ternary(const ckksmi_ctx *c, uint64_t seed, int64_t *out) {
    if (!c || !out) return CKKSMI_EINVAL;
    Stream g(seed);
    const u64 lim = (~(u64)0 / 3) * 3;
    for (u64 n = 0; n < c->N; n++) {
        u64 x;
        do x = g.next(); while (x >= lim);
        out[n] = (i64)(x % 3) - 1;
    }
    return CKKSMI_OK;
}

extern "C" int ckksmi_sample_error(const ckksmi_ctx *c, uint64_t seed, int64_t *out) {
    if (!c || !out) return CKKSMI_EINVAL;
    Stream g(seed);
    const double sigma = 3.2, two_pi = 6.283185307179586476925;
    for (u64 n = 0; n < c->N;) {
        double r = std::sqrt(-2.0 * std::log(g.unit())), th = two_pi * g.unit();
        double pair[2] = {r * std::cos(th), r * std::sin(th)};
        for (int h = 0; h < 2 && n < c->N; h++) {
            double e = std::nearbyint(sigma * pair[h]);
            if (std::fabs(e) <= 19.0) out[n++] = (i64)e;
        }
    }
    return CKKSMI_OK;
}

extern "C" int ckksmi_sample_uniform(const ckksmi_ctx *c, uint64_t seed, const int *index, int n_limbs, uint64_t *out) {
    if (!c || !out || !index || n_limbs < 0) return CKKSMI_EINVAL;
    for (int x = 0; x < n_limbs; x++)
        if (index[x] < 0 || index[x] >= c->T) return CKKSMI_EINVAL;
    Stream g(seed);
    for (int x = 0; x < n_limbs; x++) {
        const u64 q = c->mod[index[x]];
        const u64 mask = (~(u64)0) >> __builtin_clzll(q);
        for (u64 n = 0; n < c->N; n++) {
            u64 v;
            do v = g.next() & mask; while (v >= q);
            out[(size_t)x * c->N + n] = v;
        }
    }
    return CKKSMI_OK;
}

// ------------------------------------------------------------------ encoding
namespace {
// in-place radix-2 DFT of length n (power of two), sign = -1: e^{-2 pi i ut/n}, +1: e^{+...}; unscaled
void dft(std::vector<cld> &a, int sign) {
    const size_t n = a.size();
    int lg = 0;
    while (((size_t)1 << lg) < n) lg++;
    for (size_t i = 0; i < n; i++) {
        size_t j = hm::brev(i, lg);
        if (i < j) std::swap(a[i], a[j]);
    }
    const ld pi = acosl(-1.0L);
    std::vector<cld> root(n / 2 ? n / 2 : 1);
    for (size_t i = 0; i < n / 2; i++) root[i] = cld(cosl(2 * pi * i / n), sign * sinl(2 * pi * i / n));
    for (size_t len = 2; len <= n; len <<= 1) {
        const size_t stride = n / len;
        for (size_t s = 0; s < n; s += len)
            for (size_t j = 0; j < len / 2; j++) {
                cld u = a[s + j], v = a[s + j + len / 2] * root[j * stride];
                a[s + j] = u + v;
                a[s + j + len / 2] = u - v;
            }
    }
}
}  // namespace

extern "C" int ckksmi_encode(const ckksmi_ctx *c, const double *re, const double *im, double scale, int level, uint64_t *pt) {
    if (!c || !re || !pt || !(scale > 0)) return CKKSMI_EINVAL;
    if (!level_ok(c, level)) return CKKSMI_ELEVEL;
    const u64 N = c->N, twoN = 2 * N;
    // values of m at the odd powers zeta^(2u+1): slot k at exponent 5^k, its conjugate at -5^k
    std::vector<cld> v(N, cld(0, 0));
    u64 e = 1;
    for (u64 k = 0; k < N / 2; k++) {
        cld z(re[k], im ? im[k] : 0.0);
        v[(e - 1) / 2] = z;
        v[(twoN - e - 1) / 2] = std::conj(z);
        e = (e * 5) % twoN;
    }
    // v[u] = sum_t (m_t zeta^t) e^{+2 pi i ut/N}  =>  m_t zeta^t = (1/N) sum_u v[u] e^{-2 pi i ut/N}
    dft(v, -1);
    const ld pi = acosl(-1.0L);
    std::vector<i64> coef(N);
    for (u64 t = 0; t < N; t++) {
        cld tw(cosl(pi * t / N), -sinl(pi * t / N));
        ld m = (v[t] * tw).real() / (ld)N * (ld)scale;
        if (!(fabsl(m) < 4.0e18L)) return CKKSMI_EINVAL;
        coef[t] = llroundl(m);
    }
    for (int i = 0; i < level; i++) {
        u64 *o = pt + (size_t)i * N;
        for (u64 t = 0; t < N; t++) o[t] = hm::signed_mod(coef[t], c->mod[i]);
        host_ntt(c, i, o);
    }
    return CKKSMI_OK;
}

extern "C" int ckksmi_decode(const ckksmi_ctx *c, const uint64_t *pt, int level, double scale, double *re, double *im) {
    if (!c || !pt || !re || !(scale > 0)) return CKKSMI_EINVAL;
    if (!level_ok(c, level)) return CKKSMI_ELEVEL;
    const u64 N = c->N, twoN = 2 * N;
    std::vector<u64> coef((size_t)level * N);
    memcpy(coef.data(), pt, (size_t)level * N * sizeof(u64));
    for (int i = 0; i < level; i++) host_intt(c, i, coef.data() + (size_t)i * N);
    // balanced mixed-radix digits: x = v0 + q0*(v1 + q1*(v2 + ...)), |v_i| <= q_i/2, which is
    // the centred representative mod Q; summed top-down in long double.
    std::vector<u64> inv((size_t)level * level, 0);  // inv[i*level+j] = q_j^-1 mod q_i, j < i
    for (int i = 0; i < level; i++)
        for (int j = 0; j < i; j++) inv[(size_t)i * level + j] = hm::invmod(c->mod[j] % c->mod[i], c->mod[i]);
    const ld pi = acosl(-1.0L);
    std::vector<cld> b(N);
    std::vector<i64> dig(level);
    for (u64 t = 0; t < N; t++) {
        for (int i = 0; i < level; i++) {
            const u64 q = c->mod[i];
            u64 r = coef[(size_t)i * N + t] % q;
            for (int j = 0; j < i; j++) {
                r = hm::submod(r, hm::signed_mod(dig[j], q), q);
                r = hm::mulmod(r, inv[(size_t)i * level + j], q);
            }
            dig[i] = r > q / 2 ? (i64)r - (i64)q : (i64)r;
        }
        ld x = 0;
        for (int i = level - 1; i >= 0; i--) x = x * (ld)c->mod[i] + (ld)dig[i];
        b[t] = cld(x, 0) * cld(cosl(pi * t / N), sinl(pi * t / N));
    }
    dft(b, +1);  // values at zeta^(2u+1)
    u64 e = 1;
    for (u64 k = 0; k < N / 2; k++) {
        cld z = b[(e - 1) / 2] / (ld)scale;
        re[k] = (double)z.real();
        if (im) im[k] = (double)z.imag();
        e = (e * 5) % twoN;
    }
    return CKKSMI_OK;
}

// ------------------------------------------------------------------ keys, encryption
namespace {
void small_to_eval(const ckksmi_ctx *c, const i64 *coef, int t, u64 *out) {
    for (u64 n = 0; n < c->N; n++) out[n] = hm::signed_mod(coef[n], c->mod[t]);
    host_ntt(c, t, out);
}

// key[j][0][t] = -a*s + e_j + [t in digit j]*(P mod t)*s',  key[j][1][t] = a
// sprime_coef == nullptr means s' = s^2 (squared pointwise in evaluation form)
int make_switch_key(const ckksmi_ctx *c, const i64 *s, const std::vector<i64> *sprime_coef, const u64 *a, const i64 *e, u64 *key) {
    const u64 N = c->N;
    const int T = c->T;
    std::vector<u64> sh(N), eh(N), sp(N);
    for (int t = 0; t < T; t++) {
        const u64 q = c->mod[t];
        small_to_eval(c, s, t, sh.data());
        if (sprime_coef) small_to_eval(c, sprime_coef->data(), t, sp.data());
        else for (u64 n = 0; n < N; n++) sp[n] = hm::mulmod(sh[n], sh[n], q);
        u64 Pq = 1;
        for (int m = 0; m < c->k; m++) Pq = hm::mulmod(Pq, c->mod[c->n_q + m] % q, q);
        for (int j = 0; j < c->beta_top; j++) {
            small_to_eval(c, e + (size_t)j * N, t, eh.data());
            const bool gadget = t < c->n_q && t / c->alpha == j;
            const u64 *aj = a + ((size_t)j * T + t) * N;
            u64 *kb = key + (((size_t)j * 2 + 0) * T + t) * N;
            u64 *ka = key + (((size_t)j * 2 + 1) * T + t) * N;
            for (u64 n = 0; n < N; n++) {
                if (aj[n] >= q) return CKKSMI_EINVAL;
                u64 v = hm::addmod(hm::submod(0, hm::mulmod(aj[n], sh[n], q), q), eh[n], q);
                if (gadget) v = hm::addmod(v, hm::mulmod(Pq, sp[n], q), q);
                kb[n] = v;
                ka[n] = aj[n];
            }
        }
    }
    return CKKSMI_OK;
}

}  // namespace

extern "C" int ckksmi_keygen_public(const ckksmi_ctx *c, const int64_t *s, const uint64_t *a, const int64_t *e, uint64_t *pk) {
    if (!c || !s || !a || !e || !pk) return CKKSMI_EINVAL;
    const u64 N = c->N;
    std::vector<u64> sh(N), eh(N);
    for (int i = 0; i < c->n_q; i++) {
        const u64 q = c->mod[i];
        small_to_eval(c, s, i, sh.data());
        small_to_eval(c, e, i, eh.data());
        u64 *b = pk + (size_t)i * N, *a_out = pk + (size_t)(c->n_q + i) * N;
        const u64 *ai = a + (size_t)i * N;
        for (u64 n = 0; n < N; n++) {
            if (ai[n] >= q) return CKKSMI_EINVAL;
            b[n] = hm::addmod(hm::submod(0, hm::mulmod(ai[n], sh[n], q), q), eh[n], q);
            a_out[n] = ai[n];
        }
    }
    return CKKSMI_OK;
}

extern "C" int ckksmi_keygen_relin(const ckksmi_ctx *c, const int64_t *s, const uint64_t *a, const int64_t *e, uint64_t *evk) {
    if (!c || !s || !a || !e || !evk) return CKKSMI_EINVAL;
    if (c->k == 0) return CKKSMI_EUNSUPPORTED;
    return make_switch_key(c, s, nullptr, a, e, evk);
}

static u64 galois_element(const ckksmi_ctx *c, int rot) {
    const i64 half = (i64)(c->N / 2);
    i64 r = ((i64)rot % half + half) % half;
    return hm::powmod(5, (u64)r, 2 * c->N);
}

extern "C" int ckksmi_keygen_galois(const ckksmi_ctx *c, const int64_t *s, int rot, const uint64_t *a, const int64_t *e, uint64_t *gk) {
    if (!c || !s || !a || !e || !gk) return CKKSMI_EINVAL;
    if (c->k == 0) return CKKSMI_EUNSUPPORTED;
    const u64 N = c->N, g = galois_element(c, rot);
    std::vector<i64> sg(N);
    for (u64 t = 0; t < N; t++) {
        u64 idx = (t * g) % (2 * N);
        if (idx < N) sg[idx] = s[t];
        else sg[idx - N] = -s[t];
    }
    return make_switch_key(c, s, &sg, a, e, gk);
}

extern "C" int ckksmi_encrypt(const ckksmi_ctx *c, const uint64_t *pk, const uint64_t *pt, const int64_t *r, const int64_t *e0, const int64_t *e1, int level, uint64_t *ct) {
    if (!c || !pk || !pt || !r || !e0 || !e1 || !ct) return CKKSMI_EINVAL;
    if (!level_ok(c, level)) return CKKSMI_ELEVEL;
    const u64 N = c->N;
    std::vector<u64> rh(N), e0h(N), e1h(N);
    for (int i = 0; i < level; i++) {
        const u64 q = c->mod[i];
        small_to_eval(c, r, i, rh.data());
        small_to_eval(c, e0, i, e0h.data());
        small_to_eval(c, e1, i, e1h.data());
        const u64 *b = pk + (size_t)i * N, *a = pk + (size_t)(c->n_q + i) * N, *m = pt + (size_t)i * N;
        u64 *c0 = ct + (size_t)i * N, *c1 = ct + (size_t)(level + i) * N;
        for (u64 n = 0; n < N; n++) {
            if (b[n] >= q || a[n] >= q || m[n] >= q) return CKKSMI_EINVAL;
            c0[n] = hm::addmod(hm::addmod(hm::mulmod(rh[n], b[n], q), e0h[n], q), m[n], q);
            c1[n] = hm::addmod(hm::mulmod(rh[n], a[n], q), e1h[n], q);
        }
    }
    return CKKSMI_OK;
}

extern "C" int ckksmi_decrypt(const ckksmi_ctx *c, const int64_t *s, const uint64_t *ct, int level, int n_comp, uint64_t *pt) {
    if (!c || !s || !ct || !pt || n_comp < 2 || n_comp > 3) return CKKSMI_EINVAL;
    if (!level_ok(c, level)) return CKKSMI_ELEVEL;
    const u64 N = c->N;
    std::vector<u64> sh(N);
    for (int i = 0; i < level; i++) {
        const u64 q = c->mod[i];
        small_to_eval(c, s, i, sh.data());
        u64 *o = pt + (size_t)i * N;
        for (u64 n = 0; n < N; n++) {
            // Horner in s: (c2*s + c1)*s + c0
            u64 acc = 0;
            for (int comp = n_comp - 1; comp >= 0; comp--) {
                u64 w = ct[((size_t)comp * level + i) * N + n];
                if (w >= q) return CKKSMI_EINVAL;
                acc = hm::addmod(hm::mulmod(acc, sh[n], q), w, q);
            }
            o[n] = acc;
        }
    }
    return CKKSMI_OK;
}

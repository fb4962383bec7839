// Device-side encoding and encryption (section 2.1: m = round(scale * phi^-1(z)), ct = (r*b + e0 + m, r*a + e1)).
//
// Encoding is the INVERSE of "evaluate the polynomial at the odd powers of zeta = exp(i*pi/N)", i.e. the inverse
// negacyclic transform over the complex numbers: the same Gentleman-Sande butterfly network as the modular inverse
// transform (kernels.h), with complex twiddles zeta^-brev(x) and complex double arithmetic.  Slot k belongs to the
// exponent 5^k mod 2N and its conjugate to -5^k; in the transform's evaluation order, exponent 2u+1 sits at index
// brev(u).  The real parts of the result, times scale/N, rounded to nearest, are the plaintext coefficients.
// Encryption is exact integer work: the small polynomials r, e0, e1 go to residues and through the forward transform,
// then one pointwise kernel combines them with the public key and the plaintext.
#pragma once
#include "kernels.h"

#define CFFT_TILE 4096  // complex words staged in LDS per workgroup (64 KiB)

struct EncodeArgs {
    const double *re, *im;   // [batch][N/2], im may be null
    double2 *cbuf;           // [batch][N]
    const unsigned *slot_exp;  // [N/2]: 5^k mod 2N
    const double2 *ctw;      // [N]: zeta^-brev(x)
    int logN, LA;
    int *flag;               // this call's overflow word: cleared here by the first kernel of the sequence, raised by the last
};

__device__ __forceinline__ double2 cmul(double2 a, double2 b) { return make_double2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x); }

// grid: x = block of slots, y = item
__global__ __launch_bounds__(EW_THREADS) void encode_scatter_kernel(EncodeArgs A) {
    const unsigned N = 1u << A.logN, half = N >> 1;
    const unsigned k = blockIdx.x * EW_THREADS + threadIdx.x;
    if (k == 0 && blockIdx.y == 0) *A.flag = 0;  // the rounding kernel that may raise it runs later on the same stream
    if (k >= half) return;
    const size_t item = blockIdx.y;
    const double zr = A.re[item * half + k], zi = A.im ? A.im[item * half + k] : 0.0;
    const unsigned e = A.slot_exp[k];
    const unsigned j = __brev((e - 1u) >> 1) >> (32 - A.logN);
    const unsigned jc = __brev((2u * N - e - 1u) >> 1) >> (32 - A.logN);
    double2 *v = A.cbuf + item * N;
    v[j] = make_double2(zr, zi);
    v[jc] = make_double2(zr, -zi);
}

// Inverse complex negacyclic transform, the stage split of ntt_inv_kernel: COL = false first (stages logN-1 .. LA on
// contiguous rows of N >> LA words), COL = true second (stages LA-1 .. 0 on strided tiles).  Unscaled (no 1/N).
// grid: x = item, y = tile
template <bool COL>
__global__ __launch_bounds__(NTT_THREADS) void cfft_inv_kernel(EncodeArgs A) {
    __shared__ double2 tile[CFFT_TILE];
    const unsigned N = 1u << A.logN;
    double2 *buf = A.cbuf + (size_t)blockIdx.x * N;
    const double2 *tw = A.ctw;
    const unsigned tid = threadIdx.x;
    if (!COL) {
        const unsigned N2 = N >> A.LA, N1 = 1u << A.LA;
        const unsigned R = (N2 >= CFFT_TILE) ? 1u : CFFT_TILE / N2;
        const unsigned rows_here = (N1 - blockIdx.y * R < R) ? N1 - blockIdx.y * R : R;
        const unsigned row0 = blockIdx.y * R;
        const unsigned cnt = rows_here * N2;
        const size_t g0 = (size_t)row0 * N2;
        for (unsigned e = tid; e < cnt; e += NTT_THREADS) tile[e] = buf[g0 + e];
        __syncthreads();
        const int LB = A.logN - A.LA;
        for (int s = LB - 1; s >= 0; s--) {
            const unsigned mp = 1u << s, tt = N2 >> (s + 1);
            for (unsigned b = tid; b < cnt / 2; b += NTT_THREADS) {
                const unsigned rr = b / (N2 / 2), bb = b % (N2 / 2);
                const unsigned i = bb / tt, j = bb % tt;
                const unsigned lo = rr * N2 + i * 2 * tt + j, hi = lo + tt;
                const double2 x = tile[lo], y = tile[hi];
                const double2 W = tw[mp * (N1 + row0 + rr) + i];
                tile[lo] = make_double2(x.x + y.x, x.y + y.y);
                tile[hi] = cmul(make_double2(x.x - y.x, x.y - y.y), W);
            }
            __syncthreads();
        }
        for (unsigned e = tid; e < cnt; e += NTT_THREADS) buf[g0 + e] = tile[e];
    } else {
        const unsigned N1 = 1u << A.LA, N2 = N >> A.LA;
        const unsigned c0 = blockIdx.y * NTT_TC;
        for (unsigned e = tid; e < N1 * NTT_TC; e += NTT_THREADS) {
            const unsigned r = e / NTT_TC, c = e % NTT_TC;
            tile[e] = buf[(size_t)r * N2 + c0 + c];
        }
        __syncthreads();
        for (int s = A.LA - 1; s >= 0; s--) {
            const unsigned m = 1u << s, tr = N1 >> (s + 1);
            for (unsigned b = tid; b < (N1 / 2) * NTT_TC; b += NTT_THREADS) {
                const unsigned c = b % NTT_TC, rb = b / NTT_TC;
                const unsigned i = rb / tr, jr = rb % tr;
                const unsigned lo = (i * 2 * tr + jr) * NTT_TC + c, hi = lo + tr * NTT_TC;
                const double2 x = tile[lo], y = tile[hi];
                const double2 W = tw[m + i];
                tile[lo] = make_double2(x.x + y.x, x.y + y.y);
                tile[hi] = cmul(make_double2(x.x - y.x, x.y - y.y), W);
            }
            __syncthreads();
        }
        for (unsigned e = tid; e < N1 * NTT_TC; e += NTT_THREADS) {
            const unsigned r = e / NTT_TC, c = e % NTT_TC;
            buf[(size_t)r * N2 + c0 + c] = tile[e];
        }
    }
}

// coefficients m_t = rint(Re(v_t) * factor) (factor = scale / N), then their residues: out [batch][level][N] in
// coefficient form.  A coefficient of 2^62 or more in magnitude raises *overflow (the host reports CKKSMI_EINVAL).
__global__ __launch_bounds__(EW_THREADS) void encode_round_kernel(const double2 *cbuf, double factor, u64d *out, const ModConst *modc, int logN,
                                                                  int level, size_t total /* batch*N */, int *overflow) {
    const size_t w = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (w >= total) return;
    const size_t N = (size_t)1 << logN, item = w >> logN, t = w & (N - 1);
    const double m = rint(cbuf[w].x * factor);
    if (!(fabs(m) < 4.0e18)) {
        *overflow = 1;
        return;
    }
    const long long mi = (long long)m;
    for (int i = 0; i < level; i++) {
        const long long q = (long long)modc[i].p;
        long long r = mi % q;
        if (r < 0) r += q;
        out[(item * level + i) * N + t] = (u64d)r;
    }
}

// residues of small signed polynomials: in [rows][N] (int64), row r written to out + r*out_row_stride as [level][N],
// coefficient form
__global__ __launch_bounds__(EW_THREADS) void small_to_rns_kernel(const long long *in, u64d *out, unsigned long long out_row_stride,
                                                                  const ModConst *modc, int logN, int level, size_t total /* rows*N */) {
    const size_t w = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (w >= total) return;
    const size_t N = (size_t)1 << logN, row = w >> logN, t = w & (N - 1);
    const long long v = in[w];
    for (int i = 0; i < level; i++) {
        const long long q = (long long)modc[i].p;
        long long r = v % q;
        if (r < 0) r += q;
        out[row * out_row_stride + (size_t)i * N + t] = (u64d)r;
    }
}

// ct0 = r*b + e0 + m, ct1 = r*a + e1 (all in evaluation form); small: [batch][3][level][N] = (r, e0, e1) per item,
// pk: [2][n_q][N], pt: [batch][level][N], ct: [batch][2][level][N]
__global__ __launch_bounds__(EW_THREADS) void encrypt_combine_kernel(const u64d *small, const u64d *pk, const u64d *pt, u64d *ct,
                                                                     const ModConst *modc, int logN, int level, int n_q, size_t total /* batch*level*N */) {
    const size_t w = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (w >= total) return;
    const size_t N = (size_t)1 << logN, limb = w >> logN, n = w & (N - 1);
    const size_t item = limb / level, i = limb % level;
    const ModConst mc = modc[i];
    const size_t st = (size_t)level * N, so = (item * 3 * level + i) * N + n;
    const double r = u2d(small[so]), e0 = u2d(small[so + st]), e1 = u2d(small[so + 2 * st]);
    const double b = u2d(pk[i * N + n]), a = u2d(pk[((size_t)n_q + i) * N + n]);
    const double m = u2d(pt[(item * level + i) * N + n]);
    // mulmod: |result| <= 1.25p; plus two canonical words: below 4p
    const double c0 = canon(mulmod(r, b, mc.p, mc.pinv) + e0 + m, mc.p, mc.pinv);
    const double c1 = canon(mulmod(r, a, mc.p, mc.pinv) + e1, mc.p, mc.pinv);
    ct[(item * 2 * level + i) * N + n] = d2u(c0);
    ct[(item * 2 * level + level + i) * N + n] = d2u(c1);
}

// The same on the register-tiled kernels (2^12 <= N <= 2^16), after the forward column pass of r, e0, e1
// (ntt_v2_fwd_cols_small_kernel): a workgroup takes the three polynomials' tiles of one limb through the forward row pass one
// after the other and forms both ciphertext words while the results are on chip, so that the transformed r, e0, e1 are
// never written.  mid: [items][3][level][N] column-pass output (reduced doubles).
struct EncryptRowsArgs {
    const u64d *mid, *pk, *pt;
    u64d *ct;
    const ModConst *modc;
    const double *tw;  // forward twiddles
    int logN, level, n_q, items, items_per_x;
    P51Mask p51;
};

template <bool P51>
__device__ __forceinline__ void encrypt_rows_body(const EncryptRowsArgs &A, double *lds, double *tw1_lds, int i) {
    const unsigned N = 1u << A.logN, N1 = N >> 8;
    const double p = A.modc[i].p, pinv = A.modc[i].pinv;
    const unsigned tid = threadIdx.x, hi4 = tid >> 4, lo4 = tid & 15, tile = blockIdx.y;
    double tw2[15];
    load_row_twiddles(A.tw + (size_t)i * N, N1, tile, hi4, lo4, tw1_lds, tw2);
    const size_t tile0 = (size_t)tile * 4096, st = (size_t)A.level * N;
    // the public key's words of this tile serve every item of the workgroup
    ulonglong2 kb[8], ka[8];
#pragma unroll
    for (int s = 0; s < 8; s++) {
        kb[s] = ((const ulonglong2 *)(A.pk + (size_t)i * N + tile0))[row_pair_index(hi4, lo4, s)];
        ka[s] = ((const ulonglong2 *)(A.pk + ((size_t)A.n_q + i) * N + tile0))[row_pair_index(hi4, lo4, s)];
    }
    const unsigned it0 = blockIdx.x * (unsigned)A.items_per_x;
    const unsigned it1 = (it0 + A.items_per_x < (unsigned)A.items) ? it0 + A.items_per_x : (unsigned)A.items;
    for (unsigned it = it0; it < it1; it++) {
        const u64d *mid = A.mid + ((size_t)it * 3 * A.level + i) * N + tile0;
        ulonglong2 mm[8];
#pragma unroll
        for (int s = 0; s < 8; s++) mm[s] = ((const ulonglong2 *)(A.pt + ((size_t)it * A.level + i) * N + tile0))[row_pair_index(hi4, lo4, s)];
        rows_fwd_to_lds<P51>(mid, lds, tw1_lds, tw2, p, pinv, hi4, lo4);
        double r[16];
#pragma unroll
        for (int s = 0; s < 8; s++) {
            const double *rr = lds + hi4 * V2_GS + row_pair_lds(lo4, s);
            r[2 * s] = rr[0];
            r[2 * s + 1] = rr[1];
        }
        ROW_GROUP_SYNC();
        rows_fwd_to_lds<P51>(mid + st, lds, tw1_lds, tw2, p, pinv, hi4, lo4);
        u64d *c0 = A.ct + ((size_t)it * 2 * A.level + i) * N + tile0, *c1 = c0 + st;
#pragma unroll
        for (int s = 0; s < 8; s++) {
            // a product (1.25p), a balanced-reduced word and a canonical one: below 4p
            const double *ee = lds + hi4 * V2_GS + row_pair_lds(lo4, s);
            const double v0 = mulmod(r[2 * s], u2d(kb[s].x), p, pinv) + ee[0] + u2d(mm[s].x);
            const double v1 = mulmod(r[2 * s + 1], u2d(kb[s].y), p, pinv) + ee[1] + u2d(mm[s].y);
            ((ulonglong2 *)c0)[row_pair_index(hi4, lo4, s)] = make_ulonglong2(d2u(canon(v0, p, pinv)), d2u(canon(v1, p, pinv)));
        }
        ROW_GROUP_SYNC();
        rows_fwd_to_lds<P51>(mid + 2 * st, lds, tw1_lds, tw2, p, pinv, hi4, lo4);
#pragma unroll
        for (int s = 0; s < 8; s++) {
            const double *ee = lds + hi4 * V2_GS + row_pair_lds(lo4, s);
            const double v0 = mulmod(r[2 * s], u2d(ka[s].x), p, pinv) + ee[0];
            const double v1 = mulmod(r[2 * s + 1], u2d(ka[s].y), p, pinv) + ee[1];
            ((ulonglong2 *)c1)[row_pair_index(hi4, lo4, s)] = make_ulonglong2(d2u(canon(v0, p, pinv)), d2u(canon(v1, p, pinv)));
        }
        ROW_GROUP_SYNC();
    }
}

// grid: x = chunk of items, y = row tile (N/4096), z = limb
__global__ __launch_bounds__(V2_THREADS) void encrypt_rows_kernel(EncryptRowsArgs A) {
    __shared__ double lds[16 * V2_GS];
    __shared__ double tw1_lds[16 * 16];
    const int i = (int)blockIdx.z;
    if (is_p51(A.p51, i))
        encrypt_rows_body<true>(A, lds, tw1_lds, i);
    else
        encrypt_rows_body<false>(A, lds, tw1_lds, i);
}

// ---------------------------------------------------------------- sampling
// Counter-based (Philox4x32-10: Salmon, Moraes, Dror, Shaw 2011), one block per coefficient: counter
// (t, kind, lo32(p), hi32(p)) for coefficient t of polynomial p, key = the two halves of the seed.
//   kind 0, ternary : ((w0 * 3) >> 32) - 1
//   kind 1, Gaussian: magnitude = number of thresholds T_k <= u, u = w1*2^32 + w0; negative when w2 is odd
#define SAMPLE_K 40
struct SampleArgs {
    long long *out;  // [rows][N]
    unsigned long long seed, first_index;
    int kind, logN;
    size_t total;    // rows * N
    unsigned long long T[SAMPLE_K];  // floor(2^64 * P(|X| <= k)) of the rounded Gaussian
};

__device__ __forceinline__ void philox4x32_10(unsigned c0, unsigned c1, unsigned c2, unsigned c3, unsigned k0, unsigned k1, unsigned (&w)[4]) {
#pragma unroll
    for (int r = 0; r < 10; r++) {
        if (r) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
        const unsigned long long p0 = 0xD2511F53ull * c0, p1 = 0xCD9E8D57ull * c2;
        const unsigned n0 = (unsigned)(p1 >> 32) ^ c1 ^ k0, n1 = (unsigned)p1, n2 = (unsigned)(p0 >> 32) ^ c3 ^ k1, n3 = (unsigned)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    w[0] = c0; w[1] = c1; w[2] = c2; w[3] = c3;
}

__global__ __launch_bounds__(EW_THREADS) void sample_kernel(SampleArgs A) {
    const size_t idx = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= A.total) return;
    const unsigned long long p = A.first_index + (idx >> A.logN);
    const unsigned t = (unsigned)(idx & (((size_t)1 << A.logN) - 1));
    unsigned w[4];
    philox4x32_10(t, (unsigned)A.kind, (unsigned)p, (unsigned)(p >> 32), (unsigned)A.seed, (unsigned)(A.seed >> 32), w);
    long long v;
    if (A.kind == 0) {
        v = (long long)(((unsigned long long)w[0] * 3ull) >> 32) - 1;
    } else {
        const unsigned long long u = ((unsigned long long)w[1] << 32) | w[0];
        int mag = 0;
#pragma unroll
        for (int k = 0; k < SAMPLE_K; k++) mag += (u >= A.T[k]) ? 1 : 0;
        v = (w[2] & 1u) ? -(long long)mag : (long long)mag;
    }
    A.out[idx] = v;
}

// HIP kernels of the RNS-CKKS hot path (gfx950).  All modular arithmetic runs on the
// FP64 vector ALU (device_arith.h); words in HBM are canonical uint64 residues.
#pragma once
#include "device_arith.h"

typedef unsigned long long u64d;

#define NTT_THREADS 256
#define NTT_TILE 4096   // doubles staged in LDS per workgroup (32 KiB)
#define NTT_TC 16       // contiguous words per row segment in the strided (column) pass

// How the limb handled by blockIdx.x maps to memory and to a modulus.
//   limb = item * per_item + li;  address = base + item * item_stride + li * N
//   mode 0: modulus index = modidx[li]
//   mode 1: key-switch extended basis: li = j*E + x, modulus = x < level ? x : n_q + x - level,
//           and the limb is skipped when x belongs to digit j (it is already in evaluation form)
struct LimbMap {
    int per_item;
    int mode;
    int level, E, n_q, alpha;
    unsigned long long src_item_stride, dst_item_stride;
    unsigned char modidx[CKKSMI_MAX_MODULI];
};

struct NttArgs {
    const u64d *src;
    u64d *dst;
    const ModConst *modc;
    const WMul *tw;       // [T][N]
    const WMul *tw_last;  // [T] inverse only: psi^-brev(1) / N
    int logN, LA;         // LA = stages done by the strided pass (0 = none)
    LimbMap map;
};

__device__ __forceinline__ int resolve_limb(const LimbMap &M, unsigned limb, unsigned &item, unsigned &li) {
    item = limb / (unsigned)M.per_item;
    li = limb % (unsigned)M.per_item;
    if (M.mode == 0) return M.modidx[li];
    unsigned j = li / (unsigned)M.E, x = li % (unsigned)M.E;
    if ((int)x < M.level) return ((int)(x / (unsigned)M.alpha) == (int)j) ? -1 : (int)x;
    return M.n_q + (int)x - M.level;
}

// ---------------------------------------------------------------- forward transform
// Decimation in time with the negacyclic twist merged into the twiddles: stage s has
// m = 2^s blocks of span N/(2m); block i multiplies its upper half by psi^brev(m+i).
// COL = true : stages [0, LA) on a strided tile (2^LA rows x NTT_TC columns)
// COL = false: stages [LA, logN) on contiguous rows of N2 = N >> LA words
template <bool COL>
__global__ __launch_bounds__(NTT_THREADS) void ntt_fwd_kernel(NttArgs A) {
    __shared__ double tile[NTT_TILE];
    unsigned item, li;
    const int t = resolve_limb(A.map, blockIdx.x, item, li);
    if (t < 0) return;
    const unsigned N = 1u << A.logN;
    const u64d *src = A.src + (size_t)item * A.map.src_item_stride + (size_t)li * N;
    u64d *dst = A.dst + (size_t)item * A.map.dst_item_stride + (size_t)li * N;
    const double p = A.modc[t].p, pinv = A.modc[t].pinv;
    const WMul *tw = A.tw + (size_t)t * N;
    const unsigned tid = threadIdx.x;
    if (COL) {
        const unsigned N1 = 1u << A.LA, N2 = N >> A.LA;
        const unsigned c0 = blockIdx.y * NTT_TC;
        for (unsigned e = tid; e < N1 * NTT_TC; e += NTT_THREADS) {
            unsigned r = e / NTT_TC, c = e % NTT_TC;
            tile[e] = u2d(src[(size_t)r * N2 + c0 + c]);
        }
        __syncthreads();
        for (int s = 0; s < A.LA; s++) {
            const unsigned m = 1u << s, tr = N1 >> (s + 1);
            const bool red = (s & 1) != 0;
            for (unsigned b = tid; b < (N1 / 2) * NTT_TC; b += NTT_THREADS) {
                unsigned c = b % NTT_TC, rb = b / NTT_TC;
                unsigned i = rb / tr, jr = rb % tr;
                unsigned lo = (i * 2 * tr + jr) * NTT_TC + c, hi = lo + tr * NTT_TC;
                WMul W = tw[m + i];
                double x = tile[lo], v = mulmod_w(tile[hi], W.w, W.wp, p);
                double X = x + v, Y = x - v;
                if (red) { X = reduce_balanced(X, p, pinv); Y = reduce_balanced(Y, p, pinv); }
                tile[lo] = X;
                tile[hi] = Y;
            }
            __syncthreads();
        }
        for (unsigned e = tid; e < N1 * NTT_TC; e += NTT_THREADS) {
            unsigned r = e / NTT_TC, c = e % NTT_TC;
            dst[(size_t)r * N2 + c0 + c] = d2u(canon(tile[e], p, pinv));
        }
    } else {
        const unsigned N2 = N >> A.LA, N1 = 1u << A.LA;
        const unsigned R = (N2 >= NTT_TILE) ? 1u : NTT_TILE / N2;  // rows per workgroup
        const unsigned rows_here = (N1 - blockIdx.y * R < R) ? N1 - blockIdx.y * R : R;
        const unsigned row0 = blockIdx.y * R;
        const unsigned cnt = rows_here * N2;
        const size_t g0 = (size_t)row0 * N2;
        for (unsigned e = tid; e < cnt; e += NTT_THREADS) tile[e] = u2d(src[g0 + e]);
        __syncthreads();
        const int LB = A.logN - A.LA;
        for (int s = 0; s < LB; s++) {
            const unsigned mp = 1u << s, tt = N2 >> (s + 1);
            const bool red = (s & 1) != 0;
            for (unsigned b = tid; b < cnt / 2; b += NTT_THREADS) {
                unsigned rr = b / (N2 / 2), bb = b % (N2 / 2);
                unsigned i = bb / tt, j = bb % tt;
                unsigned lo = rr * N2 + i * 2 * tt + j, hi = lo + tt;
                WMul W = tw[mp * (N1 + row0 + rr) + i];
                double x = tile[lo], v = mulmod_w(tile[hi], W.w, W.wp, p);
                double X = x + v, Y = x - v;
                if (red) { X = reduce_balanced(X, p, pinv); Y = reduce_balanced(Y, p, pinv); }
                tile[lo] = X;
                tile[hi] = Y;
            }
            __syncthreads();
        }
        for (unsigned e = tid; e < cnt; e += NTT_THREADS) dst[g0 + e] = d2u(canon(tile[e], p, pinv));
    }
}

// ---------------------------------------------------------------- inverse transform
// Gentleman-Sande butterflies undoing the forward stages last to first; the factor
// 1/N is folded into the very last stage (m = 1).
// COL = false runs first: stages logN-1 .. LA on contiguous rows;
// COL = true  second   : stages LA-1 .. 0 on the strided tile.
template <bool COL>
__global__ __launch_bounds__(NTT_THREADS) void ntt_inv_kernel(NttArgs A) {
    __shared__ double tile[NTT_TILE];
    unsigned item, li;
    const int t = resolve_limb(A.map, blockIdx.x, item, li);
    if (t < 0) return;
    const unsigned N = 1u << A.logN;
    const u64d *src = A.src + (size_t)item * A.map.src_item_stride + (size_t)li * N;
    u64d *dst = A.dst + (size_t)item * A.map.dst_item_stride + (size_t)li * N;
    const double p = A.modc[t].p, pinv = A.modc[t].pinv;
    const WMul *tw = A.tw + (size_t)t * N;
    const WMul ninv = tw[0], wlast = A.tw_last[t];
    const unsigned tid = threadIdx.x;
    if (!COL) {
        const unsigned N2 = N >> A.LA, N1 = 1u << A.LA;
        const unsigned R = (N2 >= NTT_TILE) ? 1u : NTT_TILE / N2;
        const unsigned rows_here = (N1 - blockIdx.y * R < R) ? N1 - blockIdx.y * R : R;
        const unsigned row0 = blockIdx.y * R;
        const unsigned cnt = rows_here * N2;
        const size_t g0 = (size_t)row0 * N2;
        for (unsigned e = tid; e < cnt; e += NTT_THREADS) tile[e] = u2d(src[g0 + e]);
        __syncthreads();
        const int LB = A.logN - A.LA;
        int done = 0;
        for (int s = LB - 1; s >= 0; s--, done++) {
            const unsigned mp = 1u << s, tt = N2 >> (s + 1);
            const bool red = (done & 1) != 0;
            const bool final_stage = (A.LA == 0 && s == 0);
            for (unsigned b = tid; b < cnt / 2; b += NTT_THREADS) {
                unsigned rr = b / (N2 / 2), bb = b % (N2 / 2);
                unsigned i = bb / tt, j = bb % tt;
                unsigned lo = rr * N2 + i * 2 * tt + j, hi = lo + tt;
                double x = tile[lo], y = tile[hi];
                double X, Y;
                if (final_stage) {
                    X = mulmod_w(x + y, ninv.w, ninv.wp, p);
                    Y = mulmod_w(x - y, wlast.w, wlast.wp, p);
                } else {
                    WMul W = tw[mp * (N1 + row0 + rr) + i];
                    X = x + y;
                    Y = mulmod_w(x - y, W.w, W.wp, p);
                    if (red) { X = reduce_balanced(X, p, pinv); Y = reduce_balanced(Y, p, pinv); }
                }
                tile[lo] = X;
                tile[hi] = Y;
            }
            __syncthreads();
        }
        for (unsigned e = tid; e < cnt; e += NTT_THREADS) dst[g0 + e] = d2u(canon(tile[e], p, pinv));
    } else {
        const unsigned N1 = 1u << A.LA, N2 = N >> A.LA;
        const unsigned c0 = blockIdx.y * NTT_TC;
        for (unsigned e = tid; e < N1 * NTT_TC; e += NTT_THREADS) {
            unsigned r = e / NTT_TC, c = e % NTT_TC;
            tile[e] = u2d(src[(size_t)r * N2 + c0 + c]);
        }
        __syncthreads();
        int done = 0;
        for (int s = A.LA - 1; s >= 0; s--, done++) {
            const unsigned m = 1u << s, tr = N1 >> (s + 1);
            const bool red = (done & 1) != 0;
            for (unsigned b = tid; b < (N1 / 2) * NTT_TC; b += NTT_THREADS) {
                unsigned c = b % NTT_TC, rb = b / NTT_TC;
                unsigned i = rb / tr, jr = rb % tr;
                unsigned lo = (i * 2 * tr + jr) * NTT_TC + c, hi = lo + tr * NTT_TC;
                double x = tile[lo], y = tile[hi];
                double X, Y;
                if (s == 0) {
                    X = mulmod_w(x + y, ninv.w, ninv.wp, p);
                    Y = mulmod_w(x - y, wlast.w, wlast.wp, p);
                } else {
                    WMul W = tw[m + i];
                    X = x + y;
                    Y = mulmod_w(x - y, W.w, W.wp, p);
                    if (red) { X = reduce_balanced(X, p, pinv); Y = reduce_balanced(Y, p, pinv); }
                }
                tile[lo] = X;
                tile[hi] = Y;
            }
            __syncthreads();
        }
        for (unsigned e = tid; e < N1 * NTT_TC; e += NTT_THREADS) {
            unsigned r = e / NTT_TC, c = e % NTT_TC;
            dst[(size_t)r * N2 + c0 + c] = d2u(canon(tile[e], p, pinv));
        }
    }
}

// ---------------------------------------------------------------- limb-wise kernels
// Arrays are [rows][level][N] with row = (item, component); word w of the array belongs
// to limb (w / N) % level.
#define EW_THREADS 256

struct ScalarTab { WMul c[64]; double cpos[64]; };  // per limb: constant as multiplicand / canonical value

__global__ __launch_bounds__(EW_THREADS) void addsub_kernel(const u64d *a, const u64d *b, u64d *out, const ModConst *modc,
                                                             int logN, int level, size_t total, int sub) {
    size_t w = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (w >= total) return;
    const u64d q = (u64d)modc[(w >> logN) % level].p;
    u64d x = a[w], y = b[w];
    u64d r = sub ? (x >= y ? x - y : x + q - y) : (x + y >= q ? x + y - q : x + y);
    out[w] = r;
}

// out = a * pt ; pt is [level][N], pt_stride words between items (0 = shared)
__global__ __launch_bounds__(EW_THREADS) void mul_plain_kernel(const u64d *a, const u64d *pt, size_t pt_stride, u64d *out,
                                                               const ModConst *modc, int logN, int level, size_t total) {
    size_t w = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (w >= total) return;
    const size_t N = (size_t)1 << logN;
    const size_t limb = w >> logN, i = limb % level, item = limb / (2 * (size_t)level);
    const ModConst mc = modc[i];
    double x = u2d(a[w]), y = u2d(pt[item * pt_stride + i * N + (w & (N - 1))]);
    out[w] = d2u(canon(mulmod(x, y, mc.p, mc.pinv), mc.p, mc.pinv));
}

// out[g] = sum over the ciphertexts s with term[g][s] >= 0 of pts[term[g][s]] * cts[s] (both components).
// grid: x = word blocks, y = limb, z = chunks of PM_GROUPS groups: a thread loads the word of ciphertext s once for the
// chunk's groups (the ciphertexts are re-read once per chunk, the plaintexts once in all).  A table entry beyond the
// plaintexts counts as "none", so a wrong table gives wrong sums, never an access outside the buffers.  The running
// sums are balanced-reduced after every second term.
#define PM_GROUPS 8
// the word pairs of source ciphertext `sct` and of the plaintexts its PM_GROUPS table entries name (0 where there is none)
__device__ __forceinline__ void plain_mac_fetch(const u64d *cts, const u64d *pts, const int *term, int sct, int n_ct, int n_pts, int n_groups, int g0,
                                                size_t ct_words, size_t pt_words, size_t off, ulonglong2 &x0, ulonglong2 &x1,
                                                ulonglong2 (&y)[PM_GROUPS]) {
    const u64d *x = cts + (size_t)sct * ct_words + off;
    x0 = *(const ulonglong2 *)x;
    x1 = *(const ulonglong2 *)(x + pt_words);
#pragma unroll
    for (int k = 0; k < PM_GROUPS; k++) {
        const int t = g0 + k < n_groups ? term[(size_t)(g0 + k) * n_ct + sct] : -1;  // the same for every thread
        y[k] = (t >= 0 && t < n_pts) ? *(const ulonglong2 *)(pts + (size_t)t * pt_words + off) : make_ulonglong2(0ull, 0ull);
    }
}

// a thread owns two neighbouring words (16 bytes per lane and access); grid x = blocks over N/2 pairs
__global__ __launch_bounds__(EW_THREADS) void plain_mac_kernel(const u64d *cts, int n_ct, const u64d *pts, int n_pts, const int *term, int n_groups,
                                                               u64d *out, const ModConst *modc, int logN, int level) {
    const size_t N = (size_t)1 << logN;
    const size_t w = 2 * ((size_t)blockIdx.x * EW_THREADS + threadIdx.x);
    if (w >= N) return;
    const int i = (int)blockIdx.y, g0 = (int)blockIdx.z * PM_GROUPS;
    const ModConst mc = modc[i];
    const size_t ct_words = 2 * (size_t)level * N, pt_words = (size_t)level * N, off = (size_t)i * N + w;
    double a0[PM_GROUPS][2], a1[PM_GROUPS][2];
#pragma unroll
    for (int k = 0; k < PM_GROUPS; k++) a0[k][0] = a0[k][1] = a1[k][0] = a1[k][1] = 0.0;
    // the words of source sct + 1 are requested before the products of source sct, so that their latency (table entry,
    // then plaintext word) lies under arithmetic; an absent term is a product with 0
    ulonglong2 xn0 = make_ulonglong2(0ull, 0ull), xn1 = xn0, yn[PM_GROUPS];
    if (n_ct > 0) plain_mac_fetch(cts, pts, term, 0, n_ct, n_pts, n_groups, g0, ct_words, pt_words, off, xn0, xn1, yn);
    for (int sct = 0; sct < n_ct; sct++) {
        const double x0[2] = {u2d(xn0.x), u2d(xn0.y)}, x1[2] = {u2d(xn1.x), u2d(xn1.y)};
        double y[PM_GROUPS][2];
#pragma unroll
        for (int k = 0; k < PM_GROUPS; k++) {
            y[k][0] = u2d(yn[k].x);
            y[k][1] = u2d(yn[k].y);
        }
        if (sct + 1 < n_ct) plain_mac_fetch(cts, pts, term, sct + 1, n_ct, n_pts, n_groups, g0, ct_words, pt_words, off, xn0, xn1, yn);
#pragma unroll
        for (int k = 0; k < PM_GROUPS; k++) {
#pragma unroll
            for (int b = 0; b < 2; b++) {
                // a reduced sum (p/2 + 1) and two products (1.25p each) stay below 3p + 1 < 2^53
                a0[k][b] += mulmod(x0[b], y[k][b], mc.p, mc.pinv);
                a1[k][b] += mulmod(x1[b], y[k][b], mc.p, mc.pinv);
                if (sct & 1) {
                    a0[k][b] = reduce_balanced(a0[k][b], mc.p, mc.pinv);
                    a1[k][b] = reduce_balanced(a1[k][b], mc.p, mc.pinv);
                }
            }
        }
    }
#pragma unroll
    for (int k = 0; k < PM_GROUPS; k++) {
        if (g0 + k >= n_groups) continue;
        u64d *o = out + (size_t)(g0 + k) * ct_words + off;
        *(ulonglong2 *)o = make_ulonglong2(d2u(canon(a0[k][0], mc.p, mc.pinv)), d2u(canon(a0[k][1], mc.p, mc.pinv)));
        *(ulonglong2 *)(o + pt_words) = make_ulonglong2(d2u(canon(a1[k][0], mc.p, mc.pinv)), d2u(canon(a1[k][1], mc.p, mc.pinv)));
    }
}

__global__ __launch_bounds__(EW_THREADS) void mul_scalar_kernel(const u64d *a, u64d *out, const ModConst *modc, ScalarTab S,
                                                                int logN, int level, size_t total) {
    size_t w = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (w >= total) return;
    const int i = (int)((w >> logN) % level);
    const ModConst mc = modc[i];
    out[w] = d2u(canon(mulmod_w(u2d(a[w]), S.c[i].w, S.c[i].wp, mc.p), mc.p, mc.pinv));
}

// out = a, plus the constant on component 0
__global__ __launch_bounds__(EW_THREADS) void add_const_kernel(const u64d *a, u64d *out, const ModConst *modc, ScalarTab S,
                                                               int logN, int level, size_t total) {
    size_t w = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (w >= total) return;
    const size_t limb = w >> logN;
    const int i = (int)(limb % level);
    u64d x = a[w];
    if ((limb / level) % 2 == 0) {
        const u64d q = (u64d)modc[i].p, c = (u64d)S.cpos[i];
        x = (x + c >= q) ? x + c - q : x + c;
    }
    out[w] = x;
}

// rows of level_in limbs -> rows of level_out limbs (first limbs kept)
__global__ __launch_bounds__(EW_THREADS) void mod_drop_kernel(const u64d *a, u64d *out, int logN, int level_in, int level_out,
                                                              size_t total_out) {
    size_t w = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (w >= total_out) return;
    const size_t N = (size_t)1 << logN;
    const size_t limb = w >> logN, row = limb / level_out, i = limb % level_out;
    out[w] = a[(row * level_in + i) * N + (w & (N - 1))];
}

// d = (a0*b0, a0*b1 + a1*b0, a1*b1); a, b: [batch][2][level][N], d: [batch][3][level][N].
// One thread per pair of adjacent words (16 bytes per lane and memory instruction); total = batch*level*N/2 pairs.
__device__ __forceinline__ void tensor_word(double a0, double a1, double b0, double b1, const ModConst &mc, u64d &d0, u64d &d1, u64d &d2) {
    d0 = d2u(canon(mulmod(a0, b0, mc.p, mc.pinv), mc.p, mc.pinv));
    d1 = d2u(canon(mulmod(a0, b1, mc.p, mc.pinv) + mulmod(a1, b0, mc.p, mc.pinv), mc.p, mc.pinv));
    d2 = d2u(canon(mulmod(a1, b1, mc.p, mc.pinv), mc.p, mc.pinv));
}
// terms > 1: d = sum over t of the tensors of (a_t, b_t), items laid out [batch][terms][2][level][N] (lazy relinearisation)
__device__ __forceinline__ void tensor_accumulate(u64d &acc, u64d v, double p) {
    const double s = u2d(acc) + u2d(v);
    acc = d2u(s >= p ? s - p : s);
}
__global__ __launch_bounds__(EW_THREADS) void tensor_kernel(const u64d *a, const u64d *b, u64d *d, const ModConst *modc, int logN,
                                                            int level, size_t total /* batch*level*N/2 */, int terms) {
    const size_t pr = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (pr >= total) return;
    const size_t N = (size_t)1 << logN, w = 2 * pr;
    const size_t limb = w >> logN, item = limb / level, i = limb % level, n = w & (N - 1);
    const ModConst mc = modc[i];
    const size_t st = (size_t)level * N;
    ulonglong2 D0, D1, D2;
    for (int t = 0; t < terms; t++) {
        const size_t ia = ((item * terms + t) * 2 * level + i) * N + n;
        const ulonglong2 A0 = *(const ulonglong2 *)(a + ia), A1 = *(const ulonglong2 *)(a + ia + st);
        const ulonglong2 B0 = *(const ulonglong2 *)(b + ia), B1 = *(const ulonglong2 *)(b + ia + st);
        ulonglong2 T0, T1, T2;
        tensor_word(u2d(A0.x), u2d(A1.x), u2d(B0.x), u2d(B1.x), mc, T0.x, T1.x, T2.x);
        tensor_word(u2d(A0.y), u2d(A1.y), u2d(B0.y), u2d(B1.y), mc, T0.y, T1.y, T2.y);
        if (t == 0) {
            D0 = T0; D1 = T1; D2 = T2;
        } else {
            tensor_accumulate(D0.x, T0.x, mc.p); tensor_accumulate(D0.y, T0.y, mc.p);
            tensor_accumulate(D1.x, T1.x, mc.p); tensor_accumulate(D1.y, T1.y, mc.p);
            tensor_accumulate(D2.x, T2.x, mc.p); tensor_accumulate(D2.y, T2.y, mc.p);
        }
    }
    const size_t id = (item * 3 * level + i) * N + n;
    *(ulonglong2 *)(d + id) = D0;
    *(ulonglong2 *)(d + id + st) = D1;
    *(ulonglong2 *)(d + id + 2 * st) = D2;
}

// Evaluation-form automorphism X -> X^g: out[j] = in[pi(j)],
// pi(j) = brev(((2*brev(j)+1)*g mod 2N - 1)/2).  Rows = (item, comp, limb); g per item.
struct GaloisTab { unsigned g[CKKSMI_MAX_ITEMS]; };

__global__ __launch_bounds__(EW_THREADS) void automorphism_kernel(const u64d *in, u64d *out, GaloisTab G, int logN, int limbs_per_item,
                                                                  size_t total) {
    size_t w = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (w >= total) return;
    const unsigned N = 1u << logN;
    const size_t limb = w >> logN;
    const unsigned j = (unsigned)(w & (N - 1));
    const unsigned g = G.g[limb / limbs_per_item];
    const unsigned bj = __brev(j) >> (32 - logN);
    const unsigned e = ((2u * bj + 1u) * g) & (2u * N - 1u);
    const unsigned src = __brev((e - 1u) >> 1) >> (32 - logN);
    out[w] = in[limb * N + src];
}

// ---------------------------------------------------------------- key switching
// ModUp of one item's polynomial d (coefficient form, [level][N]) into the extended
// basis for every digit: out [beta][E][N].  Limbs that belong to the digit are copied
// from the evaluation-form source (they need no transform).
struct ModUpArgs {
    const u64d *d_coef;      // [items][level][N]
    const u64d *d_eval;      // evaluation-form source of the same polynomial
    unsigned long long d_eval_item_stride;
    u64d *out;               // [items][beta][E][N]
    const ModConst *modc;
    const WMul *inv;         // [beta_top][alpha][alpha]
    const WMul *cc;          // [beta_top][alpha][alpha][T]
    int logN, level, E, n_q, alpha, beta, T;
};

__global__ __launch_bounds__(EW_THREADS) void modup_kernel(ModUpArgs A) {
    const unsigned N = 1u << A.logN;
    const unsigned n = blockIdx.x * EW_THREADS + threadIdx.x;
    if (n >= N) return;
    const unsigned j = blockIdx.y, item = blockIdx.z;
    const int lo = (int)j * A.alpha;
    const int nd = (A.level - lo < A.alpha) ? A.level - lo : A.alpha;
    const size_t row = ((size_t)j * A.alpha + (nd - 1)) * A.alpha;
    const u64d *dc = A.d_coef + (size_t)item * A.level * N;
    const u64d *de = A.d_eval + (size_t)item * A.d_eval_item_stride;
    u64d *out = A.out + ((size_t)item * A.beta + j) * A.E * N;
    double y[CKKSMI_MAX_ALPHA];
    for (int a = 0; a < nd; a++) {
        const ModConst mc = A.modc[lo + a];
        const WMul W = A.inv[row + a];
        // canonical representative in [0, q): the integer sum_a y_a*qhat_a is what gets reduced
        y[a] = canon(mulmod_w(u2d(dc[(size_t)(lo + a) * N + n]), W.w, W.wp, mc.p), mc.p, mc.pinv);
    }
    for (int x = 0; x < A.E; x++) {
        if (x >= lo && x < lo + nd) {
            out[(size_t)x * N + n] = de[(size_t)x * N + n];
            continue;
        }
        const int t = x < A.level ? x : A.n_q + x - A.level;
        const ModConst mc = A.modc[t];
        double acc = 0.0;
        for (int a = 0; a < nd; a++) {
            const WMul W = A.cc[(row + a) * A.T + t];
            acc += mulmod_w(y[a], W.w, W.wp, mc.p);
        }
        out[(size_t)x * N + n] = d2u(canon(acc, mc.p, mc.pinv));
    }
}

// acc_c[x] = sum_j dt_j[x] * key_j,c[T(x)]   (evaluation form, extended basis)
struct KeyTab {
    const u64d *key[CKKSMI_MAX_KEYS];
    unsigned char slot[CKKSMI_MAX_ITEMS];
};

struct InnerArgs {
    const u64d *dt;  // [items][beta][E][N]
    const u64d *d_eval;  // optional: when set, the limbs that belong to a digit are read from here (item i at + i*stride, [level][N])
    unsigned long long d_eval_item_stride;
    int alpha;
    u64d *acc;       // [items][2][E][N]
    const ModConst *modc;
    int logN, level, E, n_q, beta, T;
    int items, items_per_z;
};

// grid: x = word block, y = extended limb, z = chunk of items.  A thread keeps the key words of its
// position (2*beta values) in registers and loops over the items of its chunk, so the key is read
// once per chunk instead of once per item.
#define INNER_MAX_BETA 16
template <int BETA>
__device__ __forceinline__ void inner_product_body(const InnerArgs &A, const KeyTab &K) {
    const unsigned N = 1u << A.logN;
    const unsigned n = blockIdx.x * EW_THREADS + threadIdx.x;
    if (n >= N) return;
    const unsigned x = blockIdx.y;
    const int t = (int)x < A.level ? (int)x : A.n_q + (int)x - A.level;
    const ModConst mc = A.modc[t];
    const unsigned i0 = blockIdx.z * (unsigned)A.items_per_z;
    const unsigned i1 = (i0 + A.items_per_z < (unsigned)A.items) ? i0 + A.items_per_z : (unsigned)A.items;
    const u64d *key_loaded = nullptr;
    double k0[BETA], k1[BETA];
    for (unsigned item = i0; item < i1; item++) {
        const u64d *key = K.key[K.slot[item]];
        if (key != key_loaded) {  // uniform across the workgroup
#pragma unroll
            for (int j = 0; j < BETA; j++) {
                k0[j] = u2d(key[(((size_t)j * 2 + 0) * A.T + t) * N + n]);
                k1[j] = u2d(key[(((size_t)j * 2 + 1) * A.T + t) * N + n]);
            }
            key_loaded = key;
        }
        double v[BETA];
#pragma unroll
        for (int j = 0; j < BETA; j++) {
            const bool own = A.d_eval && (int)x < A.level && (int)x / A.alpha == j;
            v[j] = own ? u2d(A.d_eval[(size_t)item * A.d_eval_item_stride + (size_t)x * N + n])
                       : u2d(A.dt[(((size_t)item * BETA + j) * A.E + x) * N + n]);
        }
        double a0 = 0.0, a1 = 0.0;
#pragma unroll
        for (int j = 0; j < BETA; j++) {
            a0 = reduce_balanced(a0 + mulmod(v[j], k0[j], mc.p, mc.pinv), mc.p, mc.pinv);
            a1 = reduce_balanced(a1 + mulmod(v[j], k1[j], mc.p, mc.pinv), mc.p, mc.pinv);
        }
        A.acc[(((size_t)item * 2 + 0) * A.E + x) * N + n] = d2u(canon_small(a0, mc.p));
        A.acc[(((size_t)item * 2 + 1) * A.E + x) * N + n] = d2u(canon_small(a1, mc.p));
    }
}

// any number of digits: no key caching
__device__ __forceinline__ void inner_product_generic(const InnerArgs &A, const KeyTab &K) {
    const unsigned N = 1u << A.logN;
    const unsigned n = blockIdx.x * EW_THREADS + threadIdx.x;
    if (n >= N) return;
    const unsigned x = blockIdx.y;
    const int t = (int)x < A.level ? (int)x : A.n_q + (int)x - A.level;
    const ModConst mc = A.modc[t];
    const unsigned i0 = blockIdx.z * (unsigned)A.items_per_z;
    const unsigned i1 = (i0 + A.items_per_z < (unsigned)A.items) ? i0 + A.items_per_z : (unsigned)A.items;
    for (unsigned item = i0; item < i1; item++) {
        const u64d *key = K.key[K.slot[item]];
        double a0 = 0.0, a1 = 0.0;
        for (int j = 0; j < A.beta; j++) {
            const bool own = A.d_eval && (int)x < A.level && (int)x / A.alpha == j;
            const double v = own ? u2d(A.d_eval[(size_t)item * A.d_eval_item_stride + (size_t)x * N + n])
                                 : u2d(A.dt[(((size_t)item * A.beta + j) * A.E + x) * N + n]);
            const double k0 = u2d(key[(((size_t)j * 2 + 0) * A.T + t) * N + n]);
            const double k1 = u2d(key[(((size_t)j * 2 + 1) * A.T + t) * N + n]);
            a0 = reduce_balanced(a0 + mulmod(v, k0, mc.p, mc.pinv), mc.p, mc.pinv);
            a1 = reduce_balanced(a1 + mulmod(v, k1, mc.p, mc.pinv), mc.p, mc.pinv);
        }
        A.acc[(((size_t)item * 2 + 0) * A.E + x) * N + n] = d2u(canon_small(a0, mc.p));
        A.acc[(((size_t)item * 2 + 1) * A.E + x) * N + n] = d2u(canon_small(a1, mc.p));
    }
}

__global__ __launch_bounds__(EW_THREADS) void inner_product_kernel(InnerArgs A, KeyTab K) {
    switch (A.beta) {
        case 1: inner_product_body<1>(A, K); break;
        case 2: inner_product_body<2>(A, K); break;
        case 3: inner_product_body<3>(A, K); break;
        case 4: inner_product_body<4>(A, K); break;
        case 5: inner_product_body<5>(A, K); break;
        case 6: inner_product_body<6>(A, K); break;
        case 7: inner_product_body<7>(A, K); break;
        case 8: inner_product_body<8>(A, K); break;
        case 9: inner_product_body<9>(A, K); break;
        case 10: inner_product_body<10>(A, K); break;
        case 11: inner_product_body<11>(A, K); break;
        case 12: inner_product_body<12>(A, K); break;
        case 13: inner_product_body<13>(A, K); break;
        case 14: inner_product_body<14>(A, K); break;
        case 15: inner_product_body<15>(A, K); break;
        case 16: inner_product_body<16>(A, K); break;
        default: inner_product_generic(A, K); break;
    }
}

// ---------------------------------------------------------------- DivRound
// Rows = (item, component).  Step 1 (coefficient form): from the nb dropped limbs of a
// row compute, for each kept limb i, r_i - h where r_i = [(x + h) mod Bbar] mod c_i by fast
// basis conversion.  Step 2 (evaluation form, after transforming step 1's output):
// out_i = (x_i - NTT(r_i - h)) * Bbar^-1 mod c_i, optionally + addend_i.
struct DivConvArgs {
    const u64d *b_limbs;  // dropped limbs, coefficient form: row r, limb m at b_limbs + r*b_row_stride + m*N
    unsigned long long b_row_stride;
    u64d *tmp;            // [rows][nc][N]
    const ModConst *modc;
    DivRoundDev D;
    int logN, nc, T;      // kept limbs are modulus indices 0 .. nc-1
    int exact;            // 1: the conversion's overshoot v = floor(sum_m y_m * (1/b_m)) (doubles, in this order) is removed
};

__global__ __launch_bounds__(EW_THREADS) void divround_conv_kernel(DivConvArgs A) {
    const unsigned N = 1u << A.logN;
    const unsigned n = blockIdx.x * EW_THREADS + threadIdx.x;
    if (n >= N) return;
    const unsigned row = blockIdx.y;
    double y[CKKSMI_MAX_SPECIAL];
    for (int m = 0; m < A.D.nb; m++) {
        const ModConst mc = A.modc[A.D.b_idx[m]];
        double x = u2d(A.b_limbs[(size_t)row * A.b_row_stride + (size_t)m * N + n]) + A.D.hb[m];
        x = x >= mc.p ? x - mc.p : x;
        y[m] = canon(mulmod_w(x, A.D.invb[m].w, A.D.invb[m].wp, mc.p), mc.p, mc.pinv);
    }
    double v = 0.0;
    if (A.exact) {
        double sum = y[0] * A.D.invb_f[0];
        for (int m = 1; m < A.D.nb; m++) sum = sum + y[m] * A.D.invb_f[m];
        v = floor(sum);
    }
    for (int i = 0; i < A.nc; i++) {
        const ModConst mc = A.modc[i];
        double acc = -A.D.hc[i];
        if (A.exact) acc = -reduce_balanced(A.D.hc[i] + v * A.D.Bmod[i], mc.p, mc.pinv);  // v <= nb - 1: exact product
        for (int m = 0; m < A.D.nb; m++) {
            const WMul W = A.D.conv[(size_t)m * A.T + i];
            acc += mulmod_w(y[m], W.w, W.wp, mc.p);
        }
        A.tmp[((size_t)row * A.nc + i) * N + n] = d2u(canon(acc, mc.p, mc.pinv));
    }
}

struct DivFinalArgs {
    const u64d *x;       // kept limbs, evaluation form: row r, limb i at x + r*x_row_stride + i*N
    unsigned long long x_row_stride;
    const u64d *tmp;     // [rows][nc][N] evaluation form
    const u64d *addend;  // optional, row r limb i at addend + (r/2)*add_item_stride + (r%2)*add_comp_stride + i*N
    unsigned long long add_item_stride, add_comp_stride;
    int add_both;        // 1: both components receive the addend, 0: component 0 only
    u64d *out;           // [rows][nc][N]
    const ModConst *modc;
    const WMul *Binv;    // [T]
    const WMul *pre;     // optional [T]: the addend enters BEFORE the division, out = (x + pre_i*addend - r) * Binv
    int logN, nc;
};

__global__ __launch_bounds__(EW_THREADS) void divround_final_kernel(DivFinalArgs A) {
    const unsigned N = 1u << A.logN;
    const unsigned n = blockIdx.x * EW_THREADS + threadIdx.x;
    if (n >= N) return;
    const unsigned i = blockIdx.y, row = blockIdx.z;
    const ModConst mc = A.modc[i];
    const WMul W = A.Binv[i];
    double x = u2d(A.x[(size_t)row * A.x_row_stride + (size_t)i * N + n]);
    double r = u2d(A.tmp[((size_t)row * A.nc + i) * N + n]);
    if (A.pre) {
        const WMul Pm = A.pre[i];
        const double ad = u2d(A.addend[(size_t)(row / 2) * A.add_item_stride + (size_t)(row % 2) * A.add_comp_stride + (size_t)i * N + n]);
        x += mulmod_w(ad, Pm.w, Pm.wp, mc.p);
    }
    double v = canon(mulmod_w(x - r, W.w, W.wp, mc.p), mc.p, mc.pinv);
    if (!A.pre && A.addend && (A.add_both || (row & 1u) == 0)) {
        v += u2d(A.addend[(size_t)(row / 2) * A.add_item_stride + (size_t)(row % 2) * A.add_comp_stride + (size_t)i * N + n]);
        v = v >= mc.p ? v - mc.p : v;
    }
    A.out[((size_t)row * A.nc + i) * N + n] = d2u(v);
}

// x[row][n] = (wx * x[row][n] + w * a[row][n]) mod p on one limb of every row: row r of x at x + r*x_row_stride, of a at
// a + (r/2)*a_item_stride + (r%2)*a_comp_stride.  Two words per thread.
__global__ __launch_bounds__(EW_THREADS) void axpy_limb_kernel(u64d *x, unsigned long long x_row_stride, const u64d *a,
                                                               unsigned long long a_item_stride, unsigned long long a_comp_stride, ModConst mc,
                                                               WMul wx, WMul w, int logN) {
    const unsigned pairs = 1u << (logN - 1);
    const unsigned n = blockIdx.x * EW_THREADS + threadIdx.x;
    if (n >= pairs) return;
    const unsigned row = blockIdx.y;
    ulonglong2 *xp = (ulonglong2 *)(x + (size_t)row * x_row_stride) + n;
    const ulonglong2 av = ((const ulonglong2 *)(a + (size_t)(row / 2) * a_item_stride + (size_t)(row % 2) * a_comp_stride))[n];
    ulonglong2 xv = *xp;
    xv.x = d2u(canon(mulmod_w(u2d(xv.x), wx.w, wx.wp, mc.p) + mulmod_w(u2d(av.x), w.w, w.wp, mc.p), mc.p, mc.pinv));
    xv.y = d2u(canon(mulmod_w(u2d(xv.y), wx.w, wx.wp, mc.p) + mulmod_w(u2d(av.y), w.w, w.wp, mc.p), mc.p, mc.pinv));
    *xp = xv;
}

// out[row][i] = a[row][i] + b[row][i] for rows of `level` limbs where only component 0
// rows (even rows) receive the addend; used by rotation: (sigma(c0) + ks0, ks1)
// is produced directly by divround_final's addend with add_comp_stride, so no kernel here.

// ---------------------------------------------------------------- rotations with a shared ModUp
// R rotations of each item from ONE lifted decomposition dt of its second component: rotation r applies its
// automorphism to the lifted digits on the fly (a gather: out word m takes word pi_r(m)) and multiplies by its own key,
//     acc[item][r][c][x][m] = sum_j dt[item][j][x][pi_r(m)] * key_r[j][c][x][m].
// The permutation keeps the high bits of a word index among themselves (the low bits of brev), so the 256 outputs of
// a workgroup gather from one 256-word run of the source: the gather is local to cache lines the workgroup uses up.
struct HoistArgs {
    const u64d *dt;      // [items][beta][E][N] evaluation form
    const u64d *d_eval;  // optional: limbs that belong to a digit are read from here (item i at + i*stride, [level][N])
    unsigned long long d_eval_item_stride;
    u64d *acc;           // [items][R][2][E][N]
    const ModConst *modc;
    int logN, level, E, n_q, alpha, beta, T;
    int items, R;
    int items_per_wg;                  // tile kernel: items whose source rows share the workgroup's LDS
    int rots_per_wg, item_chunks;      // tile kernel: grid z = item chunk + item_chunks * rotation chunk
    unsigned g[CKKSMI_MAX_KEYS];
    unsigned ginv[CKKSMI_MAX_KEYS];    // g^-1 mod 2N
    const u64d *key[CKKSMI_MAX_KEYS];
};

__device__ __forceinline__ unsigned automorphism_source(unsigned j, unsigned g, int logN) {
    const unsigned N = 1u << logN;
    const unsigned bj = __brev(j) >> (32 - logN);
    const unsigned e = ((2u * bj + 1u) * g) & (2u * N - 1u);
    return __brev((e - 1u) >> 1) >> (32 - logN);
}

// The automorphism seen from the row-pair layout of the register-tiled kernels.  j and j + 1 (j even) differ in the top
// bit of brev(j), so their sources differ in the lowest bit only: the two words of a result pair are the two words of ONE
// source pair, in either order.  The low eight bits of j reach only the low eight bits of the source: a 256-word row comes
// from one source row, and 32 neighbouring words of it from 32 neighbouring words.  A kernel that reads rows in pairs can
// therefore read THROUGH the automorphism with the same 16-byte accesses and the same cache lines per instruction.
__device__ __forceinline__ ulonglong2 galois_pair_load(const u64d *limb, unsigned j_even, unsigned g, int logN) {
    const unsigned src = automorphism_source(j_even, g, logN);
    const ulonglong2 v = ((const ulonglong2 *)limb)[src >> 1];
    return (src & 1u) ? make_ulonglong2(v.y, v.x) : v;
}

// grid: x = word block, y = extended limb, z = rotation
__global__ __launch_bounds__(EW_THREADS) void inner_product_hoisted_kernel(HoistArgs A) {
    const unsigned N = 1u << A.logN;
    const unsigned m = blockIdx.x * EW_THREADS + threadIdx.x;
    if (m >= N) return;
    const unsigned x = blockIdx.y, r = blockIdx.z;
    const int t = (int)x < A.level ? (int)x : A.n_q + (int)x - A.level;
    const ModConst mc = A.modc[t];
    const unsigned src = automorphism_source(m, A.g[r], A.logN);
    const u64d *key = A.key[r];
    const int j_own = (A.d_eval && (int)x < A.level) ? (int)x / A.alpha : -1;
    if (A.beta <= INNER_MAX_BETA) {
        // the key words of this position stay in registers over the items
        double k0[INNER_MAX_BETA], k1[INNER_MAX_BETA];
#pragma unroll
        for (int j = 0; j < INNER_MAX_BETA; j++)
            if (j < A.beta) {
                k0[j] = u2d(key[(((size_t)j * 2 + 0) * A.T + t) * N + m]);
                k1[j] = u2d(key[(((size_t)j * 2 + 1) * A.T + t) * N + m]);
            }
        for (int item = 0; item < A.items; item++) {
            double v[INNER_MAX_BETA];
#pragma unroll
            for (int j = 0; j < INNER_MAX_BETA; j++)
                if (j < A.beta)
                    v[j] = j == j_own ? u2d(A.d_eval[(size_t)item * A.d_eval_item_stride + (size_t)x * N + src])
                                      : u2d(A.dt[(((size_t)item * A.beta + j) * A.E + x) * N + src]);
            double a0 = 0.0, a1 = 0.0;
#pragma unroll
            for (int j = 0; j < INNER_MAX_BETA; j++)
                if (j < A.beta) {
                    a0 = reduce_balanced(a0 + mulmod(v[j], k0[j], mc.p, mc.pinv), mc.p, mc.pinv);
                    a1 = reduce_balanced(a1 + mulmod(v[j], k1[j], mc.p, mc.pinv), mc.p, mc.pinv);
                }
            const size_t row = ((size_t)item * A.R + r) * 2;
            A.acc[((row + 0) * A.E + x) * N + m] = d2u(canon_small(a0, mc.p));
            A.acc[((row + 1) * A.E + x) * N + m] = d2u(canon_small(a1, mc.p));
        }
        return;
    }
    for (int item = 0; item < A.items; item++) {
        double a0 = 0.0, a1 = 0.0;
        for (int j = 0; j < A.beta; j++) {
            const double v = j == j_own ? u2d(A.d_eval[(size_t)item * A.d_eval_item_stride + (size_t)x * N + src])
                                        : u2d(A.dt[(((size_t)item * A.beta + j) * A.E + x) * N + src]);
            const double k0 = u2d(key[(((size_t)j * 2 + 0) * A.T + t) * N + m]);
            const double k1 = u2d(key[(((size_t)j * 2 + 1) * A.T + t) * N + m]);
            a0 = reduce_balanced(a0 + mulmod(v, k0, mc.p, mc.pinv), mc.p, mc.pinv);
            a1 = reduce_balanced(a1 + mulmod(v, k1, mc.p, mc.pinv), mc.p, mc.pinv);
        }
        const size_t row = ((size_t)item * A.R + r) * 2;
        A.acc[((row + 0) * A.E + x) * N + m] = d2u(canon_small(a0, mc.p));
        A.acc[((row + 1) * A.E + x) * N + m] = d2u(canon_small(a1, mc.p));
    }
}

// The same sums organised around the SOURCE: a workgroup stages one 256-word run of every lifted digit of a few items
// in LDS (read from HBM once for all rotations), then walks the rotations: rotation r sends this run to exactly one
// 256-word run of its output (found through the inverse automorphism), gathered out of LDS.
// Words travel in pairs: an output pair (2m, 2m + 1) is one source pair, possibly with its words exchanged (see
// galois_pair_load), so key words, staged words and results all move 16 bytes per lane.  The first 128 threads form the
// first component's sums, the other 128 the second's (each key word is read once).
#define HOIST_LDS_WORDS 8192  // 64 KiB: items_per_wg * beta * 256 words at most
// LW: words of LDS, the smallest of 1024 .. HOIST_LDS_WORDS that holds the staged rows (few items: more workgroups per
// compute unit, whose dependent key reads then overlap); MB: bound on the number of digits (4, 8 or INNER_MAX_BETA), which
// sizes the registers that hold a rotation's key words
// grid: x = source run (N/256), y = extended limb, z = (chunk of items_per_wg items, chunk of rots_per_wg rotations)
template <int LW, int MB>
__global__ __launch_bounds__(EW_THREADS) void inner_product_hoisted_tile_kernel(HoistArgs A) {
    __shared__ double tile[LW];
    const unsigned N = 1u << A.logN;
    const unsigned tid = threadIdx.x, pr = tid & 127u, comp = tid >> 7, src0 = blockIdx.x * 256u, x = blockIdx.y;
    const int t = (int)x < A.level ? (int)x : A.n_q + (int)x - A.level;
    const ModConst mc = A.modc[t];
    const int j_own = (A.d_eval && (int)x < A.level) ? (int)x / A.alpha : -1;
    const int item0 = (int)(blockIdx.z % (unsigned)A.item_chunks) * A.items_per_wg;
    const int r_begin = (int)(blockIdx.z / (unsigned)A.item_chunks) * A.rots_per_wg;
    const int r_end = r_begin + A.rots_per_wg < A.R ? r_begin + A.rots_per_wg : A.R;
    const int n_items = (item0 + A.items_per_wg < A.items ? item0 + A.items_per_wg : A.items) - item0;
    {
        // the staged rows (item, digit), at most LW / 256 of them: the two halves of the workgroup take
        // them in turn, all of a half's rows requested together (a load per iteration followed by its LDS write would
        // serialise them)
        const int n_rows = n_items * A.beta;
        ulonglong2 raw[LW / 512];
#pragma unroll
        for (int k = 0; k < LW / 512; k++) {
            const int q = 2 * k + (int)comp;
            if (q < n_rows) {
                const size_t item = (size_t)(item0 + q / A.beta);
                const int j = q % A.beta;
                const u64d *row = j == j_own ? A.d_eval + item * A.d_eval_item_stride + (size_t)x * N : A.dt + ((item * A.beta + j) * A.E + x) * N;
                raw[k] = ((const ulonglong2 *)(row + src0))[pr];
            }
        }
#pragma unroll
        for (int k = 0; k < LW / 512; k++) {
            const int q = 2 * k + (int)comp;
            if (q < n_rows) ((double2 *)(tile + q * 256))[pr] = make_double2(u2d(raw[k].x), u2d(raw[k].y));
        }
    }
    __syncthreads();
    // the key words of rotation r + 1 are requested before the sums of rotation r, so their latency is covered
    ulonglong2 kn[MB];
    unsigned m_next = (automorphism_source(src0, A.ginv[r_begin], A.logN) & ~255u) + 2u * pr;  // this run's image under the first rotation
#pragma unroll
    for (int j = 0; j < MB; j++)
        if (j < A.beta) kn[j] = *(const ulonglong2 *)(A.key[r_begin] + (((size_t)j * 2 + comp) * A.T + t) * N + m_next);
    for (int r = r_begin; r < r_end; r++) {
        const unsigned m = m_next;
        const unsigned s = automorphism_source(m, A.g[r], A.logN) - src0;  // below 256; the word after m comes from s ^ 1
        const bool swap = s & 1u;
        double k0[MB], k1[MB];
#pragma unroll
        for (int j = 0; j < MB; j++) {
            k0[j] = u2d(kn[j].x);
            k1[j] = u2d(kn[j].y);
        }
        if (r + 1 < r_end) {
            m_next = (automorphism_source(src0, A.ginv[r + 1], A.logN) & ~255u) + 2u * pr;
            const u64d *key = A.key[r + 1];
#pragma unroll
            for (int j = 0; j < MB; j++)
                if (j < A.beta) kn[j] = *(const ulonglong2 *)(key + (((size_t)j * 2 + comp) * A.T + t) * N + m_next);
        }
        for (int ii = 0; ii < n_items; ii++) {
            double a0 = 0.0, a1 = 0.0;  // the sums of the words m and m + 1
#pragma unroll
            for (int j = 0; j < MB; j++)
                if (j < A.beta) {
                    const double2 vv = *(const double2 *)(tile + (ii * A.beta + j) * 256 + (s & ~1u));
                    const double v0 = swap ? vv.y : vv.x, v1 = swap ? vv.x : vv.y;
                    // a reduced sum (p/2 + 1) and two products (1.25p each) stay below 3p + 1 < 2^53
                    a0 += mulmod(v0, k0[j], mc.p, mc.pinv);
                    a1 += mulmod(v1, k1[j], mc.p, mc.pinv);
                    if (j & 1) {
                        a0 = reduce_balanced(a0, mc.p, mc.pinv);
                        a1 = reduce_balanced(a1, mc.p, mc.pinv);
                    }
                }
            if (A.beta & 1) {
                a0 = reduce_balanced(a0, mc.p, mc.pinv);
                a1 = reduce_balanced(a1, mc.p, mc.pinv);
            }
            const size_t row = ((size_t)(item0 + ii) * A.R + r) * 2 + comp;
            *(ulonglong2 *)(A.acc + (row * A.E + x) * N + m) = make_ulonglong2(d2u(canon_small(a0, mc.p)), d2u(canon_small(a1, mc.p)));
        }
    }
}

// sigma_r of the first component of every item, for every rotation: out[item][r][i][m] = in[item][i][pi_r(m)]
__global__ __launch_bounds__(EW_THREADS) void automorphism_bcast_kernel(const u64d *in, unsigned long long in_item_stride, u64d *out,
                                                                        HoistArgs A, size_t total) {
    const size_t w = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (w >= total) return;
    const unsigned N = 1u << A.logN;
    const size_t row = w >> A.logN;
    const unsigned m = (unsigned)(w & (N - 1));
    const unsigned i = (unsigned)(row % (size_t)A.level);
    const size_t ir = row / (size_t)A.level;
    const unsigned r = (unsigned)(ir % (size_t)A.R);
    const size_t item = ir / (size_t)A.R;
    out[w] = in[item * in_item_stride + (size_t)i * N + automorphism_source(m, A.g[r], A.logN)];
}

// ---------------------------------------------------------------- conv / FC multiply-accumulate
// Weights prepared per limb: wtab[i][widx] = (w mod q_i balanced, that / q_i)
__global__ __launch_bounds__(EW_THREADS) void mac_prepare_kernel(const long long *w, WMul *wtab, const ModConst *modc, int level,
                                                                 size_t n_weights) {
    size_t idx = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= n_weights * (size_t)level) return;
    const int i = (int)(idx / n_weights);
    const long long q = (long long)modc[i].p;
    long long r = w[idx % n_weights] % q;  // (-q, q)
    if (r > q / 2) r -= q;
    if (r < -(q / 2)) r += q;
    const double rb = (double)r;
    wtab[idx] = WMul{rb, rb / modc[i].p};
}

#define MAC_OC 32  // output channels accumulated per thread (each input word is loaded once per 32 outputs)

struct MacArgs {
    const u64d *in;   // [C][in_rows][W] ciphertexts of 2*level limbs: image rows in_row0 .. in_row0+in_rows-1
    u64d *out;        // [O][out_rows][Wo]: output rows out_row0 .. out_row0+out_rows-1
    const WMul *wtab; // [level][O*C*kh*kw]
    const ModConst *modc;
    int logN, level;
    int C, H, W, O, kh, kw, stride, pad, Ho, Wo;
    int in_row0, in_rows, out_row0, out_rows;
};

// grid: x = out_rows*Wo*ceil(O/MAC_OC) (fastest: workgroups that share input words run together), y = N / EW_THREADS,
// z = 2*level (component-major limb)
__global__ __launch_bounds__(EW_THREADS) void conv_mac_kernel(MacArgs A) {
    const unsigned N = 1u << A.logN;
    const unsigned n = blockIdx.y * EW_THREADS + threadIdx.x;
    if (n >= N) return;
    const unsigned lc = blockIdx.z, i = lc % (unsigned)A.level;
    const unsigned ogroups = (unsigned)(A.O + MAC_OC - 1) / MAC_OC;
    const unsigned og = blockIdx.x % ogroups, pos = blockIdx.x / ogroups;
    const int oyl = (int)(pos / (unsigned)A.Wo), ox = (int)(pos % (unsigned)A.Wo);
    const int oy = A.out_row0 + oyl;
    const int o0 = (int)og * MAC_OC;
    const ModConst mc = A.modc[i];
    const size_t ctw = (size_t)2 * A.level * N;
    const size_t taps = (size_t)A.C * A.kh * A.kw;
    const WMul *wt = A.wtab + (size_t)i * A.O * taps;
    double acc[MAC_OC];
    for (int o = 0; o < MAC_OC; o++) acc[o] = 0.0;
    int pending = 0;
    for (int c = 0; c < A.C; c++)
        for (int u = 0; u < A.kh; u++)
            for (int v = 0; v < A.kw; v++) {
                const int iy = oy * A.stride + u - A.pad, ix = ox * A.stride + v - A.pad;
                if (iy < 0 || iy >= A.H || ix < 0 || ix >= A.W) continue;
                // the host has checked that every image row a tap can touch lies inside the strip
                const double xv = u2d(A.in[(((size_t)c * A.in_rows + (iy - A.in_row0)) * A.W + ix) * ctw + (size_t)lc * N + n]);
                const size_t tap = ((size_t)c * A.kh + u) * A.kw + v;
                for (int o = 0; o < MAC_OC; o++) {
                    if (o0 + o < A.O) {
                        const WMul Wt = wt[(size_t)(o0 + o) * taps + tap];
                        acc[o] += mulmod_w(xv, Wt.w, Wt.wp, mc.p);
                    }
                }
                if (++pending == 4) {  // each term is below 0.75p: four terms on a reduced value stay under 4p
                    for (int o = 0; o < MAC_OC; o++) acc[o] = reduce_balanced(acc[o], mc.p, mc.pinv);
                    pending = 0;
                }
            }
    for (int o = 0; o < MAC_OC; o++)
        if (o0 + o < A.O)
            A.out[((((size_t)(o0 + o) * A.out_rows + oyl) * A.Wo + ox) * ctw) + (size_t)lc * N + n] = d2u(canon(acc[o], mc.p, mc.pinv));
}

// k x k sum pooling of per-pixel ciphertexts over the image padded with `pad` zero rows / columns on every side:
// out[c][y][x] = sum_{u,v<k} in[c][k*y+u-pad][k*x+v-pad], word by word, positions outside the image skipped.
// one thread per output word; idx runs over [C*Ho*Wo][2*level][N]
__global__ __launch_bounds__(EW_THREADS) void sum_pool_kernel(const u64d *in, u64d *out, const ModConst *modc, int logN, int level, int H, int W,
                                                              int k, int pad, int Ho, int Wo, size_t total) {
    const size_t idx = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= total) return;
    const size_t N = (size_t)1 << logN, ctw = (size_t)2 * level * N;
    const size_t ct = idx / ctw, off = idx % ctw;
    const unsigned i = (unsigned)((off >> logN) % (unsigned)level);
    const u64d p = (u64d)modc[i].p;
    const size_t x = ct % Wo, y = (ct / Wo) % Ho, c = ct / ((size_t)Wo * Ho);
    u64d acc = 0;
    for (int u = 0; u < k; u++)
        for (int v = 0; v < k; v++) {
            const int iy = k * (int)y + u - pad, ix = k * (int)x + v - pad;
            if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
            acc += in[((c * H + (size_t)iy) * W + (size_t)ix) * ctw + off];
            acc = acc >= p ? acc - p : acc;
        }
    out[idx] = acc;
}

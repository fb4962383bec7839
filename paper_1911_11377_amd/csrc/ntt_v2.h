// Register-tiled limb transforms for N = N1 x 256, N1 = 16 .. 256 (2^12 <= N <= 2^16), gfx950.
//
// A transform of N = 2^logN points is split into a strided pass over columns (the first
// k = logN-8 stages, N1 = 2^k-point sub-transforms down the columns of the N1 x 256 matrix)
// and a contiguous pass over rows of 256 words (the last 8 stages).  In both, a workgroup of
// 256 threads works on a tile of 4096 words: every thread keeps 16 words in registers and does
// up to four butterfly stages on them without touching memory ("round"); one exchange through
// LDS regroups the words for the second round.
//
//   row pass   : tile = 16 rows.  A row is a 16x16 matrix M[a][b] (position 16a+b); round 1
//                (spans >= 16) works along a, round 2 (spans < 16) along b.
//   column pass: tile = N1 rows x C columns, C = 4096/N1.  With G = N1/16 = 2^Q: round 1 does the
//                first four stages on the rows {r + G*e}; round 2 does the remaining Q stages on
//                groups of G consecutive rows, a thread holding 16/G columns of one group.
//
// Twiddles: stage s of the whole transform multiplies block i by psi^brev(2^s + i).  For a thread
// they reduce to at most 15 values per round that depend only on the tile position and the lane,
// so they are loaded into registers once per workgroup and reused for every item the workgroup
// loops over (same modulus, same tile): twiddle traffic is amortised over the batch.
//
// Between the two passes the words are stored as balanced-reduced doubles (mid_store / mid_load), not as canonical
// integers: that intermediate never leaves the library.
//
// Lazy ranges (units of p, see device_arith.h): with the quotient w/p recomputed in registers a twiddle
// product of y is bounded by (1/2 + 1.5*|y|/2^53) p, so a butterfly stage maps a bound B to
// B + 1/2 + 1.5*B*p/2^53 forward and to 2B inverse; values must stay below 2^53, i.e. 8p for
// p < 2^50 and 4p for p < 2^51, so the reduction points differ (template parameter P51).
#pragma once
#include "device_arith.h"

#define V2_THREADS 256
#ifdef CKKSMI_EMULATE
#define NTT_SCHED_FENCE() ((void)0)
#else
#define NTT_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)
#endif
#define V2_GS 272  // doubles per padded 16x17 group in LDS (row pass)

// Row pass: the 16 lanes that work on one row of 256 words exchange their words through that row's own LDS group and
// nothing else, and 16 consecutive lanes always sit in one wavefront.  A wavefront's LDS instructions execute in program
// order, so these exchanges need no workgroup barrier: the fences only keep the compiler from moving LDS accesses across
// the exchange point.  (The CPU stand-in runs one thread at a time and needs a real barrier there.)
#ifdef CKKSMI_EMULATE
#define ROW_GROUP_SYNC() __syncthreads()
#else
#define ROW_GROUP_SYNC()                                        \
    do {                                                        \
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  \
        __builtin_amdgcn_wave_barrier();                        \
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");  \
    } while (0)
#endif

// Pointwise layout of the row-pass kernels: thread (hi4 = tid / 16, lo4 = tid % 16) owns the word pairs at columns
// 32*s + 2*lo4, +1 (s < 8) of row hi4 of the tile: 16 bytes per lane and memory instruction, 256 contiguous bytes per
// row and instruction, and every word of a row stays with the 16 lanes that transform that row.
__device__ __forceinline__ unsigned row_pair_index(unsigned hi4, unsigned lo4, int s) { return hi4 * 128u + 16u * s + lo4; }  // in 16-byte units from the tile
// the same pair in the row's LDS group (padded 16 x 17 doubles; word q of the row at (q / 16) * 17 + q % 16)
__device__ __forceinline__ unsigned row_pair_lds(unsigned lo4, int s) { return (2u * s + (lo4 >> 3)) * 17u + 2u * (lo4 & 7u); }

struct NttV2Args {
    const u64d *src;
    u64d *dst;
    const ModConst *modc;
    const double *tw;     // [T][N] twiddles of the direction, balanced representatives
    const WMul *tw_ninv;  // [T] inverse only: 1/N
    const WMul *tw_last;  // [T] inverse only: psi^-brev(1)/N
    const FinConst *fin;  // optional, inverse column pass: per limb slot, replaces the 1/N constants of the last stage
    int logN;
    int items, items_per_z;
    P51Mask p51;
    LimbMap map;
};

__device__ __forceinline__ void reduce16(double (&x)[16], double p, double pinv) {
#pragma unroll
    for (int e = 0; e < 16; e++) x[e] = reduce_balanced(x[e], p, pinv);
}

// decimation-in-time stages S0..3 of a 16-point round (spans 8 >> s over the register index);
// MASK bit s: reduce all words after stage s
template <int S0, int MASK>
__device__ __forceinline__ void fwd_stages(double (&x)[16], const double (&tw)[15], double p, double pinv) {
#pragma unroll
    for (int s = S0; s < 4; s++) {
        const int span = 8 >> s;
#pragma unroll
        for (int b = 0; b < (1 << s); b++) {
            // registers hold w only; w/p is recomputed per block (one multiply, within 3 ulp of w/p)
            const double Ww = tw[(1 << s) - 1 + b], Wp = Ww * pinv;
#pragma unroll
            for (int j = 0; j < span; j++) {
                const int lo = b * 2 * span + j, hi = lo + span;
                const double v = mulmod_w(x[hi], Ww, Wp, p);
                const double u = x[lo];
                x[lo] = u + v;
                x[hi] = u - v;
            }
        }
        if (MASK & (1 << s)) reduce16(x, p, pinv);
    }
}
template <int MASK>
__device__ __forceinline__ void fwd_round(double (&x)[16], const double (&tw)[15], double p, double pinv) {
    fwd_stages<0, MASK>(x, tw, p, pinv);
}

// the same stages undone, 3 down to S0 (spans 1,2,..); MASK bit k: reduce after the k-th executed
// stage; FINAL folds 1/N into the very last stage (s = 0) of the whole transform
template <int S0, int MASK, bool FINAL>
__device__ __forceinline__ void inv_stages(double (&x)[16], const double (&tw)[15], double p, double pinv, WMul ninv, WMul wlast) {
#pragma unroll
    for (int k = 0; k < 4 - S0; k++) {
        const int s = 3 - k, span = 8 >> s;
#pragma unroll
        for (int b = 0; b < (1 << s); b++) {
            const double Ww = tw[(1 << s) - 1 + b], Wp = Ww * pinv;
#pragma unroll
            for (int j = 0; j < span; j++) {
                const int lo = b * 2 * span + j, hi = lo + span;
                const double u = x[lo], v = x[hi];
                if (FINAL && s == 0) {
                    x[lo] = mulmod_w(u + v, ninv.w, ninv.wp, p);
                    x[hi] = mulmod_w(u - v, wlast.w, wlast.wp, p);
                } else {
                    x[lo] = u + v;
                    x[hi] = mulmod_w(u - v, Ww, Wp, p);
                }
            }
        }
        if (MASK & (1 << k)) reduce16(x, p, pinv);
    }
}
template <int MASK, bool FINAL>
__device__ __forceinline__ void inv_round(double (&x)[16], const double (&tw)[15], double p, double pinv, WMul ninv, WMul wlast) {
    inv_stages<0, MASK, FINAL>(x, tw, p, pinv, ninv, wlast);
}

// ------------------------------------------------------------------ row pass twiddles
// base1 = N1 + row; round 1 uses tw[(base1 << s) + b], round 2 (lane = the thread's a) tw[((16*base1 + lane) << s) + b]
__device__ __forceinline__ void load_twiddles(const double *tw, unsigned base1, unsigned lane, double (&tw1)[15], double (&tw2)[15]) {
#pragma unroll
    for (int s = 0; s < 4; s++)
#pragma unroll
        for (int b = 0; b < (1 << s); b++) {
            tw1[(1 << s) - 1 + b] = tw[(base1 << s) + b];
            tw2[(1 << s) - 1 + b] = tw[((16u * base1 + lane) << s) + b];
        }
}

// ------------------------------------------------------------------ column pass geometry
// Q = log2(N1/16).  Round 1: register e <-> row r + G*e, column c0 + c   (r = tid / C, c = tid % C).
// Round 2: register pp*G + g <-> row G*a + g, column c0 + l16 + 16*pp     (a = tid >> 4, l16 = tid & 15).
template <int Q>
struct ColsGeom {
    static constexpr unsigned G = 1u << Q, C = 256u >> Q, P = 16u >> Q;
    static constexpr int S0 = 4 - Q;  // first register stage of round 2
    unsigned r, c, a, l16, c0;
    __device__ __forceinline__ ColsGeom(unsigned tid, unsigned tile) : r(tid / C), c(tid % C), a(tid >> 4), l16(tid & 15), c0(tile * C) {}
    __device__ __forceinline__ size_t g1(int e) const { return (size_t)(r + G * e) * 256 + c0 + c; }                       // global, round-1 register e
    __device__ __forceinline__ size_t g2(int i) const { return (size_t)(G * a + (i % G)) * 256 + c0 + l16 + 16 * (i / G); }  // global, round-2 register i
    __device__ __forceinline__ unsigned l1(int e) const { return (r + G * e) * C + c; }                                    // LDS [N1][C]
    __device__ __forceinline__ unsigned l2(int i) const { return (G * a + (i % G)) * C + l16 + 16 * (i / G); }
};

// round 1: the first four stages, block b of stage s uses tw[2^s + b] (same for every thread);
// round 2: register stage s = S0 + u is transform stage 4 + u, block = a*2^u + (b mod 2^u)
template <int Q>
__device__ __forceinline__ void load_cols_twiddles(const double *tw, unsigned a, double (&tw1)[15], double (&tw2)[15]) {
#pragma unroll
    for (int s = 0; s < 4; s++)
#pragma unroll
        for (int b = 0; b < (1 << s); b++) {
            tw1[(1 << s) - 1 + b] = tw[(1u << s) + b];
            if (s >= 4 - Q) {
                const int u = s - (4 - Q);
                tw2[(1 << s) - 1 + b] = tw[(16u << u) + (a << u) + (b & ((1 << u) - 1))];
            } else {
                tw2[(1 << s) - 1 + b] = 0.0;
            }
        }
}

// lazy-range reduction points of the column pass (see header comment)
template <int Q, bool P51>
struct ColsMasks {
    static constexpr int F1 = P51 ? 0xA : 0x8;            // forward round 1 from canonical input, ends reduced
    static constexpr int F2 = (P51 && Q == 4) ? 0x2 : 0;  // forward round 2 (Q stages) from a reduced value
    // inverse round 2 (Q stages, executed first, canonical input); always followed by a reduction
    static constexpr int I1 = P51 ? (Q >= 3 ? 0x2 : 0) : (Q == 4 ? 0x4 : 0);
    static constexpr int I2 = P51 ? 0x2 : 0;              // inverse round 1 from a reduced value, last stage multiplies
};

// SMALL (forward only): the source is a polynomial with small signed coefficients, one int64 per coefficient and the same
// for every limb (item i at (const long long *)A.src + i * src_item_stride): its residues are the values themselves
template <bool INV, int Q, bool P51, bool SMALL = false>
__device__ __forceinline__ void ntt_v2_cols(const NttV2Args &A, double *lds, int t, unsigned li) {
    typedef ColsGeom<Q> Geo;
    typedef ColsMasks<Q, P51> Mk;
    const unsigned N = 1u << A.logN;
    const double p = A.modc[t].p, pinv = A.modc[t].pinv;
    const double *tw = A.tw + (size_t)t * N;
    const Geo geo(threadIdx.x, blockIdx.x);
    double tw1[15], tw2[15];
    load_cols_twiddles<Q>(tw, geo.a, tw1, tw2);
    WMul ninv = WMul{0.0, 0.0}, wlast = WMul{0.0, 0.0};
    double cadd = 0.0;
    if (INV) {
        ninv = A.tw_ninv[t];
        wlast = A.tw_last[t];
        if (A.fin) { ninv = A.fin[li].ninv; wlast = A.fin[li].wlast; cadd = A.fin[li].cadd; }
    }
    const unsigned i0 = blockIdx.z * (unsigned)A.items_per_z;
    const unsigned i1 = (i0 + A.items_per_z < (unsigned)A.items) ? i0 + A.items_per_z : (unsigned)A.items;
    for (unsigned it = i0; it < i1; it++) {
        const u64d *src = A.src + (size_t)it * A.map.src_item_stride + (size_t)li * N;
        u64d *dst = A.dst + (size_t)it * A.map.dst_item_stride + (size_t)li * N;
        double x[16];
        if (!INV) {
#pragma unroll
            for (int e = 0; e < 16; e++) {
                // magnitudes below 2^51: shifted to a non-negative integer, which becomes a double without a conversion
                // instruction (those issue at a quarter of the rate); the reduction brings it into the range of the first round
                if (SMALL) {
                    const long long v = ((const long long *)A.src + (size_t)it * A.map.src_item_stride)[geo.g1(e)];
                    x[e] = reduce_balanced(u2d((unsigned long long)(v + (1ll << 51))) - 2251799813685248.0, p, pinv);
                }
                else x[e] = u2d(src[geo.g1(e)]);
            }
            fwd_round<Mk::F1>(x, tw1, p, pinv);
#pragma unroll
            for (int e = 0; e < 16; e++) lds[geo.l1(e)] = x[e];
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 16; i++) x[i] = lds[geo.l2(i)];
            fwd_stages<Geo::S0, Mk::F2>(x, tw2, p, pinv);
#pragma unroll
            for (int i = 0; i < 16; i++) dst[geo.g2(i)] = mid_store(x[i], p, pinv);
        } else {
#pragma unroll
            for (int i = 0; i < 16; i++) x[i] = mid_load(src[geo.g2(i)]);
            inv_stages<Geo::S0, Mk::I1, false>(x, tw2, p, pinv, ninv, wlast);
            reduce16(x, p, pinv);
#pragma unroll
            for (int i = 0; i < 16; i++) lds[geo.l2(i)] = x[i];
            __syncthreads();
#pragma unroll
            for (int e = 0; e < 16; e++) x[e] = lds[geo.l1(e)];
            inv_round<Mk::I2, true>(x, tw1, p, pinv, ninv, wlast);
#pragma unroll
            for (int e = 0; e < 16; e++) dst[geo.g1(e)] = d2u(canon(x[e] + cadd, p, pinv));
        }
        __syncthreads();
    }
}

// GAL (inverse only): the input is read through the automorphism X -> X^g of its item (G->g[item]): a rotation's
// polynomial enters its key switch without a pass of its own
template <bool INV, bool P51, bool GAL = false>
__device__ __forceinline__ void ntt_v2_rows(const NttV2Args &A, double *lds, int t, unsigned li, const GaloisTab *G = nullptr) {
    const unsigned N = 1u << A.logN, N1 = N >> 8;
    const double p = A.modc[t].p, pinv = A.modc[t].pinv;
    const double *tw = A.tw + (size_t)t * N;
    const unsigned tid = threadIdx.x, hi4 = tid >> 4, lo4 = tid & 15;
    double tw1[15], tw2[15];
    const WMul unused = WMul{0.0, 0.0};
    load_twiddles(tw, N1 + blockIdx.x * 16 + hi4, lo4, tw1, tw2);
    const unsigned i0 = blockIdx.z * (unsigned)A.items_per_z;
    const unsigned i1 = (i0 + A.items_per_z < (unsigned)A.items) ? i0 + A.items_per_z : (unsigned)A.items;
    constexpr int F1 = P51 ? 0xA : 0x8, F2 = P51 ? 0x2 : 0x0;
    constexpr int I1 = P51 ? 0x2 : 0x4, I2 = P51 ? 0x1 : 0x4;
    const size_t tile0 = (size_t)blockIdx.x * 4096;
    double *grp = lds + hi4 * V2_GS;
    for (unsigned it = i0; it < i1; it++) {
        const u64d *src = A.src + (size_t)it * A.map.src_item_stride + (size_t)li * N;
        u64d *dst = A.dst + (size_t)it * A.map.dst_item_stride + (size_t)li * N;
        double x[16];
        if (!INV) {
#pragma unroll
            for (int e = 0; e < 16; e++) x[e] = mid_load(src[tile0 + hi4 * 256 + lo4 + 16 * e]);
            fwd_round<F1>(x, tw1, p, pinv);
#pragma unroll
            for (int e = 0; e < 16; e++) grp[e * 17 + lo4] = x[e];
            ROW_GROUP_SYNC();
#pragma unroll
            for (int e = 0; e < 16; e++) x[e] = grp[lo4 * 17 + e];
            fwd_round<F2>(x, tw2, p, pinv);
#pragma unroll
            for (int e = 0; e < 16; e++) grp[lo4 * 17 + e] = canon(x[e], p, pinv);
            ROW_GROUP_SYNC();
            // canonical words out in the row-pair layout: 16 bytes per lane and store
#pragma unroll
            for (int s = 0; s < 8; s++) {
                const double *rr = grp + row_pair_lds(lo4, s);
                ((ulonglong2 *)(dst + tile0))[row_pair_index(hi4, lo4, s)] = make_ulonglong2(d2u(rr[0]), d2u(rr[1]));
            }
        } else {
            {
                // all 16 words requested before the first is used: one memory latency per item, not sixteen
                // (row-pair layout: 16 bytes per lane and load)
                ulonglong2 raw[8];
#pragma unroll
                for (int s = 0; s < 8; s++) {
                    if (GAL) raw[s] = galois_pair_load(src, (unsigned)tile0 + hi4 * 256u + 32u * s + 2u * lo4, G->g[it], A.logN);
                    else raw[s] = ((const ulonglong2 *)(src + tile0))[row_pair_index(hi4, lo4, s)];
                }
                NTT_SCHED_FENCE();
#pragma unroll
                for (int s = 0; s < 8; s++) {
                    double *rr = grp + row_pair_lds(lo4, s);
                    rr[0] = u2d(raw[s].x);
                    rr[1] = u2d(raw[s].y);
                }
            }
            ROW_GROUP_SYNC();
#pragma unroll
            for (int e = 0; e < 16; e++) x[e] = grp[lo4 * 17 + e];
            inv_round<I1, false>(x, tw2, p, pinv, unused, unused);
#pragma unroll
            for (int e = 0; e < 16; e++) grp[lo4 * 17 + e] = x[e];
            ROW_GROUP_SYNC();
#pragma unroll
            for (int e = 0; e < 16; e++) x[e] = grp[e * 17 + lo4];
            inv_round<I2, false>(x, tw1, p, pinv, unused, unused);
#pragma unroll
            for (int e = 0; e < 16; e++) dst[tile0 + hi4 * 256 + lo4 + 16 * e] = mid_store(x[e], p, pinv);
        }
        ROW_GROUP_SYNC();
    }
}

// forward column pass of polynomials given as small signed integers (|coefficient| far below every modulus): same grid as
// ntt_v2_kernel; the residues are never written out limb by limb
__global__ __launch_bounds__(V2_THREADS) void ntt_v2_fwd_cols_small_kernel(NttV2Args A) {
    __shared__ double lds[16 * V2_GS];
    unsigned item_unused, li;
    const int t = resolve_limb(A.map, blockIdx.y, item_unused, li);
    if (t < 0) return;
    const bool p51 = is_p51(A.p51, t);
    switch (A.logN) {
        case 12: if (p51) ntt_v2_cols<false, 0, true, true>(A, lds, t, li); else ntt_v2_cols<false, 0, false, true>(A, lds, t, li); break;
        case 13: if (p51) ntt_v2_cols<false, 1, true, true>(A, lds, t, li); else ntt_v2_cols<false, 1, false, true>(A, lds, t, li); break;
        case 14: if (p51) ntt_v2_cols<false, 2, true, true>(A, lds, t, li); else ntt_v2_cols<false, 2, false, true>(A, lds, t, li); break;
        case 15: if (p51) ntt_v2_cols<false, 3, true, true>(A, lds, t, li); else ntt_v2_cols<false, 3, false, true>(A, lds, t, li); break;
        default: if (p51) ntt_v2_cols<false, 4, true, true>(A, lds, t, li); else ntt_v2_cols<false, 4, false, true>(A, lds, t, li); break;
    }
}

// inverse row pass of a rotation's polynomial: same grid as ntt_v2_kernel, input read through the items' automorphisms
__global__ __launch_bounds__(V2_THREADS) void ntt_v2_inv_rows_gal_kernel(NttV2Args A, GaloisTab G) {
    __shared__ double lds[16 * V2_GS];
    unsigned item_unused, li;
    const int t = resolve_limb(A.map, blockIdx.y, item_unused, li);
    if (t < 0) return;
    if (is_p51(A.p51, t)) ntt_v2_rows<true, true, true>(A, lds, t, li, &G);
    else ntt_v2_rows<true, false, true>(A, lds, t, li, &G);
}

// grid: x = tile (N/4096), y = limb slot within an item, z = chunk of items
template <bool INV, bool COLS>
__global__ __launch_bounds__(V2_THREADS) void ntt_v2_kernel(NttV2Args A) {
    __shared__ double lds[16 * V2_GS];
    unsigned item_unused, li;
    const int t = resolve_limb(A.map, blockIdx.y, item_unused, li);
    if (t < 0) return;
    const bool p51 = is_p51(A.p51, t);
    if (!COLS) {
        if (p51) ntt_v2_rows<INV, true>(A, lds, t, li);
        else ntt_v2_rows<INV, false>(A, lds, t, li);
    } else {
        switch (A.logN) {
            case 12: if (p51) ntt_v2_cols<INV, 0, true>(A, lds, t, li); else ntt_v2_cols<INV, 0, false>(A, lds, t, li); break;
            case 13: if (p51) ntt_v2_cols<INV, 1, true>(A, lds, t, li); else ntt_v2_cols<INV, 1, false>(A, lds, t, li); break;
            case 14: if (p51) ntt_v2_cols<INV, 2, true>(A, lds, t, li); else ntt_v2_cols<INV, 2, false>(A, lds, t, li); break;
            case 15: if (p51) ntt_v2_cols<INV, 3, true>(A, lds, t, li); else ntt_v2_cols<INV, 3, false>(A, lds, t, li); break;
            default: if (p51) ntt_v2_cols<INV, 4, true>(A, lds, t, li); else ntt_v2_cols<INV, 4, false>(A, lds, t, li); break;
        }
    }
}

// Register-tiled limb transforms for N = N1 x 256 (gfx950).
//
// A transform of N = 2^logN points is split into a strided pass over columns (the first
// logN-8 stages) and a contiguous pass over rows of 256 words (the last 8 stages).  In
// both, a workgroup of 256 threads works on 16 independent 256-point sub-transforms
// (4096 words): every thread keeps 16 words in registers and does four butterfly stages
// on them without touching memory ("round"); one exchange through LDS regroups the words
// for the second round of four stages.  Viewing a 256-point sub-transform as a 16x16
// matrix M[a][b] (point index 16a+b), the round on stages with span >= 16 works along a
// (a thread owns a column b), the round on spans < 16 works along b (a thread owns a row).
//
// Twiddles: stage s of the whole transform multiplies block i by psi^brev(2^s + i).  For a
// thread they reduce to 15 values per round that depend only on the sub-transform's
// position and the thread's lane, so they are loaded into registers once per workgroup
// and reused for every item the workgroup loops over (same modulus, same tile): twiddle
// traffic is amortised over the batch.
//
// Lazy ranges (units of p, see device_arith.h): for p < 2^50 values may reach 8p, for
// p < 2^51 only 4p, so the reduction points differ (template parameter P51).
#pragma once
#include "device_arith.h"

#define V2_THREADS 256
#define V2_GS 272  // doubles per padded 16x17 group in LDS

struct NttV2Args {
    const u64d *src;
    u64d *dst;
    const ModConst *modc;
    const WMul *tw;       // [T][N] table of the direction
    const WMul *tw_last;  // [T] inverse only
    const FinConst *fin;  // optional, inverse column pass: per limb slot, replaces the 1/N constants of the last stage
    int logN;
    int items, items_per_z;
    LimbMap map;
};

__device__ __forceinline__ void reduce16(double (&x)[16], double p, double pinv) {
#pragma unroll
    for (int e = 0; e < 16; e++) x[e] = reduce_balanced(x[e], p, pinv);
}

// four decimation-in-time stages (spans 8,4,2,1 over the register index); MASK bit s:
// reduce all words after stage s
template <int MASK>
__device__ __forceinline__ void fwd_round(double (&x)[16], const WMul (&tw)[15], double p, double pinv) {
#pragma unroll
    for (int s = 0; s < 4; s++) {
        const int span = 8 >> s;
#pragma unroll
        for (int b = 0; b < (1 << s); b++) {
            const WMul W = tw[(1 << s) - 1 + b];
#pragma unroll
            for (int j = 0; j < span; j++) {
                const int lo = b * 2 * span + j, hi = lo + span;
                const double v = mulmod_w(x[hi], W.w, W.wp, p);
                const double u = x[lo];
                x[lo] = u + v;
                x[hi] = u - v;
            }
        }
        if (MASK & (1 << s)) reduce16(x, p, pinv);
    }
}

// the same four stages undone (spans 1,2,4,8); MASK bit k: reduce after the k-th executed
// stage; FINAL folds 1/N into the very last stage of the whole transform
template <int MASK, bool FINAL>
__device__ __forceinline__ void inv_round(double (&x)[16], const WMul (&tw)[15], double p, double pinv, WMul ninv, WMul wlast) {
#pragma unroll
    for (int k = 0; k < 4; k++) {
        const int s = 3 - k, span = 8 >> s;
#pragma unroll
        for (int b = 0; b < (1 << s); b++) {
            const WMul W = tw[(1 << s) - 1 + b];
#pragma unroll
            for (int j = 0; j < span; j++) {
                const int lo = b * 2 * span + j, hi = lo + span;
                const double u = x[lo], v = x[hi];
                if (FINAL && s == 0) {
                    x[lo] = mulmod_w(u + v, ninv.w, ninv.wp, p);
                    x[hi] = mulmod_w(u - v, wlast.w, wlast.wp, p);
                } else {
                    x[lo] = u + v;
                    x[hi] = mulmod_w(u - v, W.w, W.wp, p);
                }
            }
        }
        if (MASK & (1 << k)) reduce16(x, p, pinv);
    }
}

// twiddles of one thread: base1 = position of the sub-transform in the stage numbering
// (1 for the column pass, N1 + row for the row pass), lane = the thread's row a in round 2
__device__ __forceinline__ void load_twiddles(const WMul *tw, unsigned base1, unsigned lane, WMul (&tw1)[15], WMul (&tw2)[15]) {
#pragma unroll
    for (int s = 0; s < 4; s++)
#pragma unroll
        for (int b = 0; b < (1 << s); b++) {
            tw1[(1 << s) - 1 + b] = tw[(base1 << s) + b];
            tw2[(1 << s) - 1 + b] = tw[((16u * base1 + lane) << s) + b];
        }
}

template <bool INV, bool COLS, bool P51>
__device__ __forceinline__ void ntt_v2_body(const NttV2Args &A, double *lds, int t, unsigned li) {
    const unsigned N = 1u << A.logN, N1 = N >> 8;
    const double p = A.modc[t].p, pinv = A.modc[t].pinv;
    const WMul *tw = A.tw + (size_t)t * N;
    const unsigned tid = threadIdx.x, hi4 = tid >> 4, lo4 = tid & 15;
    WMul tw1[15], tw2[15];
    WMul ninv = tw[0], wlast = tw[0];
    double cadd = 0.0;
    if (INV) {
        wlast = A.tw_last[t];
        if (COLS && A.fin) { ninv = A.fin[li].ninv; wlast = A.fin[li].wlast; cadd = A.fin[li].cadd; }
    }
    // COLS: column c = lo4 of tile blockIdx.x, lane = hi4.  rows: sub-transform = row hi4 of the tile, lane = lo4.
    const unsigned lane = COLS ? hi4 : lo4;
    const unsigned row = blockIdx.x * 16 + hi4;  // rows pass only
    load_twiddles(tw, COLS ? 1u : N1 + row, lane, tw1, tw2);
    const unsigned i0 = blockIdx.z * (unsigned)A.items_per_z;
    const unsigned i1 = (i0 + A.items_per_z < (unsigned)A.items) ? i0 + A.items_per_z : (unsigned)A.items;
    // lazy-range reduction points (see header comment)
    constexpr int F1 = P51 ? 0xA : 0x8, F2 = P51 ? 0x2 : 0x0;
    constexpr int I1 = P51 ? 0x2 : 0x4, I2 = P51 ? 0x1 : 0x4;
    for (unsigned it = i0; it < i1; it++) {
        const u64d *src = A.src + (size_t)it * A.map.src_item_stride + (size_t)li * N;
        u64d *dst = A.dst + (size_t)it * A.map.dst_item_stride + (size_t)li * N;
        double x[16];
        if (COLS) {
            const unsigned c = blockIdx.x * 16 + lo4;  // column of the N1 x 256 matrix (N1 = 256 here)
            if (!INV) {
#pragma unroll
                for (int e = 0; e < 16; e++) x[e] = u2d(src[(size_t)(hi4 + 16 * e) * 256 + c]);
                fwd_round<F1>(x, tw1, p, pinv);
#pragma unroll
                for (int e = 0; e < 16; e++) lds[(hi4 + 16 * e) * 16 + lo4] = x[e];
                __syncthreads();
#pragma unroll
                for (int e = 0; e < 16; e++) x[e] = lds[(16 * hi4 + e) * 16 + lo4];
                fwd_round<F2>(x, tw2, p, pinv);
#pragma unroll
                for (int e = 0; e < 16; e++) dst[(size_t)(16 * hi4 + e) * 256 + c] = d2u(canon(x[e], p, pinv));
            } else {
#pragma unroll
                for (int e = 0; e < 16; e++) x[e] = u2d(src[(size_t)(16 * hi4 + e) * 256 + c]);
                inv_round<I1, false>(x, tw2, p, pinv, ninv, wlast);
#pragma unroll
                for (int e = 0; e < 16; e++) lds[(16 * hi4 + e) * 16 + lo4] = x[e];
                __syncthreads();
#pragma unroll
                for (int e = 0; e < 16; e++) x[e] = lds[(hi4 + 16 * e) * 16 + lo4];
                inv_round<I2, true>(x, tw1, p, pinv, ninv, wlast);
#pragma unroll
                for (int e = 0; e < 16; e++) dst[(size_t)(hi4 + 16 * e) * 256 + c] = d2u(canon(x[e] + cadd, p, pinv));
            }
            __syncthreads();
        } else {
            const size_t tile0 = (size_t)blockIdx.x * 4096;
            double *grp = lds + hi4 * V2_GS;
            if (!INV) {
#pragma unroll
                for (int e = 0; e < 16; e++) x[e] = u2d(src[tile0 + hi4 * 256 + lo4 + 16 * e]);
                fwd_round<F1>(x, tw1, p, pinv);
#pragma unroll
                for (int e = 0; e < 16; e++) grp[e * 17 + lo4] = x[e];
                __syncthreads();
#pragma unroll
                for (int e = 0; e < 16; e++) x[e] = grp[lo4 * 17 + e];
                fwd_round<F2>(x, tw2, p, pinv);
#pragma unroll
                for (int e = 0; e < 16; e++) grp[lo4 * 17 + e] = canon(x[e], p, pinv);
                __syncthreads();
#pragma unroll
                for (int i = 0; i < 16; i++) dst[tile0 + i * 256 + tid] = d2u(lds[i * V2_GS + hi4 * 17 + lo4]);
            } else {
#pragma unroll
                for (int i = 0; i < 16; i++) lds[i * V2_GS + hi4 * 17 + lo4] = u2d(src[tile0 + i * 256 + tid]);
                __syncthreads();
#pragma unroll
                for (int e = 0; e < 16; e++) x[e] = grp[lo4 * 17 + e];
                inv_round<I1, false>(x, tw2, p, pinv, ninv, wlast);
#pragma unroll
                for (int e = 0; e < 16; e++) grp[lo4 * 17 + e] = x[e];
                __syncthreads();
#pragma unroll
                for (int e = 0; e < 16; e++) x[e] = grp[e * 17 + lo4];
                inv_round<I2, false>(x, tw1, p, pinv, ninv, wlast);
#pragma unroll
                for (int e = 0; e < 16; e++) dst[tile0 + hi4 * 256 + lo4 + 16 * e] = d2u(canon(x[e], p, pinv));
            }
            __syncthreads();
        }
    }
}

// grid: x = tile (N/4096), y = limb slot within an item, z = chunk of items
// COLS requires N1 = 256 (logN = 16); the row pass works for any N1 >= 16
template <bool INV, bool COLS>
__global__ __launch_bounds__(V2_THREADS) void ntt_v2_kernel(NttV2Args A) {
    __shared__ double lds[16 * V2_GS];
    unsigned item_unused, li;
    const int t = resolve_limb(A.map, blockIdx.y, item_unused, li);
    if (t < 0) return;
    if (A.modc[t].p >= 1125899906842624.0)  // 2^50
        ntt_v2_body<INV, COLS, true>(A, lds, t, li);
    else
        ntt_v2_body<INV, COLS, false>(A, lds, t, li);
}

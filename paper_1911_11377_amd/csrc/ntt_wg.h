// Whole limb transforms inside one workgroup for N = 2^13 and 2^14: the limb crosses HBM once.
//
// The transform is the same N1 x 256 decomposition as in ntt_v2.h, with the same butterflies, twiddles and lazy-range
// schedule (so the same bits), but both passes run in one workgroup of N/16 threads and the intermediate between them
// lives in LDS instead of HBM: every thread keeps 16 words in registers, and the N1 x 256 matrix sits in LDS in the
// padded row layout of the row pass (row r, column q at r*V2_GS + (q/16)*17 + q%16: 68 KiB at N = 2^13, 136 KiB at
// N = 2^14).  Each 256-thread quarter of the workgroup does the column pass of one 4096-word column tile, exchanging
// through the tile's own columns of that matrix in place; after one workgroup barrier every row is finished by its own
// 16 lanes exactly as in ntt_v2_rows.  Twiddles are fetched per round (they are shared by every limb of the modulus and
// stay in L2) instead of being held across items: a thread's registers hold one round's set at a time.
#pragma once
#include "ntt_v2.h"

__device__ __forceinline__ unsigned wg_pad(unsigned row, unsigned col) { return row * V2_GS + (col >> 4) * 17u + (col & 15u); }

template <bool INV, int LOGN, bool P51>
__device__ __forceinline__ void ntt_wg_body(const NttV2Args &A, double *lds, int t, unsigned li) {
    constexpr int Q = LOGN - 12;
    typedef ColsGeom<Q> Geo;
    typedef ColsMasks<Q, P51> Mk;
    constexpr unsigned N = 1u << LOGN, N1 = N >> 8;
    constexpr int RF1 = P51 ? 0xA : 0x8, RF2 = P51 ? 0x2 : 0x0;   // row pass, forward (as ntt_v2_rows)
    constexpr int RI1 = P51 ? 0x2 : 0x4, RI2 = P51 ? 0x1 : 0x4;   // row pass, inverse
    const double p = A.modc[t].p, pinv = A.modc[t].pinv;
    const double *tw = A.tw + (size_t)t * N;
    const unsigned tid = threadIdx.x;
    const Geo geo(tid & 255u, tid >> 8);          // column pass: this quarter's column tile
    const unsigned row = tid >> 4, lo4 = tid & 15;  // row pass: one row per 16 lanes
    double *grp = lds + row * V2_GS;
    WMul ninv = WMul{0.0, 0.0}, wlast = WMul{0.0, 0.0};
    double cadd = 0.0;
    if (INV) {
        ninv = A.tw_ninv[t];
        wlast = A.tw_last[t];
        if (A.fin) { ninv = A.fin[li].ninv; wlast = A.fin[li].wlast; cadd = A.fin[li].cadd; }
    }
    const WMul unused = WMul{0.0, 0.0};
    const unsigned i0 = blockIdx.y * (unsigned)A.items_per_z;
    const unsigned i1 = (i0 + A.items_per_z < (unsigned)A.items) ? i0 + A.items_per_z : (unsigned)A.items;
    for (unsigned it = i0; it < i1; it++) {
        const u64d *src = A.src + (size_t)it * A.map.src_item_stride + (size_t)li * N;
        u64d *dst = A.dst + (size_t)it * A.map.dst_item_stride + (size_t)li * N;
        double x[16];
        if (!INV) {
            // ---- column pass, from HBM into the LDS matrix
            {
                u64d raw[16];
#pragma unroll
                for (int e = 0; e < 16; e++) raw[e] = src[geo.g1(e)];
                {
                    double tw1[15];
#pragma unroll
                    for (int i = 0; i < 15; i++) tw1[i] = tw[1 + i];
                    NTT_SCHED_FENCE();
#pragma unroll
                    for (int e = 0; e < 16; e++) x[e] = u2d(raw[e]);
                    fwd_round<Mk::F1>(x, tw1, p, pinv);
                }
                // the second round's twiddles are requested here: their latency overlaps the exchange
                double tw1u[15], tw2u[15];
                load_cols_twiddles<Q>(tw, geo.a, tw1u, tw2u);
#pragma unroll
                for (int e = 0; e < 16; e++) lds[wg_pad(geo.r + Geo::G * e, geo.c0 + geo.c)] = x[e];
                __syncthreads();
#pragma unroll
                for (int i = 0; i < 16; i++) x[i] = lds[wg_pad(Geo::G * geo.a + (i % Geo::G), geo.c0 + geo.l16 + 16 * (i / Geo::G))];
                fwd_stages<Geo::S0, Mk::F2>(x, tw2u, p, pinv);
#pragma unroll
                for (int i = 0; i < 16; i++)
                    lds[wg_pad(Geo::G * geo.a + (i % Geo::G), geo.c0 + geo.l16 + 16 * (i / Geo::G))] = reduce_balanced(x[i], p, pinv);
            }
            __syncthreads();
            // ---- row pass, from the LDS matrix to HBM
            {
                double tw1[15], tw2[15];
                load_twiddles(tw, N1 + row, lo4, tw1, tw2);
#pragma unroll
                for (int e = 0; e < 16; e++) x[e] = grp[e * 17 + lo4];
                fwd_round<RF1>(x, tw1, p, pinv);
#pragma unroll
                for (int e = 0; e < 16; e++) grp[e * 17 + lo4] = x[e];
                ROW_GROUP_SYNC();
#pragma unroll
                for (int e = 0; e < 16; e++) x[e] = grp[lo4 * 17 + e];
                fwd_round<RF2>(x, tw2, p, pinv);
#pragma unroll
                for (int e = 0; e < 16; e++) grp[lo4 * 17 + e] = canon(x[e], p, pinv);
                ROW_GROUP_SYNC();
                // canonical words out in word pairs: 16 bytes per lane, 256 contiguous bytes per row and store
#pragma unroll
                for (int s = 0; s < 8; s++) {
                    const double *rr = grp + row_pair_lds(lo4, s);
                    ((ulonglong2 *)dst)[row_pair_index(row, lo4, s)] = make_ulonglong2(d2u(rr[0]), d2u(rr[1]));
                }
            }
        } else {
            // ---- row pass, from HBM into the LDS matrix
            {
                ulonglong2 raw[8];
#pragma unroll
                for (int s = 0; s < 8; s++) raw[s] = ((const ulonglong2 *)src)[row_pair_index(row, lo4, s)];
                double tw1[15], tw2[15];
                load_twiddles(tw, N1 + row, lo4, tw1, tw2);
                NTT_SCHED_FENCE();
#pragma unroll
                for (int s = 0; s < 8; s++) {
                    double *rr = grp + row_pair_lds(lo4, s);
                    rr[0] = u2d(raw[s].x);
                    rr[1] = u2d(raw[s].y);
                }
                ROW_GROUP_SYNC();
#pragma unroll
                for (int e = 0; e < 16; e++) x[e] = grp[lo4 * 17 + e];
                inv_round<RI1, false>(x, tw2, p, pinv, unused, unused);
#pragma unroll
                for (int e = 0; e < 16; e++) grp[lo4 * 17 + e] = x[e];
                ROW_GROUP_SYNC();
#pragma unroll
                for (int e = 0; e < 16; e++) x[e] = grp[e * 17 + lo4];
                inv_round<RI2, false>(x, tw1, p, pinv, unused, unused);
#pragma unroll
                for (int e = 0; e < 16; e++) grp[e * 17 + lo4] = reduce_balanced(x[e], p, pinv);
            }
            __syncthreads();
            // ---- column pass, from the LDS matrix to HBM
            {
                double tw1[15], tw2u[15];
                load_cols_twiddles<Q>(tw, geo.a, tw1, tw2u);
#pragma unroll
                for (int i = 0; i < 16; i++) x[i] = lds[wg_pad(Geo::G * geo.a + (i % Geo::G), geo.c0 + geo.l16 + 16 * (i / Geo::G))];
                inv_stages<Geo::S0, Mk::I1, false>(x, tw2u, p, pinv, ninv, wlast);
                reduce16(x, p, pinv);
#pragma unroll
                for (int i = 0; i < 16; i++) lds[wg_pad(Geo::G * geo.a + (i % Geo::G), geo.c0 + geo.l16 + 16 * (i / Geo::G))] = x[i];
                __syncthreads();
#pragma unroll
                for (int e = 0; e < 16; e++) x[e] = lds[wg_pad(geo.r + Geo::G * e, geo.c0 + geo.c)];
                inv_round<Mk::I2, true>(x, tw1, p, pinv, ninv, wlast);
#pragma unroll
                for (int e = 0; e < 16; e++) dst[geo.g1(e)] = d2u(canon(x[e] + cadd, p, pinv));
            }
        }
        __syncthreads();  // the matrix is free for the next item
    }
}

// grid: x = limb slot within an item, y = chunk of items; block = N/16 threads; dynamic LDS: (N/256) * V2_GS doubles
template <bool INV, int LOGN>
__global__ __launch_bounds__((1 << LOGN) / 16) void ntt_wg_kernel(NttV2Args A) {
    __shared__ double lds[((1 << LOGN) >> 8) * V2_GS];
    unsigned item_unused, li;
    const int t = resolve_limb(A.map, blockIdx.x, item_unused, li);
    if (t < 0) return;
    if (is_p51(A.p51, t))
        ntt_wg_body<INV, LOGN, true>(A, lds, t, li);
    else
        ntt_wg_body<INV, LOGN, false>(A, lds, t, li);
}

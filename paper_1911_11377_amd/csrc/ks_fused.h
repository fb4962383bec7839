// Fused key-switch / DivRound kernels for 2^12 <= N <= 2^16, built on the register-tiled
// transform passes of ntt_v2.h.  They remove the HBM round trips between a transform and the
// limb-wise step next to it:
//
//   tensor_rows_kernel : tensor product of a tile + the inverse row pass of its third component;
//   modup_cols_kernel  : inverse column pass of the source tiles, fast basis conversion (ModUp of
//                        a digit, or the conversion step of DivRound) and the column pass of the
//                        forward transform of every converted limb -- neither the conversion
//                        inputs nor the converted limbs are ever stored in coefficient form;
//   rows_inner_kernel  : row pass of the forward transform of every digit's extended limb,
//                        multiplied by the switching key and accumulated over the digits in
//                        registers -- the transformed limbs are never stored;
//   rows_final_kernel  : row pass fused with DivRound's last step
//                        out = (x - NTT(r - h)) * Bbar^-1 (+ addend).
//
// The conversion inputs y (y_i = d_i * qhat_i^-1 mod q_i, canonical) come out of the inverse
// transform itself: its last stage multiplies by 1/N anyway, so the extra constant rides along
// (FinConst).
#pragma once
#include "ntt_v2.h"

#ifdef CKKSMI_EMULATE
#define SCHED_FENCE() ((void)0)
#else
#define SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)
#endif

// ------------------------------------------------------------------ third tensor component + its inverse row pass
// The composite multiply feeds d2 = a1*b1 straight into key switching, whose first step is the inverse transform of
// d2.  This kernel forms d2 of one 4096-word tile (summed over the terms of a sum of products) and takes it through the
// inverse ROW pass while it is on chip; the column pass follows in the ModUp kernel.  Nothing else of the tensor is
// written anywhere: the fused inner product forms d0, d1 and d2 again from the operands where it needs them
// (rows_inner_kernel, tensor mode), which costs it one more limb read and saves this kernel six limb transfers.
struct TensorRowsArgs {
    const u64d *a, *b;   // [items][terms][2][level][N]
    u64d *ymid;          // [items][level][N]: inverse row pass of d2 (reduced doubles)
    const ModConst *modc;
    const double *tw_inv;
    int logN, level;
    int terms;
    P51Mask p51;
};

template <bool P51>
__device__ __forceinline__ void tensor_rows_body(const TensorRowsArgs &A, double *lds, unsigned item, int i) {
    constexpr int I1 = P51 ? 0x2 : 0x4, I2 = P51 ? 0x1 : 0x4;
    const unsigned N = 1u << A.logN, N1 = N >> 8;
    const ModConst mc = A.modc[i];
    const double p = mc.p, pinv = mc.pinv;
    const unsigned tid = threadIdx.x, hi4 = tid >> 4, lo4 = tid & 15;
    const size_t tile0 = (size_t)blockIdx.x * 4096, st = (size_t)A.level * N;
    double tw1[15], tw2[15];
    load_twiddles(A.tw_inv + (size_t)i * N, N1 + blockIdx.x * 16 + hi4, lo4, tw1, tw2);
    // second components of the operands
    const ulonglong2 *a1 = (const ulonglong2 *)(A.a + ((size_t)item * A.terms * 2 * A.level + A.level + i) * N + tile0);
    const ulonglong2 *b1 = (const ulonglong2 *)(A.b + ((size_t)item * A.terms * 2 * A.level + A.level + i) * N + tile0);
    double *grp = lds + hi4 * V2_GS;
    // word pairs in the row-pair layout (every row stays with its 16 lanes: no workgroup barrier)
    ulonglong2 A1[8], B1[8];
#pragma unroll
    for (int s = 0; s < 8; s++) {
        A1[s] = a1[row_pair_index(hi4, lo4, s)];
        B1[s] = b1[row_pair_index(hi4, lo4, s)];
    }
    SCHED_FENCE();
    double d2[16];
#pragma unroll
    for (int s = 0; s < 8; s++) {
        d2[2 * s] = mulmod(u2d(A1[s].x), u2d(B1[s].x), p, pinv);
        d2[2 * s + 1] = mulmod(u2d(A1[s].y), u2d(B1[s].y), p, pinv);
    }
    for (int t = 1; t < A.terms; t++) {  // further terms of a sum of products
        const size_t to = (size_t)t * st;  // 2*level*N words = st pairs
#pragma unroll
        for (int s = 0; s < 8; s++) {
            A1[s] = a1[to + row_pair_index(hi4, lo4, s)];
            B1[s] = b1[to + row_pair_index(hi4, lo4, s)];
        }
        SCHED_FENCE();
#pragma unroll
        for (int s = 0; s < 8; s++) {  // |sum| <= p/2 + 1 + 1.25p
            d2[2 * s] = reduce_balanced(d2[2 * s] + mulmod(u2d(A1[s].x), u2d(B1[s].x), p, pinv), p, pinv);
            d2[2 * s + 1] = reduce_balanced(d2[2 * s + 1] + mulmod(u2d(A1[s].y), u2d(B1[s].y), p, pinv), p, pinv);
        }
    }
#pragma unroll
    for (int s = 0; s < 8; s++) {
        // the inverse row pass starts from the canonical representative, as it does when d2 comes from memory
        double *rr = grp + row_pair_lds(lo4, s);
        rr[0] = canon(d2[2 * s], p, pinv);
        rr[1] = canon(d2[2 * s + 1], p, pinv);
    }
    ROW_GROUP_SYNC();
    // inverse row pass of d2 exactly as in ntt_v2_rows
    const WMul unused = WMul{0.0, 0.0};
    double x[16];
#pragma unroll
    for (int e = 0; e < 16; e++) x[e] = grp[lo4 * 17 + e];
    inv_round<I1, false>(x, tw2, p, pinv, unused, unused);
#pragma unroll
    for (int e = 0; e < 16; e++) grp[lo4 * 17 + e] = x[e];
    ROW_GROUP_SYNC();
#pragma unroll
    for (int e = 0; e < 16; e++) x[e] = grp[e * 17 + lo4];
    inv_round<I2, false>(x, tw1, p, pinv, unused, unused);
    u64d *ym = A.ymid + ((size_t)item * A.level + i) * N + tile0;
#pragma unroll
    for (int e = 0; e < 16; e++) ym[hi4 * 256 + lo4 + 16 * e] = mid_store(x[e], p, pinv);
}

// grid: x = tile (N/4096), y = limb, z = item
__global__ __launch_bounds__(V2_THREADS, 2) void tensor_rows_kernel(TensorRowsArgs A) {
    __shared__ double lds[16 * V2_GS];
    const int i = (int)blockIdx.y;
    if (is_p51(A.p51, i))
        tensor_rows_body<true>(A, lds, blockIdx.z, i);
    else
        tensor_rows_body<false>(A, lds, blockIdx.z, i);
}

// ------------------------------------------------------------------ conversion + column pass, targets looped in the workgroup
// Fast basis conversion and the column pass of the forward transform of its results, organised around the SOURCE tile:
// a workgroup reads the source tiles once (as the output of the inverse row pass, and runs their inverse column pass
// itself), keeps them in registers as doubles and produces the
// column-pass tile of every target limb of its chunk from them.  What remains per target is arithmetic and stores
// (which do not stall a wave), so the loads no longer alternate with the butterflies.  Per target the 255 column-pass
// twiddles of its modulus go through LDS (one coalesced 2 KB read per workgroup, fetched one target ahead).
// MODE 0 (ModUp): grid y = item * beta + digit, sources = the digit's limbs of y, targets = the other limbs of the
// extended basis.  MODE 1 (DivRound conversion, ModDown or rescale): grid y = row, sources = the D.nb dropped limbs
// (row r at y + r*y_row_stride), targets = the nc kept limbs, h subtracted.  MODE 2: MODE 1 in the exact form of DivRound:
// the overshoot v = floor(sum_m y_m * (1/b_m)) of every coefficient (double precision, products and sums in source
// order, each rounded) is found once from the sources and v * (Bbar mod c) leaves every target.
// MODE 3: ModDown FOLLOWED BY rescale, in the strict sequence's own bits, as one conversion.  Source 0 is the limb
// u = x_last * P^-1 + d_last (last = nc, the limb the rescale drops) and sources 1.. are the special limbs (D describes the
// ModDown over them, with b_idx[0] = last put in front).  Per coefficient the workgroup first forms the ModDown result of
// the dropped limb in coefficient form, s = u - (ModDown's conversion to limb `last`) * P^-1, and from it the rescale's
// conversion input y_B = (s + h_B) mod q_last; every target then receives the combination given at modup_cols_target.
struct ModupColsArgs {
    const u64d *y;                // MODE 0: [items][level][N] conversion inputs y_i, coefficient form, canonical
    unsigned long long y_row_stride;  // MODE 1
    u64d *dst;                    // MODE 0: [items][beta][E][N]; MODE 1: [rows][nc][N]
    const ModConst *modc;
    const double *tw;             // forward twiddles [T][N]
    const WMul *cc;               // ModUp constants [beta_top][alpha][alpha][T]
    DivRoundDev D;                // MODE 1 constants
    int logN, level, E, n_q, alpha, beta, T, nc;
    int targets_per_wg;
    P51Mask p51;
    // y holds the output of the inverse ROW pass (reduced doubles); the inverse column pass with its folded
    // constants runs in the workgroup's prologue and the conversion inputs never go through memory
    const double *tw_inv;         // inverse twiddles [T][N]
    const FinConst *fin;          // last-stage constants of source limb s (MODE 0: limb index; MODE 1: s-th dropped limb)
    // MODE 3: constants of the rescale that follows the ModDown described by D
    const double *hc2;            // [T] the rescale's h mod c
    double hb2;                   // the rescale's h mod q_last
    // per-call constants of the single source of a rescale whose input is multiplied by a scalar on the way
    int use_fin_val;
    FinConst fin_val;
};

// Inverse column pass of one source tile in registers: x in the round-2 register layout on entry, the canonical
// coefficient-form words (as doubles) in the round-1 layout on return.
template <bool P51, int Q>
__device__ __forceinline__ void inv_cols_in_regs(double (&x)[16], const double *twl, double *lds, const ColsGeom<Q> &geo, double p, double pinv,
                                                 const FinConst &F) {
    typedef ColsGeom<Q> Geo;
    typedef ColsMasks<Q, P51> Mk;
    const WMul unused = WMul{0.0, 0.0};
    {
        double tw2[15];
#pragma unroll
        for (int s = 0; s < 4; s++)
#pragma unroll
            for (int b = 0; b < (1 << s); b++) {
                if (s >= 4 - Q) {
                    const int u = s - (4 - Q);
                    tw2[(1 << s) - 1 + b] = twl[(16u << u) + (geo.a << u) + (b & ((1 << u) - 1))];
                } else {
                    tw2[(1 << s) - 1 + b] = 0.0;
                }
            }
        inv_stages<Geo::S0, Mk::I1, false>(x, tw2, p, pinv, unused, unused);
    }
    reduce16(x, p, pinv);
#pragma unroll
    for (int i = 0; i < 16; i++) lds[geo.l2(i)] = x[i];
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 16; e++) x[e] = lds[geo.l1(e)];
    {
        double tw1[15];
#pragma unroll
        for (int i = 0; i < 15; i++) tw1[i] = twl[1 + i];
        inv_round<Mk::I2, true>(x, tw1, p, pinv, F.ninv, F.wlast);
    }
#pragma unroll
    for (int e = 0; e < 16; e++) x[e] = canon(x[e] + F.cadd, p, pinv);
}

// VARIANT 1 (exact DivRound): vpack holds the overshoot of the thread's 16 coefficients, 3 bits each; Bm = Bbar mod p.
// VARIANT 2 (ModDown and rescale in one conversion): source 0 is the rescale's conversion input y_B, sources 1.. are
// ModDown's; Wc[0] = P^-1 mod p, hsub = ModDown's h mod p, Bm = the rescale's h mod p:
//     value = (sum_a y_a*conv_a - hA) * P^-1 + y_B - hB     (the two conversion results the last pass would subtract,
//                                                            brought to one: the transforms are linear)
template <bool P51, int NSRC, int Q, int VARIANT>
__device__ __forceinline__ void modup_cols_target(const double (&yd)[NSRC][16], const WMul (&Wc)[NSRC], const double *twl, double *lds, u64d *dst,
                                                  const ColsGeom<Q> &geo, double p, double pinv, double *twl_next, double tw_store, double hsub,
                                                  unsigned long long vpack, double Bm, const double *ybl = nullptr) {
    typedef ColsGeom<Q> Geo;
    typedef ColsMasks<Q, P51> Mk;
    double x[16];
#pragma unroll
    for (int e = 0; e < 16; e++) {
        double v = -hsub;
        if (VARIANT == 1) v = -reduce_balanced(hsub + (double)(unsigned)((vpack >> (3 * e)) & 7u) * Bm, p, pinv);  // v <= 3: below 4p, exact
#pragma unroll
        for (int a = (VARIANT == 2 ? 1 : 0); a < NSRC; a++) {
            const double ya = (VARIANT == 0 && NSRC == 3 && a == 0 && ybl) ? ybl[e * 256 + threadIdx.x] : yd[a][e];
            v += mulmod_w(ya, Wc[a].w, Wc[a].wp, p);
        }
        x[e] = reduce_balanced(v, p, pinv);  // |v| <= p + NSRC * 0.75p
        if (VARIANT == 2)  // 0.75p + (y_B < 2^51) + p: below 2^53
            x[e] = reduce_balanced(mulmod_w(x[e], Wc[0].w, Wc[0].wp, p) + ybl[e * 256 + threadIdx.x] - Bm, p, pinv);
    }
    {
        double tw1[15];
#pragma unroll
        for (int i = 0; i < 15; i++) tw1[i] = twl[1 + i];
        fwd_round<Mk::F1>(x, tw1, p, pinv);
    }
#pragma unroll
    for (int e = 0; e < 16; e++) lds[geo.l1(e)] = x[e];
    twl_next[threadIdx.x] = tw_store;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; i++) x[i] = lds[geo.l2(i)];
    {
        double tw2[15];
#pragma unroll
        for (int s = 0; s < 4; s++)
#pragma unroll
            for (int b = 0; b < (1 << s); b++) {
                if (s >= 4 - Q) {
                    const int u = s - (4 - Q);
                    tw2[(1 << s) - 1 + b] = twl[(16u << u) + (geo.a << u) + (b & ((1 << u) - 1))];
                } else {
                    tw2[(1 << s) - 1 + b] = 0.0;
                }
            }
        fwd_stages<Geo::S0, Mk::F2>(x, tw2, p, pinv);
    }
#pragma unroll
    for (int i = 0; i < 16; i++) dst[geo.g2(i)] = mid_store(x[i], p, pinv);
}

// grid: x = column tile (N/4096), y = item * beta + digit, z = chunk of targets_per_wg target limbs
// Four source tiles do not fit the registers of two waves per SIMD.  MODE 3 keeps y_B, which enters every target as a plain
// addend, in the second exchange buffer and pays a second barrier per target (0.80 ms; all four in registers at one wave
// per SIMD: 1.0 ms).  MODE 2 multiplies all four sources per target: it runs one wave per SIMD with all of them in
// registers (0.97 ms; one of them in LDS at two waves: 1.21 ms; with spills at two: 1.4 ms).
template <int Q, int NSRC, int MODE>
__global__ __launch_bounds__(V2_THREADS, (NSRC >= 4 && MODE == 2) ? 1 : 2) void modup_cols_kernel(ModupColsArgs A) {
    // one barrier per target: the exchange buffer alternates between two copies, the twiddles rotate through three
    // (target k's set is written during target k-1, while slower waves may still read the set of target k-2... k-1)
    __shared__ double lds[2][16 * V2_GS];
    __shared__ double twl[3][256];
    const unsigned N = 1u << A.logN;
    unsigned item = 0, j = 0;
    int lo = 0, nsrc, n_targets;
    const u64d *ysrc;
    static_assert(MODE != 2 || NSRC <= 4, "overshoot below 4: 3 bits each, h + v*Bbar below 4p");
    if (MODE == 0) {
        item = blockIdx.y / (unsigned)A.beta;
        j = blockIdx.y % (unsigned)A.beta;
        lo = (int)j * A.alpha;
        nsrc = (A.level - lo < A.alpha) ? A.level - lo : A.alpha;
        n_targets = A.E - nsrc;  // every limb of the extended basis outside the digit
        ysrc = A.y + ((size_t)item * A.level + lo) * N;
    } else {
        nsrc = A.D.nb;
        n_targets = A.nc;
        ysrc = A.y + (size_t)blockIdx.y * A.y_row_stride;
    }
    const int k0 = (int)blockIdx.z * A.targets_per_wg;
    const int k1 = k0 + A.targets_per_wg < n_targets ? k0 + A.targets_per_wg : n_targets;
    if (k0 >= k1) return;
    const ColsGeom<Q> geo(threadIdx.x, blockIdx.x);
    // the source words, once: a missing source (digit cut short by the level) re-reads the first limb, its constants are zero
    double yd[NSRC][16];
    {
        // every source tile is requested first, then taken through its inverse column pass one after the other
        u64d raw[NSRC][16];
#pragma unroll
        for (int a = 0; a < NSRC; a++) {
            const u64d *ya = ysrc + (size_t)(a < nsrc ? a : 0) * N;
#pragma unroll
            for (int i = 0; i < 16; i++) raw[a][i] = ya[geo.g2(i)];
        }
#pragma unroll
        for (int a = 0; a < NSRC; a++) {
            if (a < nsrc) {  // uniform
                const int ls = MODE == 0 ? lo + a : a;                 // index of the source among the transformed limbs
                const int ts = MODE == 0 ? lo + a : A.D.b_idx[a];      // its modulus
                const double ps = A.modc[ts].p, psinv = A.modc[ts].pinv;
                const FinConst F = A.use_fin_val ? A.fin_val : A.fin[ls];
                __syncthreads();  // the previous source is done with twl[2] and lds[0]
                twl[2][threadIdx.x] = A.tw_inv[(size_t)ts * N + threadIdx.x];
                __syncthreads();
                double x[16];
#pragma unroll
                for (int i = 0; i < 16; i++) x[i] = mid_load(raw[a][i]);
                if (is_p51(A.p51, ts))
                    inv_cols_in_regs<true, Q>(x, twl[2], lds[0], geo, ps, psinv, F);
                else
                    inv_cols_in_regs<false, Q>(x, twl[2], lds[0], geo, ps, psinv, F);
#pragma unroll
                for (int e = 0; e < 16; e++) yd[a][e] = x[e];
            } else {
#pragma unroll
                for (int e = 0; e < 16; e++) yd[a][e] = 0.0;
            }
        }
        __syncthreads();  // lds[0] and twl are about to be reused by the targets
    }
    unsigned long long vpack = 0;
    if (MODE == 2) {
#pragma unroll
        for (int e = 0; e < 16; e++) {
            double sum = yd[0][e] * A.D.invb_f[0];
#pragma unroll
            for (int a = 1; a < NSRC; a++)
                if (a < nsrc) sum = sum + yd[a][e] * A.D.invb_f[a];
            vpack |= (unsigned long long)floor(sum) << (3 * e);
        }
    }
    if (MODE == 3) {
        // the dropped limb's ModDown result in coefficient form, then the rescale's conversion input, in place of source 0
        const int tl = A.nc;
        const double pl = A.modc[tl].p, plinv = A.modc[tl].pinv;
        const WMul Pinv = A.D.Binv[tl];
        const double hA = A.D.hc[tl];
        WMul Wl[NSRC];
#pragma unroll
        for (int a = 1; a < NSRC; a++) Wl[a] = a < nsrc ? A.D.conv[(size_t)(a - 1) * A.T + tl] : WMul{0.0, 0.0};
#pragma unroll
        for (int e = 0; e < 16; e++) {
            double v = -hA;
#pragma unroll
            for (int a = 1; a < NSRC; a++) v += mulmod_w(yd[a][e], Wl[a].w, Wl[a].wp, pl);
            v = reduce_balanced(v, pl, plinv);
            const double sl = yd[0][e] - mulmod_w(v, Pinv.w, Pinv.wp, pl);  // (-0.75p, 1.75p)
            // y_B lives in the second exchange buffer from here on (this mode uses one buffer and two barriers per target):
            // four source tiles do not fit the registers of two waves per SIMD
            lds[1][e * 256 + threadIdx.x] = canon(sl + A.hb2, pl, plinv);
        }
    }
    // three source tiles: the first one lives in the second exchange buffer (one buffer, two barriers per target): without
    // it the kernel spills at two waves per SIMD (ModUp at the benchmark shape: 2.35 against 2.58 ms)
    constexpr bool SRC0_LDS = (MODE <= 1 && NSRC == 3);
    if (SRC0_LDS) {
#pragma unroll
        for (int e = 0; e < 16; e++) lds[1][e * 256 + threadIdx.x] = yd[0][e];
    }
    const size_t crow = ((size_t)j * A.alpha + (nsrc - 1)) * A.alpha;
    // MODE 0: extended-basis index of target k (the digit's own limbs are skipped) and its modulus index;
    // MODE 1: target k is kept limb k
    auto ext_of = [&](int k) { return MODE == 0 ? (k < lo ? k : k + nsrc) : k; };
    auto mod_of = [&](int x) { return MODE == 0 ? (x < A.level ? x : A.n_q + x - A.level) : x; };
    twl[0][threadIdx.x] = A.tw[(size_t)mod_of(ext_of(k0)) * N + threadIdx.x];
    double tw_next = k0 + 1 < k1 ? A.tw[(size_t)mod_of(ext_of(k0 + 1)) * N + threadIdx.x] : 0.0;
    __syncthreads();
    for (int k = k0; k < k1; k++) {
        const int x = ext_of(k), t = mod_of(x);
        const double *tcur = twl[(k - k0) % 3];
        double *tnext = twl[(k - k0 + 1) % 3];
        const double tw_store = tw_next;  // twiddle of target k+1, written before this target's barrier
        if (k + 2 < k1) tw_next = A.tw[(size_t)mod_of(ext_of(k + 2)) * N + threadIdx.x];
        const double p = A.modc[t].p, pinv = A.modc[t].pinv;
        WMul Wc[NSRC];
        double hsub = 0.0, Bm = 0.0;
        u64d *dst;
        if (MODE == 0) {
#pragma unroll
            for (int a = 0; a < NSRC; a++) Wc[a] = a < nsrc ? A.cc[(crow + a) * A.T + t] : WMul{0.0, 0.0};
            dst = A.dst + (((size_t)item * A.beta + j) * A.E + x) * N;
        } else {
#pragma unroll
            for (int a = 0; a < NSRC; a++)
                Wc[a] = a < nsrc ? A.D.conv[(size_t)(MODE == 3 ? (a ? a - 1 : 0) : a) * A.T + t] : WMul{0.0, 0.0};
            hsub = A.D.hc[t];
            if (MODE == 2) Bm = A.D.Bmod[t];
            if (MODE == 3) {
                Wc[0] = A.D.Binv[t];
                Bm = A.hc2[t];
            }
            dst = A.dst + ((size_t)blockIdx.y * A.nc + t) * N;
        }
        constexpr bool ONE_BUF = MODE == 3 || SRC0_LDS;  // the second buffer holds y_B / the first source tile
        double *xbuf = ONE_BUF ? lds[0] : lds[(k - k0) & 1];
        if (is_p51(A.p51, t))
            modup_cols_target<true, NSRC, Q, (MODE >= 2 ? MODE - 1 : 0)>(yd, Wc, tcur, xbuf, dst, geo, p, pinv, tnext, tw_store, hsub, vpack, Bm, (MODE == 3 || SRC0_LDS) ? lds[1] : nullptr);
        else
            modup_cols_target<false, NSRC, Q, (MODE >= 2 ? MODE - 1 : 0)>(yd, Wc, tcur, xbuf, dst, geo, p, pinv, tnext, tw_store, hsub, vpack, Bm, (MODE == 3 || SRC0_LDS) ? lds[1] : nullptr);
        if (ONE_BUF) __syncthreads();  // single exchange buffer: everybody has read it before the next target writes
    }
}

// ------------------------------------------------------------------ row pass helper
// round-2 twiddles of a thread (registers) and the round-1 twiddles of the tile's 16 rows (LDS, [16][16])
__device__ __forceinline__ void load_row_twiddles(const double *tw, unsigned N1, unsigned tile, unsigned hi4, unsigned lo4, double *tw1_lds,
                                                  double (&tw2)[15]) {
    const unsigned base1 = N1 + tile * 16 + hi4;
#pragma unroll
    for (int s = 0; s < 4; s++)
#pragma unroll
        for (int b = 0; b < (1 << s); b++) tw2[(1 << s) - 1 + b] = tw[((16u * base1 + lo4) << s) + b];
    if (lo4 < 15) {
        // entry i = (1<<s)-1+b  ->  tw[(base1 << s) + b]
        const unsigned i = lo4, s = (i >= 7) ? 3 : (i >= 3) ? 2 : (i >= 1) ? 1 : 0, b = i - ((1u << s) - 1);
        tw1_lds[hi4 * 16 + i] = tw[(base1 << s) + b];
    }
    __syncthreads();
}

// Finish the forward transform of one 16-row tile (column pass already done) and leave the
// balanced-reduced results in LDS in the padded layout: word (row g, position q) at g*V2_GS + (q/16)*17 + q%16.
// Every row is handled by its own 16 lanes: ends with a row-group sync, and the caller puts one before the next call.
template <bool P51>
__device__ __forceinline__ void rows_fwd_to_lds(const u64d *tile, double *lds, const double *tw1_lds, const double (&tw2)[15], double p,
                                                double pinv, unsigned hi4, unsigned lo4) {
    constexpr int F1 = P51 ? 0xA : 0x8, F2 = P51 ? 0x2 : 0x0;
    double *grp = lds + hi4 * V2_GS;
    double x[16];
#pragma unroll
    for (int e = 0; e < 16; e++) x[e] = mid_load(tile[hi4 * 256 + lo4 + 16 * e]);
    {
        // round-1 twiddles are the same for the 16 lanes of a row: kept in LDS, not in registers
        double tw1[15];
#pragma unroll
        for (int i = 0; i < 15; i++) tw1[i] = tw1_lds[hi4 * 16 + i];
        fwd_round<F1>(x, tw1, p, pinv);
    }
#pragma unroll
    for (int e = 0; e < 16; e++) grp[e * 17 + lo4] = x[e];
    ROW_GROUP_SYNC();
#pragma unroll
    for (int e = 0; e < 16; e++) x[e] = grp[lo4 * 17 + e];
    fwd_round<F2>(x, tw2, p, pinv);
#pragma unroll
    for (int e = 0; e < 16; e++) grp[lo4 * 17 + e] = reduce_balanced(x[e], p, pinv);
    ROW_GROUP_SYNC();
}

// ------------------------------------------------------------------ row pass + inner product
struct RowsInnerArgs {
    const u64d *dtA;     // [items][beta][E][N] column-pass output of the converted limbs
    const u64d *d_eval;  // evaluation-form source polynomial, item i at d_eval + i*d_eval_item_stride, [level][N]
    unsigned long long d_eval_item_stride;
    u64d *acc;           // [items][2][E][N]
    const ModConst *modc;
    const double *tw;    // forward twiddles
    int logN, level, E, n_q, alpha, beta, T;
    unsigned kt;         // min(N/4096, 8): see the grid mapping in rows_inner_body
    P51Mask p51;
    // fold_tail: the ciphertext limbs leave this kernel as z = acc * P^-1 + d (d = the addend of the same row: the product's
    // component, or sigma(c0) for the first row of a rotation), which is what the ModDown (and rescale) that follows reads.
    // 1: both components have an addend, 2: the first one only
    int fold_tail;
    const WMul *Pinv;    // [T] P^-1 mod q_i
    const u64d *addend;  // item i, component c, limb l at addend + i*add_item_stride + c*add_comp_stride + l*N
    unsigned long long add_item_stride, add_comp_stride;
    // Tensor mode (ta != nullptr; the composite multiply): the source polynomial is d2 = sum_t a1_t*b1_t of the operands
    // ta, tb: [items][terms][2][level][N], formed here for the limb's own digit, and the accumulators of the ciphertext limbs
    // start at P*d0 and P*d1 (d0 = sum a0*b0, d1 = sum a0*b1 + a1*b0), so that they leave as
    // z = (acc + P*d) * P^-1 = acc * P^-1 + d, or as acc + P*d itself (keep_acc: what the merged division divides).
    const u64d *ta, *tb;
    int terms, keep_acc;
    const WMul *Pmod;    // [T] P mod q_i
};

// GAL (a rotation): the source polynomial d_eval and the addend are read through the automorphism X -> X^g of their item
// (gal->g[item]), so that no rotated copy of the ciphertext is ever written
template <bool P51, bool GAL = false>
__device__ __forceinline__ void rows_inner_body(const RowsInnerArgs &A, const KeyTab &K, double *lds, double *tw1_lds, double *tw2_lds, int t,
                                                unsigned x, const GaloisTab *gal = nullptr) {
    constexpr int F1 = P51 ? 0xA : 0x8, F2 = P51 ? 0x2 : 0x0;
    const unsigned N = 1u << A.logN, N1 = N >> 8;
    const double p = A.modc[t].p, pinv = A.modc[t].pinv;
    const unsigned tid = threadIdx.x, hi4 = tid >> 4, lo4 = tid & 15;
    // Workgroups are handed to the 8 XCDs round-robin by linear id, and every XCD has its own L2.  blockIdx.x packs
    // (row tile mod KT, item) with KT = min(tiles, 8) in the low position, so that all items' workgroups for one key
    // tile (same extended limb, same row tile) land on the same XCD and the key tile is fetched from HBM once.
    const unsigned KT = A.kt;
    const unsigned item = blockIdx.x / KT, tile = blockIdx.x % KT + KT * blockIdx.y;
    {
        // both rounds' twiddles live in LDS here (round 2: [15][256], conflict-free): the registers are needed for the
        // accumulators and the operands in flight
        double tw2[15];
        load_row_twiddles(A.tw + (size_t)t * N, N1, tile, hi4, lo4, tw1_lds, tw2);
#pragma unroll
        for (int i = 0; i < 15; i++) tw2_lds[i * 256 + tid] = tw2[i];
    }
    const u64d *key = K.key[K.slot[item]];
    const size_t tile0 = (size_t)tile * 4096;
    double *grp = lds + hi4 * V2_GS;
    double a0[16], a1[16];
#pragma unroll
    for (int i = 0; i < 16; i++) a0[i] = a1[i] = 0.0;
    // Multiply-accumulate layout (row_pair_index): a thread owns 8 word pairs of the row its 16 lanes transform, so that key
    // words, the own digit's words and the results move 16 bytes per lane and the whole digit loop needs no workgroup barrier;
    // accumulator 2*s + b belongs to the word at column 32*s + 2*lo4 + b of row hi4.
    // The digit that contains this limb needs no transform: its operand is the source polynomial itself.
    const int j_own = (int)x < A.level ? (int)x / A.alpha : -1;
    const bool tensor_mode = !GAL && A.ta != nullptr && j_own >= 0;
    int pending = 1;  // terms in the accumulators since their last reduction (the own digit's term counts)
    if (tensor_mode) {
        // d0, d1, d2 of the thread's 16 words from the operands (summed over the terms, balanced-reduced)
        const size_t st = (size_t)A.level * N / 2;  // pairs between the two components of a ciphertext
        const ulonglong2 *pa = (const ulonglong2 *)(A.ta + ((size_t)item * A.terms * 2 * A.level + x) * N + tile0);
        const ulonglong2 *pb = (const ulonglong2 *)(A.tb + ((size_t)item * A.terms * 2 * A.level + x) * N + tile0);
        const ulonglong2 *k0 = (const ulonglong2 *)(key + (((size_t)j_own * 2 + 0) * A.T + t) * N + tile0);
        const ulonglong2 *k1 = (const ulonglong2 *)(key + (((size_t)j_own * 2 + 1) * A.T + t) * N + tile0);
        const WMul Pm = A.Pmod[t];
#pragma unroll
        for (int h = 0; h < 2; h++) {  // four pairs at a time: bounds the registers in flight
            // the own digit's key words travel with the first term's operands
            ulonglong2 kr0[4], kr1[4];
#pragma unroll
            for (int s = 0; s < 4; s++) {
                kr0[s] = k0[row_pair_index(hi4, lo4, 4 * h + s)];
                kr1[s] = k1[row_pair_index(hi4, lo4, 4 * h + s)];
            }
            double l0[8], l1[8], l2[8];
            for (int tm = 0; tm < A.terms; tm++) {
                const size_t to = (size_t)tm * 2 * st;
                ulonglong2 A0[4], A1[4], B0[4], B1[4];
#pragma unroll
                for (int s = 0; s < 4; s++) {
                    const unsigned e = row_pair_index(hi4, lo4, 4 * h + s);
                    A0[s] = pa[to + e]; A1[s] = pa[to + st + e]; B0[s] = pb[to + e]; B1[s] = pb[to + st + e];
                }
                SCHED_FENCE();
#pragma unroll
                for (int s = 0; s < 4; s++) {
#pragma unroll
                    for (int b = 0; b < 2; b++) {
                        const int i = 2 * s + b;
                        const double x0 = u2d(b ? A0[s].y : A0[s].x), x1 = u2d(b ? A1[s].y : A1[s].x);
                        const double y0 = u2d(b ? B0[s].y : B0[s].x), y1 = u2d(b ? B1[s].y : B1[s].x);
                        const double t0 = mulmod(x0, y0, p, pinv), t1 = mulmod(x0, y1, p, pinv) + mulmod(x1, y0, p, pinv), t2 = mulmod(x1, y1, p, pinv);
                        // |t| <= 2.5p on top of a reduced sum: below 2^53
                        l0[i] = reduce_balanced((tm ? l0[i] : 0.0) + t0, p, pinv);
                        l1[i] = reduce_balanced((tm ? l1[i] : 0.0) + t1, p, pinv);
                        l2[i] = reduce_balanced((tm ? l2[i] : 0.0) + t2, p, pinv);
                    }
                }
            }
#pragma unroll
            for (int s = 0; s < 4; s++) {
                const double v0 = l2[2 * s], vp0 = v0 * pinv, v1 = l2[2 * s + 1], vp1 = v1 * pinv;
                // two terms below 0.875p each: the own digit's product and P*d
                a0[8 * h + 2 * s] = mulmod_w(u2d(kr0[s].x), v0, vp0, p) + mulmod_w(l0[2 * s], Pm.w, Pm.wp, p);
                a1[8 * h + 2 * s] = mulmod_w(u2d(kr1[s].x), v0, vp0, p) + mulmod_w(l1[2 * s], Pm.w, Pm.wp, p);
                a0[8 * h + 2 * s + 1] = mulmod_w(u2d(kr0[s].y), v1, vp1, p) + mulmod_w(l0[2 * s + 1], Pm.w, Pm.wp, p);
                a1[8 * h + 2 * s + 1] = mulmod_w(u2d(kr1[s].y), v1, vp1, p) + mulmod_w(l1[2 * s + 1], Pm.w, Pm.wp, p);
            }
        }
        pending = 2;
    } else if (j_own >= 0) {
        const u64d *k0 = key + (((size_t)j_own * 2 + 0) * A.T + t) * N + tile0;
        const u64d *k1 = key + (((size_t)j_own * 2 + 1) * A.T + t) * N + tile0;
        const u64d *limb = A.d_eval + (size_t)item * A.d_eval_item_stride + (size_t)x * N, *src = limb + tile0;
        ulonglong2 kr0[8], kr1[8], xo[8];
#pragma unroll
        for (int s = 0; s < 8; s++) {
            if (GAL) xo[s] = galois_pair_load(limb, (unsigned)tile0 + hi4 * 256u + 32u * s + 2u * lo4, gal->g[item], A.logN);
            else xo[s] = ((const ulonglong2 *)src)[row_pair_index(hi4, lo4, s)];
            kr0[s] = ((const ulonglong2 *)k0)[row_pair_index(hi4, lo4, s)];
            kr1[s] = ((const ulonglong2 *)k1)[row_pair_index(hi4, lo4, s)];
        }
        SCHED_FENCE();
#pragma unroll
        for (int s = 0; s < 8; s++) {
            const double v0 = reduce_balanced(u2d(xo[s].x), p, pinv), vp0 = v0 * pinv;
            const double v1 = reduce_balanced(u2d(xo[s].y), p, pinv), vp1 = v1 * pinv;
            a0[2 * s] = mulmod_w(u2d(kr0[s].x), v0, vp0, p);
            a1[2 * s] = mulmod_w(u2d(kr1[s].x), v0, vp0, p);
            a0[2 * s + 1] = mulmod_w(u2d(kr0[s].y), v1, vp1, p);
            a1[2 * s + 1] = mulmod_w(u2d(kr1[s].y), v1, vp1, p);
        }
    }
    // The other digits, software-pipelined so that no memory latency sits in front of arithmetic: the limb words of a
    // digit are requested while the previous digit is multiplied, its key words while the limb goes through the row
    // pass.  xr holds the column-pass output of the converted limb in the register layout of the row pass.
    int j = (j_own == 0) ? 1 : 0;
    u64d xr[16];
    if (j < A.beta) {
        const u64d *src = A.dtA + (((size_t)item * A.beta + j) * A.E + x) * N + tile0;
#pragma unroll
        for (int i = 0; i < 16; i++) xr[i] = src[hi4 * 256 + lo4 + 16 * i];
    }
    while (j < A.beta) {
        const u64d *k0 = key + (((size_t)j * 2 + 0) * A.T + t) * N + tile0;
        const u64d *k1 = key + (((size_t)j * 2 + 1) * A.T + t) * N + tile0;
        ulonglong2 kr0[8], kr1[8];
#pragma unroll
        for (int s = 0; s < 8; s++) {
            kr0[s] = ((const ulonglong2 *)k0)[row_pair_index(hi4, lo4, s)];
            kr1[s] = ((const ulonglong2 *)k1)[row_pair_index(hi4, lo4, s)];
        }
        SCHED_FENCE();
        {
            double xx[16];
#pragma unroll
            for (int e = 0; e < 16; e++) xx[e] = mid_load(xr[e]);
            {
                double tw1[15];
#pragma unroll
                for (int i = 0; i < 15; i++) tw1[i] = tw1_lds[hi4 * 16 + i];
                fwd_round<F1>(xx, tw1, p, pinv);
            }
#pragma unroll
            for (int e = 0; e < 16; e++) grp[e * 17 + lo4] = xx[e];
            ROW_GROUP_SYNC();
#pragma unroll
            for (int e = 0; e < 16; e++) xx[e] = grp[lo4 * 17 + e];
            {
                double tw2[15];
#pragma unroll
                for (int i = 0; i < 15; i++) tw2[i] = tw2_lds[i * 256 + tid];
                fwd_round<F2>(xx, tw2, p, pinv);
            }
#pragma unroll
            for (int e = 0; e < 16; e++) grp[lo4 * 17 + e] = reduce_balanced(xx[e], p, pinv);
        }
        ROW_GROUP_SYNC();
        int jn = j + 1;
        if (jn == j_own) jn++;
        if (jn < A.beta) {
            const u64d *src = A.dtA + (((size_t)item * A.beta + jn) * A.E + x) * N + tile0;
#pragma unroll
            for (int i = 0; i < 16; i++) xr[i] = src[hi4 * 256 + lo4 + 16 * i];
        }
        SCHED_FENCE();
#pragma unroll
        for (int s = 0; s < 8; s++) {
            // the transformed word is the prepared factor (|v| <= p/2 + 1, v/p computed once for both components), the
            // key word the other one: each term is below 0.875p and the sum is reduced only when it could pass 2^53
            const double *vrow = grp + row_pair_lds(lo4, s);
            const double v0 = vrow[0], vp0 = v0 * pinv, v1 = vrow[1], vp1 = v1 * pinv;
            a0[2 * s] += mulmod_w(u2d(kr0[s].x), v0, vp0, p);
            a1[2 * s] += mulmod_w(u2d(kr1[s].x), v0, vp0, p);
            a0[2 * s + 1] += mulmod_w(u2d(kr0[s].y), v1, vp1, p);
            a1[2 * s + 1] += mulmod_w(u2d(kr1[s].y), v1, vp1, p);
        }
        if (++pending == (P51 ? 4 : 8)) {  // p < 2^51: 0.5p + 4 * 0.875p = 4p < 2^53; p < 2^50: 0.5p + 8 * 0.875p < 8p <= 2^53
#pragma unroll
            for (int i = 0; i < 16; i++) {
                a0[i] = reduce_balanced(a0[i], p, pinv);
                a1[i] = reduce_balanced(a1[i], p, pinv);
            }
            pending = 0;
        }
        ROW_GROUP_SYNC();  // the row's lanes have read its words before the next digit overwrites them
        j = jn;
    }
    u64d *o0 = A.acc + (((size_t)item * 2 + 0) * A.E + x) * N + tile0;
    u64d *o1 = A.acc + (((size_t)item * 2 + 1) * A.E + x) * N + tile0;
    if (tensor_mode && !A.keep_acc) {
        // z = (acc + P*d) * P^-1; accumulators are below 2^53: the prepared product is exact for them as they are
        const WMul Pi = A.Pinv[t];
#pragma unroll
        for (int s = 0; s < 8; s++) {
            const double z00 = mulmod_w(a0[2 * s], Pi.w, Pi.wp, p), z01 = mulmod_w(a0[2 * s + 1], Pi.w, Pi.wp, p);
            const double z10 = mulmod_w(a1[2 * s], Pi.w, Pi.wp, p), z11 = mulmod_w(a1[2 * s + 1], Pi.w, Pi.wp, p);
            ((ulonglong2 *)o0)[row_pair_index(hi4, lo4, s)] = make_ulonglong2(d2u(canon(z00, p, pinv)), d2u(canon(z01, p, pinv)));
            ((ulonglong2 *)o1)[row_pair_index(hi4, lo4, s)] = make_ulonglong2(d2u(canon(z10, p, pinv)), d2u(canon(z11, p, pinv)));
        }
        return;
    }
    if (!tensor_mode && A.fold_tail && (int)x < A.level) {
        const WMul Pi = A.Pinv[t];
        const u64d *l0 = A.addend + (size_t)item * A.add_item_stride + (size_t)x * N, *d0 = l0 + tile0;
        const bool both = A.fold_tail == 1;  // 2: only the first component has an addend (rotation)
        const u64d *l1 = both ? l0 + A.add_comp_stride : l0, *d1 = l1 + tile0;
        const double has1 = both ? 1.0 : 0.0;
        ulonglong2 dw0[8], dw1[8];
#pragma unroll
        for (int s = 0; s < 8; s++) {
            if (GAL) {
                const unsigned j = (unsigned)tile0 + hi4 * 256u + 32u * s + 2u * lo4;
                dw0[s] = galois_pair_load(l0, j, gal->g[item], A.logN);
                dw1[s] = both ? galois_pair_load(l1, j, gal->g[item], A.logN) : dw0[s];
            } else {
                dw0[s] = ((const ulonglong2 *)d0)[row_pair_index(hi4, lo4, s)];
                dw1[s] = ((const ulonglong2 *)d1)[row_pair_index(hi4, lo4, s)];
            }
        }
#pragma unroll
        for (int s = 0; s < 8; s++) {
            // accumulators are below 2^53: the prepared product is exact for them as they are
            const double z00 = mulmod_w(a0[2 * s], Pi.w, Pi.wp, p) + u2d(dw0[s].x), z01 = mulmod_w(a0[2 * s + 1], Pi.w, Pi.wp, p) + u2d(dw0[s].y);
            const double z10 = mulmod_w(a1[2 * s], Pi.w, Pi.wp, p) + has1 * u2d(dw1[s].x), z11 = mulmod_w(a1[2 * s + 1], Pi.w, Pi.wp, p) + has1 * u2d(dw1[s].y);
            ((ulonglong2 *)o0)[row_pair_index(hi4, lo4, s)] = make_ulonglong2(d2u(canon(z00, p, pinv)), d2u(canon(z01, p, pinv)));
            ((ulonglong2 *)o1)[row_pair_index(hi4, lo4, s)] = make_ulonglong2(d2u(canon(z10, p, pinv)), d2u(canon(z11, p, pinv)));
        }
        return;
    }
#pragma unroll
    for (int s = 0; s < 8; s++) {
        ((ulonglong2 *)o0)[row_pair_index(hi4, lo4, s)] = make_ulonglong2(d2u(canon(a0[2 * s], p, pinv)), d2u(canon(a0[2 * s + 1], p, pinv)));
        ((ulonglong2 *)o1)[row_pair_index(hi4, lo4, s)] = make_ulonglong2(d2u(canon(a1[2 * s], p, pinv)), d2u(canon(a1[2 * s + 1], p, pinv)));
    }
}

// grid: x = (row tile mod kt) + kt * item, y = row tile / kt, z = extended limb
__global__ __launch_bounds__(V2_THREADS, 2) void rows_inner_kernel(RowsInnerArgs A, KeyTab K) {
    __shared__ double lds[16 * V2_GS];
    __shared__ double tw1_lds[16 * 16];
    __shared__ double tw2_lds[15 * 256];
    const unsigned x = blockIdx.z;
    const int t = (int)x < A.level ? (int)x : A.n_q + (int)x - A.level;
    if (is_p51(A.p51, t))
        rows_inner_body<true>(A, K, lds, tw1_lds, tw2_lds, t, x);
    else
        rows_inner_body<false>(A, K, lds, tw1_lds, tw2_lds, t, x);
}

// the same for rotations: source polynomial and addend read through the items' automorphisms (no tensor mode here)
__global__ __launch_bounds__(V2_THREADS, 2) void rows_inner_gal_kernel(RowsInnerArgs A, KeyTab K, GaloisTab G) {
    __shared__ double lds[16 * V2_GS];
    __shared__ double tw1_lds[16 * 16];
    __shared__ double tw2_lds[15 * 256];
    const unsigned x = blockIdx.z;
    const int t = (int)x < A.level ? (int)x : A.n_q + (int)x - A.level;
    if (is_p51(A.p51, t))
        rows_inner_body<true, true>(A, K, lds, tw1_lds, tw2_lds, t, x, &G);
    else
        rows_inner_body<false, true>(A, K, lds, tw1_lds, tw2_lds, t, x, &G);
}

// ------------------------------------------------------------------ row pass + DivRound final step
struct RowsFinalArgs {
    const u64d *tmpA;    // [rows][nc][N] column-pass output of (r_i - h)
    const u64d *x;       // kept limbs, evaluation form: row r, limb i at x + r*x_row_stride + i*N
    unsigned long long x_row_stride;
    const u64d *addend;  // optional: row r limb i at addend + (r/2)*add_item_stride + (r%2)*add_comp_stride + i*N
    unsigned long long add_item_stride, add_comp_stride;
    int add_both;
    u64d *out;           // row r, limb i at out + r*out_row_stride + (i - out_limb0)*N
    unsigned long long out_row_stride;
    int out_limb0;
    const ModConst *modc;
    const double *tw;
    const WMul *Binv;    // [T]
    const WMul *pre;     // optional [T]: the addend enters BEFORE the division, out = (x + pre_i*addend - r) * Binv
    const WMul *xmul;    // optional [T] (without pre): out = (x*xmul_i + addend - r) * Binv
    int zsub;            // 1: x already holds x*Binv + addend: out = x - r * Binv
    int logN, nc;
    int limb0;             // first limb handled (grid z counts from it)
    int rows, rows_per_x;  // a workgroup loops over rows_per_x rows (same limb, same tile: twiddles reused)
    P51Mask p51;
};

// Rotations from a shared ModUp: rows come in pairs (item, rotation r), R rotations per item; the first row of a pair adds
// sigma_r(c0 of its item), read through the automorphism from the input ciphertext itself (A.addend = c0 of item 0,
// A.add_item_stride = words between the items' ciphertexts)
struct RowsFinalGal { int R; unsigned g[CKKSMI_MAX_KEYS]; };

template <bool P51, bool GAL = false>
__device__ __forceinline__ void rows_final_body(const RowsFinalArgs &A, double *lds, double *tw1_lds, int i, bool xm_val = false,
                                                WMul xmv = WMul{0.0, 0.0}, const RowsFinalGal *gal = nullptr) {
    const unsigned N = 1u << A.logN, N1 = N >> 8;
    const double p = A.modc[i].p, pinv = A.modc[i].pinv;
    const unsigned tid = threadIdx.x, hi4 = tid >> 4, lo4 = tid & 15;
    const unsigned tile = blockIdx.y;
    double tw2[15];
    load_row_twiddles(A.tw + (size_t)i * N, N1, tile, hi4, lo4, tw1_lds, tw2);
    const size_t tile0 = (size_t)tile * 4096;
    const WMul W = A.Binv[i];
    const bool pre = A.pre != nullptr, xm = xm_val || A.xmul != nullptr;
    const WMul Pm = pre ? A.pre[i] : (xm_val ? xmv : (xm ? A.xmul[i] : WMul{0.0, 0.0}));
    const unsigned r0 = blockIdx.x * (unsigned)A.rows_per_x;
    const unsigned r1 = (r0 + A.rows_per_x < (unsigned)A.rows) ? r0 + A.rows_per_x : (unsigned)A.rows;
    for (unsigned row = r0; row < r1; row++) {
        const u64d *xin = A.x + (size_t)row * A.x_row_stride + (size_t)i * N + tile0;
        u64d *out = A.out + (size_t)row * A.out_row_stride + (size_t)(i - A.out_limb0) * N + tile0;
        const bool add = A.addend && (pre || xm || A.add_both || (row & 1u) == 0);
        const double has_add = add ? 1.0 : 0.0;
        const u64d *ad = add ? A.addend + (size_t)(row / 2) * A.add_item_stride + (size_t)(row % 2) * A.add_comp_stride + (size_t)i * N + tile0 : xin;
        // operands of the last step are requested before the transform so that their latency overlaps it
        // pointwise part in the row-pair layout: 16 bytes per lane and memory instruction, no workgroup barrier
        ulonglong2 xr[8], ar[8];
#pragma unroll
        for (int s = 0; s < 8; s++) {
            xr[s] = ((const ulonglong2 *)xin)[row_pair_index(hi4, lo4, s)];
            if (GAL && add) {
                const unsigned pair = row / 2u, item = pair / (unsigned)gal->R, r = pair % (unsigned)gal->R;
                ar[s] = galois_pair_load(A.addend + (size_t)item * A.add_item_stride + (size_t)i * N,
                                         (unsigned)tile0 + hi4 * 256u + 32u * s + 2u * lo4, gal->g[r], A.logN);
            } else {
                ar[s] = ((const ulonglong2 *)ad)[row_pair_index(hi4, lo4, s)];
            }
        }
        SCHED_FENCE();
        rows_fwd_to_lds<P51>(A.tmpA + ((size_t)row * A.nc + i) * N + tile0, lds, tw1_lds, tw2, p, pinv, hi4, lo4);
#pragma unroll
        for (int s = 0; s < 8; s++) {
            const double *rr = lds + hi4 * V2_GS + row_pair_lds(lo4, s);
            double x0 = u2d(xr[s].x), x1 = u2d(xr[s].y);
            if (pre) {  // |x + pre*addend - r| < p + 1.5p + p/2 + 1
                x0 += mulmod_w(u2d(ar[s].x), Pm.w, Pm.wp, p);
                x1 += mulmod_w(u2d(ar[s].y), Pm.w, Pm.wp, p);
            }
            if (xm) {  // |x*xmul + addend - r| < 0.75p + p + p/2 + 1 (without an addend `ar` is a copy of x: not used)
                // the hmul tail's addend enters before the division; the scalar rescale's one is added to the result
                const double before = xm_val ? 0.0 : has_add;
                x0 = mulmod_w(x0, Pm.w, Pm.wp, p) + before * u2d(ar[s].x);
                x1 = mulmod_w(x1, Pm.w, Pm.wp, p) + before * u2d(ar[s].y);
            }
            double v0, v1;
            if (A.zsub) {
                v0 = x0 - mulmod_w(rr[0], W.w, W.wp, p);
                v1 = x1 - mulmod_w(rr[1], W.w, W.wp, p);
            } else {
                v0 = mulmod_w(x0 - rr[0], W.w, W.wp, p);
                v1 = mulmod_w(x1 - rr[1], W.w, W.wp, p);
            }
            if (add && !pre && (!xm || xm_val)) {
                v0 += u2d(ar[s].x);
                v1 += u2d(ar[s].y);
            }
            ((ulonglong2 *)out)[row_pair_index(hi4, lo4, s)] = make_ulonglong2(d2u(canon(v0, p, pinv)), d2u(canon(v1, p, pinv)));
        }
        ROW_GROUP_SYNC();
    }
}

// grid: x = chunk of rows (item, component), y = row tile (N/4096), z = kept limb
__global__ __launch_bounds__(V2_THREADS) void rows_final_kernel(RowsFinalArgs A) {
    __shared__ double lds[16 * V2_GS];
    __shared__ double tw1_lds[16 * 16];
    const int i = A.limb0 + (int)blockIdx.z;
    if (is_p51(A.p51, i))
        rows_final_body<true>(A, lds, tw1_lds, i);
    else
        rows_final_body<false>(A, lds, tw1_lds, i);
}

// the same for rotations from a shared ModUp: the addend sigma_r(c0) is read through the automorphism
__global__ __launch_bounds__(V2_THREADS) void rows_final_gal_kernel(RowsFinalArgs A, RowsFinalGal G) {
    __shared__ double lds[16 * V2_GS];
    __shared__ double tw1_lds[16 * 16];
    const int i = A.limb0 + (int)blockIdx.z;
    if (is_p51(A.p51, i))
        rows_final_body<true, true>(A, lds, tw1_lds, i, false, WMul{0.0, 0.0}, &G);
    else
        rows_final_body<false, true>(A, lds, tw1_lds, i, false, WMul{0.0, 0.0}, &G);
}

// the same with the kept limb multiplied by a per-call scalar first: out = (c*x - r) * Binv (+ addend): rescale of c*x
__global__ __launch_bounds__(V2_THREADS) void rows_final_scalar_kernel(RowsFinalArgs A, ScalarTab S) {
    __shared__ double lds[16 * V2_GS];
    __shared__ double tw1_lds[16 * 16];
    const int i = A.limb0 + (int)blockIdx.z;
    const WMul xmv = S.c[i];
    if (is_p51(A.p51, i))
        rows_final_body<true>(A, lds, tw1_lds, i, true, xmv);
    else
        rows_final_body<false>(A, lds, tw1_lds, i, true, xmv);
}

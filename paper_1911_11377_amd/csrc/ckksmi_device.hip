// Device side of the C ABI: constant-table upload, argument validation and the
// kernel launch sequences of every ciphertext operation.
#ifndef CKKSMI_EMULATE
#include <hip/hip_runtime.h>
#define CKKSMI_LAUNCH(kern, grid, block, stream, ...) hipLaunchKernelGGL(kern, grid, block, 0, stream, __VA_ARGS__)
#endif

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "ckksmi_internal.h"
#include "kernels.h"
#include "ntt_v2.h"
#include "ks_fused.h"
#include "ntt_wg.h"
#include "encode_device.h"
#include "mac_mfma.h"

// Launch `kern`; when profiling is on, bracket it with two events on the same stream and
// remember them under kernel class `kid` together with `units` of algorithmic work.
#define KL(c, kid, units, kern, grid, block, st, ...)                                   \
    do {                                                                                \
        ProfRec *pr_ = (c)->prof_on ? prof_begin((c), (kid), (double)(units), (st)) : nullptr; \
        CKKSMI_LAUNCH(kern, grid, block, st, __VA_ARGS__);                              \
        if (pr_) (void)hipEventRecord((hipEvent_t)pr_->stop, (st));                     \
    } while (0)

// Scratch memory of ckksmi_rescale_static, the one entry point that takes no workspace: a file-scope device array, one copy
// per GPU, held until the process ends.  Host code never uses the array's name as an address: every device's copy is
// looked up once (hipGetSymbolAddress, with that device current) when the first context on that device is created.
static __device__ __align__(256) unsigned long long scratch[CKKSMI_STATIC_SCRATCH_BYTES / 8];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each GPU, nullptr until looked up

// with `device` current
bool lookup_static_scratch(int device) {
    if (device < 0 || device >= kMaxDevices) return true;  // no static scratch there: ckksmi_rescale_static reports it
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device]) return true;
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return false;
    g_scratch_ptr[device] = p;
    return true;
}

ProfRec *prof_begin(ckksmi_ctx *c, int kid, double units, hipStream_t st) {
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return nullptr;
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return nullptr; }
    (void)hipEventRecord(a, st);
    c->prof.push_back(ProfRec{kid, units, (void *)a, (void *)b});
    return &c->prof.back();
}

struct Guard {  // records the first HIP error of a call
    ckksmi_ctx *c;
    bool ok = true;
    explicit Guard(ckksmi_ctx *ctx) : c(ctx) {}
    void check(hipError_t e) {
        if (e != hipSuccess && ok) { ok = false; c->last_hip_error = (int)e; }
    }
    int rc() {
        check(hipGetLastError());
        return ok ? CKKSMI_OK : CKKSMI_EDEVICE;
    }
};

template <class Tp>
Tp *upload(ckksmi_ctx *c, const Tp *host, size_t count, bool &ok) {
    void *p = nullptr;
    const size_t bytes = count ? count * sizeof(Tp) : 16;
    if (hipMalloc(&p, bytes) != hipSuccess) { ok = false; return nullptr; }
    c->dev_allocs.push_back(p);
    if (count && hipMemcpy(p, host, count * sizeof(Tp), hipMemcpyHostToDevice) != hipSuccess) ok = false;
    return (Tp *)p;
}

inline int la_for(int logN) { return logN <= 12 ? 0 : std::min(8, logN - 8); }

inline bool dev_ok(const ckksmi_ctx *c) { return c && c->device >= 0; }
inline hipStream_t S(void *s) { return (hipStream_t)s; }

LimbMap table_map(const int *index, int n_limbs, size_t src_stride, size_t dst_stride) {
    LimbMap M;
    memset(&M, 0, sizeof(M));
    M.per_item = n_limbs;
    M.mode = 0;
    M.src_item_stride = src_stride;
    M.dst_item_stride = dst_stride;
    for (int i = 0; i < n_limbs; i++) M.modidx[i] = (unsigned char)index[i];
    return M;
}

// transform `items` groups of map.per_item limbs; forward: coefficient -> evaluation
// passes: 3 = whole transform, 1 = strided (column) pass only, 2 = contiguous (row) pass only
// gal (inverse row pass of the register-tiled sizes only): item i's input is read through the automorphism X -> X^(gal->g[i])
void launch_ntt(ckksmi_ctx *c, bool forward, const u64 *src, u64 *dst, const LimbMap &M, size_t items, hipStream_t st,
                const FinConst *fin = nullptr, int passes = 3, const GaloisTab *gal = nullptr) {
    if (items == 0 || M.per_item == 0) return;
    NttArgs A;
    A.src = (const u64d *)src;
    A.dst = (u64d *)dst;
    A.modc = c->d_mod;
    A.tw = forward ? c->d_tw_fwd : c->d_tw_inv;
    A.tw_last = c->d_tw_inv_last;
    A.logN = c->logN;
    A.LA = la_for(c->logN);
    A.map = M;
    const unsigned N = 1u << c->logN, N1 = 1u << A.LA, N2 = N >> A.LA;
    const unsigned R = N2 >= NTT_TILE ? 1u : NTT_TILE / N2;
    const unsigned limbs = (unsigned)(items * M.per_item);
    // limbs actually transformed (the key-switch map skips the limbs of each digit itself)
    const double limbs_work = M.mode == 1 ? (double)items * ((double)M.per_item - M.level) : (double)limbs;
    dim3 grow(limbs, (N1 + R - 1) / R), gcol(limbs, N2 / NTT_TC);
    // register-tiled kernels for 2^12 <= N <= 2^16 (always two passes; the generic kernels take one up to N = 2^12)
    const bool v2_rows = c->logN >= 12 && c->logN <= 16, v2_cols = v2_rows;
    const bool two_pass = v2_cols || A.LA != 0;
    NttV2Args V;
    V.src = A.src; V.dst = A.dst; V.modc = A.modc; V.tw = forward ? c->d_tww_fwd : c->d_tww_inv; V.tw_ninv = c->d_tw_ninv;
    V.tw_last = A.tw_last; V.fin = fin; V.logN = A.logN; V.map = M; V.p51 = c->p51mask;
    V.items = (int)items;
    const unsigned tiles = N >= 4096u ? N / 4096u : 1u;
    // enough workgroups to fill the chip, otherwise as many items per workgroup as possible (twiddle reuse)
    unsigned zchunks = ((unsigned)c->ntt_target_wgs + tiles * M.per_item - 1) / (tiles * M.per_item);
    if (zchunks > items) zchunks = (unsigned)items;
    if (zchunks < 1) zchunks = 1;
    V.items_per_z = (int)((items + zchunks - 1) / zchunks);
    zchunks = (unsigned)((items + V.items_per_z - 1) / V.items_per_z);
    dim3 gv2(tiles, M.per_item, zchunks);
    if (passes == 3 && (c->logN == 13 || c->logN == 14)) {
        // the whole limb in one workgroup: one trip through HBM (see ntt_wg.h); a workgroup loops over items of its limb slot
        unsigned zc = ((unsigned)c->ntt_target_wgs / 4 + M.per_item - 1) / M.per_item;
        if (zc > items) zc = (unsigned)items;
        if (zc < 1) zc = 1;
        V.items_per_z = (int)((items + zc - 1) / zc);
        zc = (unsigned)((items + V.items_per_z - 1) / V.items_per_z);
        const dim3 gw(M.per_item, zc), bw((unsigned)(N / 16));
        if (c->logN == 13) {
            if (forward) KL(c, CKKSMI_K_NTT_LDS, limbs_work, (ntt_wg_kernel<false, 13>), gw, bw, st, V);
            else KL(c, CKKSMI_K_NTT_LDS, limbs_work, (ntt_wg_kernel<true, 13>), gw, bw, st, V);
        } else {
            if (forward) KL(c, CKKSMI_K_NTT_LDS, limbs_work, (ntt_wg_kernel<false, 14>), gw, bw, st, V);
            else KL(c, CKKSMI_K_NTT_LDS, limbs_work, (ntt_wg_kernel<true, 14>), gw, bw, st, V);
        }
        return;
    }
    if (forward) {
        if (two_pass && (passes & 1)) {
            if (v2_cols) KL(c, CKKSMI_K_NTT_FWD_COL, limbs_work, (ntt_v2_kernel<false, true>), gv2, dim3(V2_THREADS), st, V);
            else KL(c, CKKSMI_K_NTT_FWD_COL, limbs_work, ntt_fwd_kernel<true>, gcol, dim3(NTT_THREADS), st, A);
            // second pass works in place on dst
            A.src = (const u64d *)dst;
            A.map.src_item_stride = A.map.dst_item_stride;
            V.src = A.src;
            V.map.src_item_stride = V.map.dst_item_stride;
        }
        if (passes & 2) {
            if (v2_rows) KL(c, CKKSMI_K_NTT_FWD_ROW, limbs_work, (ntt_v2_kernel<false, false>), gv2, dim3(V2_THREADS), st, V);
            else KL(c, CKKSMI_K_NTT_FWD_ROW, limbs_work, ntt_fwd_kernel<false>, grow, dim3(NTT_THREADS), st, A);
        }
    } else {
        // inverse: passes 2 = contiguous (row) pass only, leaving the reduced-double intermediate (register-tiled sizes)
        if (v2_rows && gal) KL(c, CKKSMI_K_NTT_INV_ROW, limbs_work, ntt_v2_inv_rows_gal_kernel, gv2, dim3(V2_THREADS), st, V, *gal);
        else if (v2_rows) KL(c, CKKSMI_K_NTT_INV_ROW, limbs_work, (ntt_v2_kernel<true, false>), gv2, dim3(V2_THREADS), st, V);
        else KL(c, CKKSMI_K_NTT_INV_ROW, limbs_work, ntt_inv_kernel<false>, grow, dim3(NTT_THREADS), st, A);
        if (two_pass && (passes & 1)) {
            A.src = (const u64d *)dst;
            A.map.src_item_stride = A.map.dst_item_stride;
            V.src = A.src;
            V.map.src_item_stride = V.map.dst_item_stride;
            if (v2_cols) KL(c, CKKSMI_K_NTT_INV_COL, limbs_work, (ntt_v2_kernel<true, true>), gv2, dim3(V2_THREADS), st, V);
            else KL(c, CKKSMI_K_NTT_INV_COL, limbs_work, ntt_inv_kernel<true>, gcol, dim3(NTT_THREADS), st, A);
        }
    }
}

inline unsigned ew_blocks(size_t total) { return (unsigned)((total + EW_THREADS - 1) / EW_THREADS); }

ScalarTab scalar_tab(const ckksmi_ctx *c, int64_t v, int level) {
    ScalarTab Sx;
    memset(&Sx, 0, sizeof(Sx));
    for (int i = 0; i < level; i++) {
        u64 r = hm::signed_mod(v, c->mod[i]);
        Sx.c[i] = make_wmul(r, c->mod[i]);
        Sx.cpos[i] = (double)r;
    }
    return Sx;
}

// words of workspace one item needs
size_t ks_words_per_item(const ckksmi_ctx *c, int level) {
    const size_t N = c->N, E = level + c->k, beta = (level + c->alpha - 1) / c->alpha;
    return N * ((size_t)level + beta * E + 2 * E + 2 * (size_t)level);
}
size_t rescale_words_per_item(const ckksmi_ctx *c, int level) { return c->N * (2 + 2 * (size_t)(level - 1)); }


// ---- fused path, N = 2^16 -------------------------------------------------------------
unsigned zchunks_for(const ckksmi_ctx *c, unsigned wgs_per_item, size_t items, int &items_per_z) {
    unsigned z = ((unsigned)c->ntt_target_wgs + wgs_per_item - 1) / wgs_per_item;
    if (z > items) z = (unsigned)items;
    if (z < 1) z = 1;
    items_per_z = (int)((items + z - 1) / z);
    return (unsigned)((items + items_per_z - 1) / items_per_z);
}

// Conversion + column pass with the targets looped inside the workgroup (see modup_cols_kernel).
// mode 0: ModUp of `items` polynomials (y: [items][level][N], dst: [items][beta][E][N]);
// mode 1: DivRound conversion of `items` rows (y: row r at y + r*y_stride, dst: [rows][nc][N])
// mode 2: mode 1 in the exact form of DivRound; mode 3: ModDown followed by rescale as one conversion (D2 = the rescale).
// y is the output of the inverse row pass; the kernel runs the inverse column pass itself with the last-stage constants fin
// (fin_val: one set of constants passed by value for the single source of a rescale)
void launch_modup_cols(ckksmi_ctx *c, int mode, const u64 *y, size_t y_stride, u64 *dst, size_t items, int level, int nc,
                       const DivRoundDev *D, double units, hipStream_t st, const FinConst *fin, const DivRoundDev *D2 = nullptr,
                       const FinConst *fin_val = nullptr) {
    ModupColsArgs A;
    memset(&A, 0, sizeof(A));
    if (fin_val) { A.use_fin_val = 1; A.fin_val = *fin_val; }
    if (D2) { A.hc2 = D2->hc; A.hb2 = D2->hb[0]; }
    A.y = (const u64d *)y; A.y_row_stride = y_stride; A.dst = (u64d *)dst; A.modc = c->d_mod; A.tw = c->d_tww_fwd; A.cc = c->d_modup_c;
    A.logN = c->logN; A.level = level; A.E = level + c->k; A.n_q = c->n_q; A.alpha = c->alpha; A.T = c->T; A.nc = nc;
    A.beta = (level + c->alpha - 1) / c->alpha;
    A.p51 = c->p51mask;
    A.tw_inv = c->d_tww_inv; A.fin = fin;
    if (D) A.D = *D;
    const unsigned tiles = (unsigned)(c->N / 4096);
    const int n_targets = mode == 0 ? A.E : nc;
    const size_t ygrid = mode == 0 ? items * A.beta : items;
    // enough workgroups to fill the chip (8 per CU), otherwise as many targets per workgroup as possible: the source
    // tiles are read and converted once per workgroup (measured: 24 targets 0.65 ms, 6 targets 0.75 ms for ModDown)
    const size_t base = (size_t)tiles * ygrid;
    int chunks = (int)((size_t)2048 / (base ? base : 1));
    if (chunks < 1) chunks = 1;
    if (chunks > n_targets) chunks = n_targets;
    A.targets_per_wg = (n_targets + chunks - 1) / chunks;
    const unsigned z = (unsigned)((n_targets + A.targets_per_wg - 1) / A.targets_per_wg);
    const dim3 grid(tiles, (unsigned)ygrid, z), block(V2_THREADS);
    const int nsrc = mode == 0 ? c->alpha : D->nb;
    const int kid = mode == 0 ? CKKSMI_K_CONV_COLS_MODUP
                               : mode == 2 ? CKKSMI_K_CONV_COLS_MERGED
                               : mode == 3 ? CKKSMI_K_CONV_COLS_TAIL : (nsrc == 1 ? CKKSMI_K_CONV_COLS_RESCALE : CKKSMI_K_CONV_COLS_DIV);
#define MODUP_COLS_CASE(Q, NS)                                                                               \
    case (Q) * 8 + (NS):                                                                                     \
        if (mode == 0) KL(c, kid, units, (modup_cols_kernel<Q, NS, 0>), grid, block, st, A);                 \
        else if (mode == 2) KL(c, kid, units, (modup_cols_kernel<Q, NS, 2>), grid, block, st, A);            \
        else if (mode == 3) KL(c, kid, units, (modup_cols_kernel<Q, NS, 3>), grid, block, st, A);            \
        else KL(c, kid, units, (modup_cols_kernel<Q, NS, 1>), grid, block, st, A);                           \
        break;
    switch ((c->logN - 12) * 8 + nsrc) {
        MODUP_COLS_CASE(0, 1) MODUP_COLS_CASE(0, 2) MODUP_COLS_CASE(0, 3) MODUP_COLS_CASE(0, 4)
        MODUP_COLS_CASE(1, 1) MODUP_COLS_CASE(1, 2) MODUP_COLS_CASE(1, 3) MODUP_COLS_CASE(1, 4)
        MODUP_COLS_CASE(2, 1) MODUP_COLS_CASE(2, 2) MODUP_COLS_CASE(2, 3) MODUP_COLS_CASE(2, 4)
        MODUP_COLS_CASE(3, 1) MODUP_COLS_CASE(3, 2) MODUP_COLS_CASE(3, 3) MODUP_COLS_CASE(3, 4)
        MODUP_COLS_CASE(4, 1) MODUP_COLS_CASE(4, 2) MODUP_COLS_CASE(4, 3) MODUP_COLS_CASE(4, 4)
        default: break;
    }
#undef MODUP_COLS_CASE
}

// limb_count < 0: every limb, out laid out [rows][nc][N]; otherwise only limbs limb0 .. limb0+limb_count-1, written to
// out + row*out_row_stride + (limb - limb0)*N
void launch_rows_final(ckksmi_ctx *c, const u64 *tmpA, const u64 *x, size_t x_row_stride, const u64 *addend, size_t add_item_stride,
                       size_t add_comp_stride, int add_both, u64 *out, const WMul *Binv, int nc, int rows, hipStream_t st, int limb0 = 0,
                       int limb_count = -1, size_t out_row_stride = 0, const WMul *pre = nullptr, const WMul *xmul = nullptr,
                       const ScalarTab *stab = nullptr, bool zsub = false, const RowsFinalGal *gal = nullptr) {
    RowsFinalArgs A;
    A.zsub = zsub ? 1 : 0;
    A.pre = pre;
    A.xmul = xmul;
    const int nz = limb_count < 0 ? nc : limb_count;
    A.limb0 = limb_count < 0 ? 0 : limb0;
    A.out_limb0 = A.limb0;
    A.out_row_stride = limb_count < 0 ? (size_t)nc * c->N : out_row_stride;
    A.tmpA = (const u64d *)tmpA; A.x = (const u64d *)x; A.x_row_stride = x_row_stride;
    A.addend = (const u64d *)addend; A.add_item_stride = add_item_stride; A.add_comp_stride = add_comp_stride; A.add_both = add_both;
    A.out = (u64d *)out; A.modc = c->d_mod; A.tw = c->d_tww_fwd; A.Binv = Binv; A.logN = c->logN; A.nc = nc;
    A.rows = rows;
    A.p51 = c->p51mask;
    const unsigned tiles = (unsigned)(c->N / 4096);
    const unsigned xch = zchunks_for(c, tiles * nz, rows, A.rows_per_x);
    if (stab)
        KL(c, CKKSMI_K_ROWS_FINAL, (double)rows * nz, rows_final_scalar_kernel, dim3(xch, tiles, nz), dim3(V2_THREADS), st, A, *stab);
    else if (gal)
        KL(c, CKKSMI_K_ROWS_FINAL, (double)rows * nz, rows_final_gal_kernel, dim3(xch, tiles, nz), dim3(V2_THREADS), st, A, *gal);
    else
        KL(c, CKKSMI_K_ROWS_FINAL, (double)rows * nz, rows_final_kernel, dim3(xch, tiles, nz), dim3(V2_THREADS), st, A);
}

// DivRound of `rows` rows on the register-tiled kernels: dropped limbs (evaluation form) at b_limbs + r*b_stride (nb limbs;
// b_scratch == b_limbs works in place), kept limbs at x + r*x_stride; out[r][i] = (x_i - NTT(r_i - h)) * Bbar^-1 (+ addend).
// zsub: the kept limbs already hold x * Bbar^-1 + addend, out = x - NTT(r - h) * Bbar^-1.
void divround_rows(ckksmi_ctx *c, const DivRoundDev &D, const FinConst *fin, const int *bidx, const u64 *b_limbs, size_t b_stride,
                   u64 *b_scratch, size_t bs_stride, const u64 *x, size_t x_stride, u64 *tmp, int nc, int rows, const u64 *addend,
                   size_t add_item_stride, size_t add_comp_stride, int add_both, u64 *out, hipStream_t st, bool zsub = false,
                   const RowsFinalGal *gal = nullptr) {
    // inverse row pass of the dropped limbs; the conversion kernel runs their inverse column pass itself
    launch_ntt(c, false, b_limbs, b_scratch, table_map(bidx, D.nb, b_stride, bs_stride), rows, st, fin, 2);
    launch_modup_cols(c, 1, b_scratch, bs_stride, tmp, rows, 0, nc, &D, (double)rows * nc, st, fin);
    launch_rows_final(c, tmp, x, x_stride, addend, add_item_stride, add_comp_stride, add_both, out, D.Binv, nc, rows, st, 0, -1, 0, nullptr, nullptr,
                      nullptr, zsub, gal);
}

// Rotations with a shared ModUp: R rotations of every item of a key-switch sweep (see inner_product_hoisted_kernel)
struct HoistPlan {
    int R;
    unsigned g[CKKSMI_MAX_KEYS], ginv[CKKSMI_MAX_KEYS];
    const u64 *key[CKKSMI_MAX_KEYS];
    const u64 *sig;  // sigma_r(c0) of every item: [items][R][level][N], the addend of the first component (generic kernels)
    const u64 *c0;   // register-tiled sizes: the input ciphertexts (item stride c0_stride words), whose first component the
    size_t c0_stride;  // last pass reads through the automorphisms instead
};

// the gather through LDS needs runs of 256 words and at most INNER_MAX_BETA digits; otherwise the plain gather kernel
inline bool hoisted_tile_ok(const ckksmi_ctx *c, int beta) { return c->logN >= 8 && beta <= INNER_MAX_BETA && EW_THREADS == 256; }

void launch_hoisted_inner(ckksmi_ctx *c, const HoistPlan &H, const u64 *dt, const u64 *d_eval, size_t d_stride, u64 *acc, int items, int level,
                          hipStream_t st) {
    HoistArgs A;
    memset(&A, 0, sizeof(A));
    A.dt = (const u64d *)dt; A.d_eval = (const u64d *)d_eval; A.d_eval_item_stride = d_stride; A.acc = (u64d *)acc; A.modc = c->d_mod;
    A.logN = c->logN; A.level = level; A.E = level + c->k; A.n_q = c->n_q; A.alpha = c->alpha; A.beta = (level + c->alpha - 1) / c->alpha;
    A.T = c->T; A.items = items; A.R = H.R;
    for (int r = 0; r < H.R; r++) { A.g[r] = H.g[r]; A.ginv[r] = H.ginv[r]; A.key[r] = (const u64d *)H.key[r]; }
    if (hoisted_tile_ok(c, A.beta)) {
        // source rows staged in LDS once for all rotations
        A.items_per_wg = std::max(1, std::min(items, HOIST_LDS_WORDS / 256 / A.beta));
        A.item_chunks = (items + A.items_per_wg - 1) / A.items_per_wg;
        // few items: the rotations are spread over workgroups as well, until the chip is filled (each rotation chunk stages
        // the source runs again)
        const size_t base = (size_t)(c->N / 256) * A.E * A.item_chunks;
        int rot_chunks = (int)std::min<size_t>((size_t)H.R, (2048 + base - 1) / base);
        A.rots_per_wg = (H.R + rot_chunks - 1) / rot_chunks;
        rot_chunks = (H.R + A.rots_per_wg - 1) / A.rots_per_wg;
        const unsigned z = (unsigned)(A.item_chunks * rot_chunks);
        const int need = A.items_per_wg * A.beta * 256;  // staged words
        const dim3 grid((unsigned)(c->N / 256), A.E, z);
        const double work = (double)items * H.R * A.E;
#define HOIST_TILE(LW, MB) KL(c, CKKSMI_K_INNER_HOISTED, work, (inner_product_hoisted_tile_kernel<LW, MB>), grid, dim3(EW_THREADS), st, A)
#define HOIST_TILE_LW(MB)                      \
    do {                                       \
        if (need <= 1024) HOIST_TILE(1024, MB);       \
        else if (need <= 2048) HOIST_TILE(2048, MB);  \
        else if (need <= 4096) HOIST_TILE(4096, MB);  \
        else HOIST_TILE(HOIST_LDS_WORDS, MB);         \
    } while (0)
        if (A.beta <= 4) HOIST_TILE_LW(4);
        else if (A.beta <= 8) HOIST_TILE_LW(8);
        else HOIST_TILE_LW(INNER_MAX_BETA);
#undef HOIST_TILE_LW
#undef HOIST_TILE
        return;
    }
    KL(c, CKKSMI_K_INNER_HOISTED, (double)items * H.R * A.E, inner_product_hoisted_kernel, dim3(ew_blocks(c->N), A.E, H.R), dim3(EW_THREADS), st, A);
}

// The product's division in one step: acc [items][2][E][N] holds the key-switch accumulators over the extended basis
// (evaluation form) and d0, d1 (the addend) join them multiplied by P before the division by P*q_{level-1}:
//     out[items][2][level-1][N] = DivRound_B(acc + P*d),  B = {q_{level-1}, p_0 .. p_{k-1}},  exact form.
// The limbs of B are contiguous in the extended layout (limbs level-1 .. E-1); they are overwritten.
// addend == nullptr: acc already holds acc + P*d on the ciphertext limbs (the fused inner product's tensor mode).
void merged_division(ckksmi_ctx *c, u64 *acc, const u64 *addend, size_t add_item_stride, size_t add_comp_stride, u64 *out, u64 *tmp, int items,
                     int level, hipStream_t st) {
    const size_t N = c->N;
    const int E = level + c->k, rows = items * 2, nc = level - 1;
    const DivRoundDev &D = c->divround_merged[level];
    u64 *bl = acc + (size_t)(level - 1) * N;
    // only the dropped limb q_{level-1} needs acc + P*d up front; the kept limbs receive P*d in the last step
    if (addend)
    KL(c, CKKSMI_K_AXPY_LIMB, (double)rows, axpy_limb_kernel, dim3(ew_blocks(N / 2), rows), dim3(EW_THREADS), st, (u64d *)bl,
       (unsigned long long)((size_t)E * N), (const u64d *)(addend + (size_t)(level - 1) * N), (unsigned long long)add_item_stride,
       (unsigned long long)add_comp_stride, c->h_modc[level - 1], make_wmul(1, c->mod[level - 1]), c->h_pmod[level - 1], c->logN);
    if (c->fused) {
        const FinConst *fin = c->d_fin_merged + (size_t)level * CKKSMI_MAX_SPECIAL;
        launch_ntt(c, false, bl, bl, table_map(D.b_idx, D.nb, (size_t)E * N, (size_t)E * N), rows, st, fin, 2);
        launch_modup_cols(c, 2, bl, (size_t)E * N, tmp, rows, 0, nc, &D, (double)rows * nc, st, fin);
        launch_rows_final(c, tmp, acc, (size_t)E * N, addend, add_item_stride, add_comp_stride, 1, out, D.Binv, nc, rows, st, 0, -1, 0,
                          addend ? c->d_pmod : nullptr);
        return;
    }
    int idx[CKKSMI_MAX_MODULI];
    for (int i = 0; i < nc; i++) idx[i] = i;
    launch_ntt(c, false, bl, bl, table_map(D.b_idx, D.nb, (size_t)E * N, (size_t)E * N), rows, st);
    DivConvArgs DC;
    DC.b_limbs = (const u64d *)bl; DC.b_row_stride = (size_t)E * N; DC.tmp = (u64d *)tmp; DC.modc = c->d_mod; DC.D = D;
    DC.logN = c->logN; DC.nc = nc; DC.T = c->T; DC.exact = 1;
    KL(c, CKKSMI_K_DIVCONV, (double)rows * nc, divround_conv_kernel, dim3(ew_blocks(N), rows), dim3(EW_THREADS), st, DC);
    launch_ntt(c, true, tmp, tmp, table_map(idx, nc, (size_t)nc * N, (size_t)nc * N), rows, st);
    DivFinalArgs DF;
    DF.x = (const u64d *)acc; DF.x_row_stride = (size_t)E * N; DF.tmp = (const u64d *)tmp;
    DF.addend = (const u64d *)addend; DF.add_item_stride = add_item_stride; DF.add_comp_stride = add_comp_stride; DF.add_both = 1;
    DF.out = (u64d *)out; DF.modc = c->d_mod; DF.Binv = D.Binv; DF.pre = c->d_pmod; DF.logN = c->logN; DF.nc = nc;
    KL(c, CKKSMI_K_DIVFINAL, (double)rows * nc, divround_final_kernel, dim3(ew_blocks(N), nc, rows), dim3(EW_THREADS), st, DF);
}

// Can ModDown + add + rescale of a product run as one conversion and one last pass (modup_cols_kernel MODE 3)?  The dropped
// limb joins the special limbs as a conversion source, so one more than k sources must fit.
inline bool one_conversion_tail_ok(const ckksmi_ctx *c) { return c->fused && c->d_fin_tail != nullptr; }

// Key switch on the register-tiled kernels (2^12 <= N <= 2^16).
// tail: the key switch is followed by a rescale of (result + addend), both components have an addend, and `out` receives
// the rescaled ciphertexts [items][2][level-1][N] (needs one_conversion_tail_ok).
// ta != nullptr (the composite multiply; d_eval and addend unused): the polynomial switched is the third tensor component
// of the operands ta, tb ([items][terms][2][level][N]), whose inverse row pass the tensor kernel already left at the start of
// the workspace, and the other two components are the addends; the fused inner product forms all three from the operands.
void ks_core_fused(ckksmi_ctx *c, const u64 *d_eval, size_t d_stride, const KeyTab &K, int items, int level, const u64 *addend,
                   size_t add_item_stride, size_t add_comp_stride, int add_both, u64 *out, u64 *ws, hipStream_t st,
                   bool tail = false, bool merged = false, const HoistPlan *hoist = nullptr, const u64 *ta = nullptr, const u64 *tb = nullptr,
                   int terms = 1, const GaloisTab *gal = nullptr) {
    const size_t N = c->N;
    const int E = level + c->k, beta = (level + c->alpha - 1) / c->alpha;
    const int R = hoist ? hoist->R : 1;  // hoisted rotations: R accumulator pairs per item
    u64 *ymid = ws;
    u64 *dtA = ymid + (size_t)items * level * N;
    u64 *acc = dtA + (size_t)items * beta * E * N;
    u64 *tmp = acc + (size_t)items * R * 2 * E * N;
    int idx[CKKSMI_MAX_MODULI];
    for (int i = 0; i < level; i++) idx[i] = i;
    // y_i = d_i * qhat_i^-1 comes straight out of the inverse transform (row pass here, column pass inside the conversion
    // kernel); the conversion rides on the column pass of the forward transform of its results
    const FinConst *fin_up = c->d_fin_modup + (size_t)level * c->n_q;
    if (!ta) launch_ntt(c, false, d_eval, ymid, table_map(idx, level, d_stride, (size_t)level * N), items, st, fin_up, 2, gal);
    launch_modup_cols(c, 0, ymid, 0, dtA, items, level, 0, nullptr, (double)items * (beta * E - level), st, fin_up);
    int sidx[CKKSMI_MAX_SPECIAL];
    for (int m = 0; m < c->k; m++) sidx[m] = c->n_q + m;
    u64 *specials = acc + (size_t)level * N;
    if (hoist) {
        // the lifted digits in evaluation form once, then every rotation gathers from them
        LimbMap M1;
        memset(&M1, 0, sizeof(M1));
        M1.per_item = beta * E; M1.mode = 1; M1.level = level; M1.E = E; M1.n_q = c->n_q; M1.alpha = c->alpha;
        M1.src_item_stride = M1.dst_item_stride = (size_t)beta * E * N;
        launch_ntt(c, true, dtA, dtA, M1, items, st, nullptr, 2);
        launch_hoisted_inner(c, *hoist, dtA, d_eval, d_stride, acc, items, level, st);
        RowsFinalGal FG;
        FG.R = R;
        for (int r = 0; r < CKKSMI_MAX_KEYS; r++) FG.g[r] = r < R ? hoist->g[r] : 1u;
        divround_rows(c, c->divround[0], c->d_fin_moddown, sidx, specials, (size_t)E * N, specials, (size_t)E * N, acc, (size_t)E * N, tmp, level,
                      items * R * 2, hoist->c0, hoist->c0_stride, 0, 0, out, st, false, &FG);
        return;
    }
    RowsInnerArgs RI;
    RI.dtA = (const u64d *)dtA; RI.d_eval = (const u64d *)d_eval; RI.d_eval_item_stride = d_stride; RI.acc = (u64d *)acc;
    RI.modc = c->d_mod; RI.tw = c->d_tww_fwd;
    RI.logN = c->logN; RI.level = level; RI.E = E; RI.n_q = c->n_q; RI.alpha = c->alpha; RI.beta = beta; RI.T = c->T;
    const unsigned tiles = (unsigned)(N / 4096);
    RI.kt = tiles < 8 ? tiles : 8;
    RI.p51 = c->p51mask;
    // the ciphertext limbs leave the inner product as z = x * P^-1 + addend, which is what ModDown's last pass (and the
    // one-conversion tail) read; the merged division wants the accumulators themselves
    RI.fold_tail = (merged || !addend || ta) ? 0 : (add_both ? 1 : 2);
    RI.Pinv = c->divround[0].Binv;
    RI.addend = (const u64d *)addend; RI.add_item_stride = add_item_stride; RI.add_comp_stride = add_comp_stride;
    RI.ta = (const u64d *)ta; RI.tb = (const u64d *)tb; RI.terms = terms; RI.keep_acc = merged ? 1 : 0; RI.Pmod = c->d_pmod;
    if (gal) KL(c, CKKSMI_K_ROWS_INNER, (double)items * E, rows_inner_gal_kernel, dim3(RI.kt * items, tiles / RI.kt, E), dim3(V2_THREADS), st, RI, K, *gal);
    else KL(c, CKKSMI_K_ROWS_INNER, (double)items * E, rows_inner_kernel, dim3(RI.kt * items, tiles / RI.kt, E), dim3(V2_THREADS), st, RI, K);
    if (merged) {
        merged_division(c, acc, ta ? nullptr : addend, add_item_stride, add_comp_stride, out, tmp, items, level, st);
        return;
    }
    const int rows = items * 2;
    if (tail) {
        // ONE conversion and ONE last pass for ModDown + add + rescale (same bits; see modup_cols_kernel MODE 3):
        // u = x_last * P^-1 + d_last (written by the inner product) stands in place of the dropped limb, its inverse
        // transform rides with the special limbs' (limbs last, p_0 .. p_{k-1} of every row are neighbours)
        const int last = level - 1;
        u64 *bl = acc + (size_t)last * N;
        const DivRoundDev &DB = c->divround[1 + last];
        DivRoundDev D3 = c->divround[0];
        D3.nb = c->k + 1;
        D3.b_idx[0] = last;
        for (int m = 0; m < c->k; m++) D3.b_idx[1 + m] = c->n_q + m;
        const FinConst *ft = c->d_fin_tail + (size_t)level * CKKSMI_MAX_SPECIAL;
        launch_ntt(c, false, bl, bl, table_map(D3.b_idx, D3.nb, (size_t)E * N, (size_t)E * N), rows, st, ft, 2);
        launch_modup_cols(c, 3, bl, (size_t)E * N, tmp, rows, 0, last, &D3, (double)rows * last, st, ft, &DB);
        launch_rows_final(c, tmp, acc, (size_t)E * N, nullptr, 0, 0, 0, out, DB.Binv, last, rows, st);
        return;
    }
    // plain ModDown; with an addend the kept limbs already hold x * P^-1 + addend
    divround_rows(c, c->divround[0], c->d_fin_moddown, sidx, specials, (size_t)E * N, specials, (size_t)E * N, acc, (size_t)E * N, tmp, level, rows,
                  nullptr, 0, 0, 0, out, st, addend != nullptr || ta != nullptr);
}

void rescale_core_fused(ckksmi_ctx *c, const u64 *a, u64 *out, int items, int level, u64 *ws, hipStream_t st) {
    const size_t N = c->N;
    u64 *last = ws;
    u64 *tmp = last + (size_t)items * 2 * N;
    int lidx[1] = {level - 1};
    divround_rows(c, c->divround[1 + (level - 1)], c->d_fin_rescale + (level - 1), lidx, a + (size_t)(level - 1) * N, (size_t)level * N, last,
                  N, a, (size_t)level * N, tmp, level - 1, items * 2, nullptr, 0, 0, 0, out, st);
}

// out = DivRound_{q_{level-1}}(v * a) without materialising v*a: the dropped limb's inverse transform multiplies by v in its
// last stage (per-call constants), the last pass multiplies the kept limb by v before the subtraction
void scalar_rescale_fused(ckksmi_ctx *c, const u64 *a, int64_t v, const u64 *addend, u64 *out, int items, int level_in, int level, u64 *ws,
                          hipStream_t st) {
    const size_t N = c->N;
    const size_t in_stride = (size_t)level_in * N;  // the input rows hold level_in limbs, of which the first `level` are used
    const int last = level - 1, rows = items * 2;
    u64 *lastbuf = ws;
    u64 *tmp = lastbuf + (size_t)rows * N;
    int lidx[1] = {last};
    const DivRoundDev &D = c->divround[1 + last];
    const u64 q = c->mod[last], vm = hm::signed_mod(v, q);
    FinConst F;
    F.ninv = make_wmul(hm::mulmod(c->h_ninv[last], vm, q), q);
    F.wlast = make_wmul(hm::mulmod(hm::mulmod(c->h_inv[last][1], c->h_ninv[last], q), vm, q), q);
    F.cadd = (double)((q - 1) / 2);
    F.pad = 0.0;
    const ScalarTab St = scalar_tab(c, v, level);
    launch_ntt(c, false, a + (size_t)last * N, lastbuf, table_map(lidx, 1, in_stride, N), rows, st, c->d_fin_rescale + last, 2);
    launch_modup_cols(c, 1, lastbuf, N, tmp, rows, 0, last, &D, (double)rows * last, st, c->d_fin_rescale + last, nullptr, &F);
    launch_rows_final(c, tmp, a, in_stride, addend, (size_t)2 * last * N, (size_t)last * N, 1, out, D.Binv, last, rows, st, 0, -1, 0, nullptr, nullptr,
                      &St);
}

// Key switch of `items` polynomials.  d_eval: item i's polynomial ([level][N], evaluation
// form) at d_eval + i*d_stride.  out[i][c][l] = ks_c (+ addend).  ws: ks_words_per_item*items.
void ks_core(ckksmi_ctx *c, const u64 *d_eval, size_t d_stride, const KeyTab &K, int items, int level, const u64 *addend,
             size_t add_item_stride, size_t add_comp_stride, int add_both, u64 *out, u64 *ws, hipStream_t st, bool merged = false,
             const HoistPlan *hoist = nullptr) {
    if (c->fused) {
        ks_core_fused(c, d_eval, d_stride, K, items, level, addend, add_item_stride, add_comp_stride, add_both, out, ws, st, false, merged, hoist);
        return;
    }
    // other ring sizes: the generic kernels, one step after the other
    const size_t N = c->N;
    const int E = level + c->k, beta = (level + c->alpha - 1) / c->alpha;
    const int rows = items * 2 * (hoist ? hoist->R : 1);
    u64 *dcoef = ws;
    u64 *dt = dcoef + (size_t)items * level * N;
    u64 *acc = dt + (size_t)items * beta * E * N;
    u64 *tmp = acc + (size_t)rows * E * N;
    if (hoist) {
        addend = hoist->sig; add_item_stride = (size_t)level * N; add_comp_stride = 0; add_both = 0;
    }
    int idx[CKKSMI_MAX_MODULI];
    for (int i = 0; i < level; i++) idx[i] = i;
    // 1. d -> coefficient form
    launch_ntt(c, false, d_eval, dcoef, table_map(idx, level, d_stride, (size_t)level * N), items, st);
    // 2. ModUp every digit
    ModUpArgs MU;
    MU.d_coef = (const u64d *)dcoef;
    MU.d_eval = (const u64d *)d_eval;
    MU.d_eval_item_stride = d_stride;
    MU.out = (u64d *)dt;
    MU.modc = c->d_mod;
    MU.inv = c->d_modup_inv;
    MU.cc = c->d_modup_c;
    MU.logN = c->logN; MU.level = level; MU.E = E; MU.n_q = c->n_q; MU.alpha = c->alpha; MU.beta = beta; MU.T = c->T;
    KL(c, CKKSMI_K_MODUP, (double)items * beta * E, modup_kernel, dim3(ew_blocks(N), beta, items), dim3(EW_THREADS), st, MU);
    // 3. converted limbs -> evaluation form (limbs of the digit itself were copied as such)
    LimbMap M1;
    memset(&M1, 0, sizeof(M1));
    M1.per_item = beta * E; M1.mode = 1; M1.level = level; M1.E = E; M1.n_q = c->n_q; M1.alpha = c->alpha;
    M1.src_item_stride = M1.dst_item_stride = (size_t)beta * E * N;
    launch_ntt(c, true, dt, dt, M1, items, st);
    // 4. inner product with the key (hoisted rotations: one per rotation, gathered through its automorphism)
    if (hoist) {
        launch_hoisted_inner(c, *hoist, dt, nullptr, 0, acc, items, level, st);
    } else {
        InnerArgs IA;
        IA.dt = (const u64d *)dt; IA.d_eval = nullptr; IA.d_eval_item_stride = 0; IA.alpha = c->alpha; IA.acc = (u64d *)acc; IA.modc = c->d_mod;
        IA.logN = c->logN; IA.level = level; IA.E = E; IA.n_q = c->n_q; IA.beta = beta; IA.T = c->T;
        IA.items = items;
        const unsigned zin = zchunks_for(c, ew_blocks(N) * E, items, IA.items_per_z);
        KL(c, CKKSMI_K_INNER, (double)items * E, inner_product_kernel, dim3(ew_blocks(N), E, zin), dim3(EW_THREADS), st, IA, K);
    }
    if (merged) {
        merged_division(c, acc, addend, add_item_stride, add_comp_stride, out, tmp, items, level, st);
        return;
    }
    // 5. ModDown: special limbs -> coefficient form, convert, back to evaluation form, combine
    int sidx[CKKSMI_MAX_SPECIAL];
    for (int m = 0; m < c->k; m++) sidx[m] = c->n_q + m;
    launch_ntt(c, false, acc + (size_t)level * N, acc + (size_t)level * N, table_map(sidx, c->k, (size_t)E * N, (size_t)E * N),
               (size_t)rows, st);
    DivConvArgs DC;
    DC.b_limbs = (const u64d *)(acc + (size_t)level * N);
    DC.b_row_stride = (size_t)E * N;
    DC.tmp = (u64d *)tmp;
    DC.modc = c->d_mod;
    DC.D = c->divround[0];
    DC.logN = c->logN; DC.nc = level; DC.T = c->T; DC.exact = 0;
    KL(c, CKKSMI_K_DIVCONV, (double)rows * DC.nc, divround_conv_kernel, dim3(ew_blocks(N), rows), dim3(EW_THREADS), st, DC);
    launch_ntt(c, true, tmp, tmp, table_map(idx, level, (size_t)level * N, (size_t)level * N), (size_t)rows, st);
    DivFinalArgs DF;
    DF.x = (const u64d *)acc; DF.x_row_stride = (size_t)E * N;
    DF.tmp = (const u64d *)tmp;
    DF.addend = (const u64d *)addend; DF.add_item_stride = add_item_stride; DF.add_comp_stride = add_comp_stride;
    DF.add_both = add_both;
    DF.out = (u64d *)out;
    DF.modc = c->d_mod; DF.Binv = c->divround[0].Binv; DF.pre = nullptr;
    DF.logN = c->logN; DF.nc = level;
    KL(c, CKKSMI_K_DIVFINAL, (double)rows * DF.nc, divround_final_kernel, dim3(ew_blocks(N), level, rows), dim3(EW_THREADS), st, DF);
}

// out[i] = DivRound_{q_{level-1}}(a[i]); ws: rescale_words_per_item*items
void rescale_core(ckksmi_ctx *c, const u64 *a, u64 *out, int items, int level, u64 *ws, hipStream_t st) {
    if (c->fused) {
        rescale_core_fused(c, a, out, items, level, ws, st);
        return;
    }
    const size_t N = c->N;
    u64 *last = ws;
    u64 *tmp = last + (size_t)items * 2 * N;
    int lidx[1] = {level - 1};
    launch_ntt(c, false, a + (size_t)(level - 1) * N, last, table_map(lidx, 1, (size_t)level * N, N), (size_t)items * 2, st);
    DivConvArgs DC;
    DC.b_limbs = (const u64d *)last; DC.b_row_stride = N;
    DC.tmp = (u64d *)tmp; DC.modc = c->d_mod;
    DC.D = c->divround[1 + (level - 1)];
    DC.logN = c->logN; DC.nc = level - 1; DC.T = c->T; DC.exact = 0;
    KL(c, CKKSMI_K_DIVCONV, (double)items * 2 * DC.nc, divround_conv_kernel, dim3(ew_blocks(N), items * 2), dim3(EW_THREADS), st, DC);
    int idx[CKKSMI_MAX_MODULI];
    for (int i = 0; i < level - 1; i++) idx[i] = i;
    launch_ntt(c, true, tmp, tmp, table_map(idx, level - 1, (size_t)(level - 1) * N, (size_t)(level - 1) * N), (size_t)items * 2, st);
    DivFinalArgs DF;
    DF.x = (const u64d *)a; DF.x_row_stride = (size_t)level * N;
    DF.tmp = (const u64d *)tmp;
    DF.addend = nullptr; DF.add_item_stride = DF.add_comp_stride = 0; DF.add_both = 0;
    DF.out = (u64d *)out;
    DF.modc = c->d_mod; DF.Binv = c->divround[1 + (level - 1)].Binv; DF.pre = nullptr;
    DF.logN = c->logN; DF.nc = level - 1;
    KL(c, CKKSMI_K_DIVFINAL, (double)items * 2 * DF.nc, divround_final_kernel, dim3(ew_blocks(N), level - 1, items * 2), dim3(EW_THREADS), st, DF);
}

// terms > 1: a, b hold [items][terms][2][level][N] and d receives the sum of the terms' tensors
void launch_tensor(ckksmi_ctx *c, const u64 *a, const u64 *b, u64 *d, int level, int items, hipStream_t st, int terms = 1) {
    const size_t total = (size_t)items * level * c->N / 2;  // word pairs
    KL(c, CKKSMI_K_TENSOR, (double)items * level * terms, tensor_kernel, dim3(ew_blocks(total)), dim3(EW_THREADS), st, (const u64d *)a, (const u64d *)b, (u64d *)d, c->d_mod,
                  c->logN, level, total, terms);
}

// third tensor component + its inverse row pass into ymid (see tensor_rows_kernel); register-tiled sizes only
void launch_tensor_rows(ckksmi_ctx *c, const u64 *a, const u64 *b, u64 *ymid, int level, int items, hipStream_t st, int terms = 1) {
    TensorRowsArgs A;
    A.terms = terms;
    A.a = (const u64d *)a; A.b = (const u64d *)b; A.ymid = (u64d *)ymid; A.modc = c->d_mod; A.tw_inv = c->d_tww_inv;
    A.logN = c->logN; A.level = level; A.p51 = c->p51mask;
    KL(c, CKKSMI_K_TENSOR_ROWS, (double)items * level, tensor_rows_kernel, dim3((unsigned)(c->N / 4096), level, items), dim3(V2_THREADS), st, A);
}

int sweep_items(size_t ws_bytes, size_t words_per_item, int batch) {
    size_t fit = ws_bytes / 8 / words_per_item;
    if (fit > (size_t)batch) fit = batch;
    if (fit > CKKSMI_MAX_ITEMS) fit = CKKSMI_MAX_ITEMS;
    return (int)fit;
}

u64 galois_element_of(const ckksmi_ctx *c, int rot) {
    const i64 half = (i64)(c->N / 2);
    i64 r = ((i64)rot % half + half) % half;
    return hm::powmod(5, (u64)r, 2 * c->N);
}
int norm_rot(const ckksmi_ctx *c, int rot) {
    const i64 half = (i64)(c->N / 2);
    return (int)(((i64)rot % half + half) % half);
}

}  // namespace

// ------------------------------------------------------------------ tables
int dev_upload_tables(ckksmi_ctx *c) {
    if (hipSetDevice(c->device) != hipSuccess) return CKKSMI_EDEVICE;
    if (!lookup_static_scratch(c->device)) { c->last_hip_error = (int)hipGetLastError(); return CKKSMI_EDEVICE; }
    bool ok = true;
    const size_t N = c->N;
    const int T = c->T;
    c->d_mod = upload(c, c->h_modc, T, ok);
    {
        std::vector<WMul> p24(T);
        for (int t = 0; t < T; t++) p24[t] = make_wmul(((u64)1 << 24) % c->mod[t], c->mod[t]);
        c->d_pow24 = upload(c, p24.data(), p24.size(), ok);
    }
    for (int t = 0; t < T; t++)
        if (c->mod[t] >= ((u64)1 << 50)) c->p51mask.w[t >> 6] |= 1ull << (t & 63);
    std::vector<WMul> fwd((size_t)T * N), inv((size_t)T * N), last(T);
    for (int t = 0; t < T; t++) {
        const u64 q = c->mod[t];
        for (size_t x = 0; x < N; x++) {
            fwd[(size_t)t * N + x] = make_wmul(c->h_fwd[t][x], q);
            inv[(size_t)t * N + x] = make_wmul(c->h_inv[t][x], q);
        }
        inv[(size_t)t * N] = make_wmul(c->h_ninv[t], q);
        last[t] = make_wmul(hm::mulmod(c->h_inv[t][1], c->h_ninv[t], q), q);
    }
    c->d_tw_fwd = upload(c, fwd.data(), fwd.size(), ok);
    c->d_tw_inv = upload(c, inv.data(), inv.size(), ok);
    c->d_tw_inv_last = upload(c, last.data(), last.size(), ok);
    {
        std::vector<double> fw((size_t)T * N), iw((size_t)T * N);
        std::vector<WMul> ni(T);
        for (int t = 0; t < T; t++) {
            for (size_t x = 0; x < N; x++) {
                fw[(size_t)t * N + x] = make_wmul(c->h_fwd[t][x], c->mod[t]).w;
                iw[(size_t)t * N + x] = make_wmul(c->h_inv[t][x], c->mod[t]).w;
            }
            ni[t] = make_wmul(c->h_ninv[t], c->mod[t]);
        }
        c->d_tww_fwd = upload(c, fw.data(), fw.size(), ok);
        c->d_tww_inv = upload(c, iw.data(), iw.size(), ok);
        c->d_tw_ninv = upload(c, ni.data(), ni.size(), ok);
    }
    if (c->k > 0) {
        std::vector<WMul> mi, mc;
        make_modup_tables(c, mi, mc);
        c->d_modup_inv = upload(c, mi.data(), mi.size(), ok);
        c->d_modup_c = upload(c, mc.data(), mc.size(), ok);
    }
    // DivRound tables: 0 = ModDown over the special primes, 1+i = rescale dropping q_i
    auto upload_divround = [&](const std::vector<int> &b) {
        DivRoundHost h = make_divround(c, b);
        DivRoundDev d;
        memset(&d, 0, sizeof(d));
        d.nb = h.nb;
        for (int m = 0; m < h.nb; m++) {
            d.b_idx[m] = h.b_idx[m]; d.hb[m] = h.hb[m]; d.invb[m] = h.invb[m];
            d.invb_f[m] = 1.0 / (double)c->mod[h.b_idx[m]];
        }
        d.conv = upload(c, h.conv.data(), h.conv.size(), ok);
        d.hc = upload(c, h.hc.data(), h.hc.size(), ok);
        d.Binv = upload(c, h.Binv.data(), h.Binv.size(), ok);
        d.Bmod = upload(c, h.Bmod.data(), h.Bmod.size(), ok);
        return d;
    };
    c->divround.assign(1 + c->n_q, DivRoundDev());
    for (int which = 0; which <= c->n_q; which++) {
        std::vector<int> b;
        if (which == 0) {
            for (int m = 0; m < c->k; m++) b.push_back(c->n_q + m);
            if (b.empty()) { memset(&c->divround[0], 0, sizeof(DivRoundDev)); continue; }
        } else {
            b.push_back(which - 1);
        }
        c->divround[which] = upload_divround(b);
    }
    // merged division of the product (ModDown and rescale at once): level l drops {q_{l-1}, p_0 .. p_{k-1}}
    c->divround_merged.assign(1 + c->n_q, DivRoundDev());
    c->h_pmod.assign(T, WMul{0.0, 0.0});
    c->h_Pinv.assign(T, WMul{0.0, 0.0});
    c->merged_ok = c->k > 0 && c->k + 1 <= CKKSMI_MAX_SPECIAL;
    if (c->merged_ok)
        for (int level = 2; level <= c->n_q; level++) {
            std::vector<int> b(1, level - 1);
            for (int m = 0; m < c->k; m++) b.push_back(c->n_q + m);
            c->divround_merged[level] = upload_divround(b);
        }
    if (c->k > 0) {
        for (int i = 0; i < c->n_q; i++) {
            u64 P = 1;
            for (int m = 0; m < c->k; m++) P = hm::mulmod(P, c->mod[c->n_q + m] % c->mod[i], c->mod[i]);
            c->h_pmod[i] = make_wmul(P, c->mod[i]);
            c->h_Pinv[i] = make_wmul(hm::invmod(P, c->mod[i]), c->mod[i]);
        }
        c->d_pmod = upload(c, c->h_pmod.data(), c->h_pmod.size(), ok);
    }
    // register-tiled sizes: constants folded into the last stage of the inverse transforms
    c->fused = c->logN >= 12 && c->logN <= 16;
    if (c->fused) {
        auto fin = [&](int t, u64 mult, u64 add) {
            const u64 q = c->mod[t];
            FinConst f;
            f.ninv = make_wmul(hm::mulmod(c->h_ninv[t], mult, q), q);
            f.wlast = make_wmul(hm::mulmod(hm::mulmod(c->h_inv[t][1], c->h_ninv[t], q), mult, q), q);
            f.cadd = (double)add;
            f.pad = 0.0;
            return f;
        };
        std::vector<FinConst> fm((size_t)(c->n_q + 1) * c->n_q, fin(0, 1, 0));
        for (int level = 1; level <= c->n_q; level++)
            for (int i = 0; i < level; i++) {
                const int lo = (i / c->alpha) * c->alpha;
                const int nd = std::min(c->alpha, level - lo);
                const u64 q = c->mod[i];
                u64 hat = 1;
                for (int b = 0; b < nd; b++)
                    if (lo + b != i) hat = hm::mulmod(hat, c->mod[lo + b] % q, q);
                fm[(size_t)level * c->n_q + i] = fin(i, hm::invmod(hat, q), 0);
            }
        c->d_fin_modup = upload(c, fm.data(), fm.size(), ok);
        std::vector<FinConst> fd;
        for (int m = 0; m < c->k; m++) {
            const int t = c->n_q + m;
            const u64 bm = c->mod[t];
            u64 bhat = 1;
            for (int m2 = 0; m2 < c->k; m2++)
                if (m2 != m) bhat = hm::mulmod(bhat, c->mod[c->n_q + m2] % bm, bm);
            const u64 inv = hm::invmod(bhat, bm);
            fd.push_back(fin(t, inv, hm::mulmod((bm - 1) / 2, inv, bm)));
        }
        c->d_fin_moddown = upload(c, fd.data(), fd.size(), ok);
        std::vector<FinConst> fr;
        for (int i = 0; i < c->n_q; i++) fr.push_back(fin(i, 1, (c->mod[i] - 1) / 2));
        c->d_fin_rescale = upload(c, fr.data(), fr.size(), ok);
        if (c->k > 0 && c->k + 1 <= CKKSMI_MAX_SPECIAL) {
            std::vector<FinConst> ft((size_t)(c->n_q + 1) * CKKSMI_MAX_SPECIAL, fin(0, 1, 0));
            for (int level = 1; level <= c->n_q; level++) {
                ft[(size_t)level * CKKSMI_MAX_SPECIAL] = fin(level - 1, 1, 0);
                for (int m = 0; m < c->k; m++) ft[(size_t)level * CKKSMI_MAX_SPECIAL + 1 + m] = fd[m];
            }
            c->d_fin_tail = upload(c, ft.data(), ft.size(), ok);
        }
        if (c->merged_ok) {
            std::vector<FinConst> fg((size_t)(c->n_q + 1) * CKKSMI_MAX_SPECIAL, fin(0, 1, 0));
            for (int level = 2; level <= c->n_q; level++) {
                const DivRoundDev &D = c->divround_merged[level];
                for (int m = 0; m < D.nb; m++) {
                    const int t = D.b_idx[m];
                    const u64 bm = c->mod[t];
                    u64 bhat = 1;
                    for (int m2 = 0; m2 < D.nb; m2++)
                        if (m2 != m) bhat = hm::mulmod(bhat, c->mod[D.b_idx[m2]] % bm, bm);
                    const u64 inv = hm::invmod(bhat, bm);
                    fg[(size_t)level * CKKSMI_MAX_SPECIAL + m] = fin(t, inv, hm::mulmod((bm - 1) / 2, inv, bm));
                }
            }
            c->d_fin_merged = upload(c, fg.data(), fg.size(), ok);
        }
    }
    {
        // device-side encoding: slot exponents and the complex twiddles of the inverse transform
        std::vector<unsigned> se(N / 2 ? N / 2 : 1);
        u64 e = 1;
        for (size_t k = 0; k < N / 2; k++) { se[k] = (unsigned)e; e = (e * 5) % (2 * N); }
        c->d_slot_exp = upload(c, se.data(), se.size(), ok);
        std::vector<double> ctw(2 * N);
        const long double pi = acosl(-1.0L);
        for (size_t x = 0; x < N; x++) {
            const long double ang = pi * (long double)hm::brev(x, c->logN) / (long double)N;
            ctw[2 * x] = (double)cosl(ang);
            ctw[2 * x + 1] = (double)(-sinl(ang));
        }
        c->d_ctw = upload(c, ctw.data(), ctw.size(), ok);
        const int zeros[CKKSMI_FLAG_SLOTS] = {0};
        c->d_flag = upload(c, zeros, CKKSMI_FLAG_SLOTS, ok);
    }
    if (!ok) { c->last_hip_error = (int)hipGetLastError(); return CKKSMI_EDEVICE; }
    return CKKSMI_OK;
}

void dev_free_tables(ckksmi_ctx *c) {
    for (ProfRec &r : c->prof) { (void)hipEventDestroy((hipEvent_t)r.start); (void)hipEventDestroy((hipEvent_t)r.stop); }
    c->prof.clear();
    for (void *p : c->dev_allocs) (void)hipFree(p);
    c->dev_allocs.clear();
}

// ------------------------------------------------------------------ C ABI, device side
// device buffers must be 16-byte aligned (two-word vector accesses)
static inline bool al16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

extern "C" int ckksmi_galois_key_register(ckksmi_ctx *c, int rot, const uint64_t *gk_dev) {
    if (!c || !gk_dev || !al16(gk_dev)) return CKKSMI_EINVAL;
    if (c->k == 0) return CKKSMI_EUNSUPPORTED;
    const int r = norm_rot(c, rot);
    for (auto &e : c->galois)
        if (e.first == r) { e.second = gk_dev; return CKKSMI_OK; }
    c->galois.push_back(std::make_pair(r, (const u64 *)gk_dev));
    return CKKSMI_OK;
}

static int ntt_api(ckksmi_ctx *c, bool fwd, uint64_t *limbs, const int *index, int n_limbs, int batch, void *stream) {
    if (!c || !limbs || !al16(limbs) || !index || n_limbs < 1 || n_limbs > CKKSMI_MAX_MODULI || batch < 0) return CKKSMI_EINVAL;
    if (!dev_ok(c)) return CKKSMI_EDEVICE;
    for (int i = 0; i < n_limbs; i++)
        if (index[i] < 0 || index[i] >= c->T) return CKKSMI_EINVAL;
    if ((size_t)batch * n_limbs > 0x7fffffffu) return CKKSMI_EINVAL;
    Guard g(c);
    const size_t stride = (size_t)n_limbs * c->N;
    launch_ntt(c, fwd, limbs, limbs, table_map(index, n_limbs, stride, stride), batch, S(stream));
    return g.rc();
}
extern "C" int ckksmi_ntt(ckksmi_ctx *c, uint64_t *limbs, const int *index, int n_limbs, int batch, void *stream) {
    return ntt_api(c, true, limbs, index, n_limbs, batch, stream);
}
extern "C" int ckksmi_intt(ckksmi_ctx *c, uint64_t *limbs, const int *index, int n_limbs, int batch, void *stream) {
    return ntt_api(c, false, limbs, index, n_limbs, batch, stream);
}

static int ct_args_ok(const ckksmi_ctx *c, int level, int batch) {
    if (!c || batch < 0) return CKKSMI_EINVAL;
    if (!dev_ok(c)) return CKKSMI_EDEVICE;
    if (level < 1 || level > c->n_q) return CKKSMI_ELEVEL;
    if ((size_t)batch * 3 * level * c->N / EW_THREADS > 0x7fffffffu) return CKKSMI_EINVAL;
    return CKKSMI_OK;
}

static int addsub_api(ckksmi_ctx *c, const uint64_t *a, const uint64_t *b, uint64_t *out, int level, int batch, void *stream, int sub) {
    int rc = ct_args_ok(c, level, batch);
    if (rc) return rc;
    if (!a || !b || !out) return CKKSMI_EINVAL;
    if (batch == 0) return CKKSMI_OK;
    Guard g(c);
    const size_t total = (size_t)batch * 2 * level * c->N;
    KL(c, CKKSMI_K_ELEMWISE, (double)batch * 2 * level, addsub_kernel, dim3(ew_blocks(total)), dim3(EW_THREADS), S(stream), (const u64d *)a, (const u64d *)b, (u64d *)out,
                  c->d_mod, c->logN, level, total, sub);
    return g.rc();
}
extern "C" int ckksmi_add(ckksmi_ctx *c, const uint64_t *a, const uint64_t *b, uint64_t *out, int level, int batch, void *stream) {
    return addsub_api(c, a, b, out, level, batch, stream, 0);
}
extern "C" int ckksmi_sub(ckksmi_ctx *c, const uint64_t *a, const uint64_t *b, uint64_t *out, int level, int batch, void *stream) {
    return addsub_api(c, a, b, out, level, batch, stream, 1);
}

extern "C" int ckksmi_mul_plain(ckksmi_ctx *c, const uint64_t *a, const uint64_t *pt, size_t pt_stride, uint64_t *out, int level,
                                int batch, void *stream) {
    int rc = ct_args_ok(c, level, batch);
    if (rc) return rc;
    if (!a || !pt || !out) return CKKSMI_EINVAL;
    if (batch == 0) return CKKSMI_OK;
    Guard g(c);
    const size_t total = (size_t)batch * 2 * level * c->N;
    KL(c, CKKSMI_K_ELEMWISE, (double)batch * 2 * level, mul_plain_kernel, dim3(ew_blocks(total)), dim3(EW_THREADS), S(stream), (const u64d *)a, (const u64d *)pt, pt_stride,
                  (u64d *)out, c->d_mod, c->logN, level, total);
    return g.rc();
}

extern "C" int ckksmi_plain_mac(ckksmi_ctx *c, const uint64_t *cts, int n_ct, const uint64_t *pts, int n_pts, const int32_t *term, int n_groups,
                                uint64_t *out, int level, void *stream) {
    int rc = ct_args_ok(c, level, n_groups);
    if (rc) return rc;
    if (n_ct < 1 || n_pts < 0) return CKKSMI_EINVAL;
    if (!cts || !out || !term || (n_pts && !pts) || !al16(cts) || !al16(pts) || !al16(out)) return CKKSMI_EINVAL;
    if (n_groups == 0) return CKKSMI_OK;
    if ((n_groups + PM_GROUPS - 1) / PM_GROUPS > 65535 || level > 65535 || c->N < 2) return CKKSMI_EUNSUPPORTED;  // words go in pairs
    const size_t ct_words = 2 * (size_t)level * c->N;
    if (out < cts + (size_t)n_ct * ct_words && cts < out + (size_t)n_groups * ct_words) return CKKSMI_EINVAL;  // the sums read every input
    Guard g(c);
    KL(c, CKKSMI_K_ELEMWISE, (double)n_pts * 2 * level, plain_mac_kernel, dim3(ew_blocks(c->N / 2), level, (n_groups + PM_GROUPS - 1) / PM_GROUPS),
       dim3(EW_THREADS), S(stream), (const u64d *)cts, n_ct, (const u64d *)pts, n_pts, (const int *)term, n_groups, (u64d *)out, c->d_mod, c->logN, level);
    return g.rc();
}

extern "C" int ckksmi_mul_scalar(ckksmi_ctx *c, const uint64_t *a, int64_t v, uint64_t *out, int level, int batch, void *stream) {
    int rc = ct_args_ok(c, level, batch);
    if (rc) return rc;
    if (!a || !out) return CKKSMI_EINVAL;
    if (batch == 0) return CKKSMI_OK;
    Guard g(c);
    const size_t total = (size_t)batch * 2 * level * c->N;
    KL(c, CKKSMI_K_ELEMWISE, (double)batch * 2 * level, mul_scalar_kernel, dim3(ew_blocks(total)), dim3(EW_THREADS), S(stream), (const u64d *)a, (u64d *)out, c->d_mod,
                  scalar_tab(c, v, level), c->logN, level, total);
    return g.rc();
}

extern "C" int ckksmi_add_const(ckksmi_ctx *c, const uint64_t *a, int64_t v, uint64_t *out, int level, int batch, void *stream) {
    int rc = ct_args_ok(c, level, batch);
    if (rc) return rc;
    if (!a || !out) return CKKSMI_EINVAL;
    if (batch == 0) return CKKSMI_OK;
    Guard g(c);
    const size_t total = (size_t)batch * 2 * level * c->N;
    KL(c, CKKSMI_K_ELEMWISE, (double)batch * 2 * level, add_const_kernel, dim3(ew_blocks(total)), dim3(EW_THREADS), S(stream), (const u64d *)a, (u64d *)out, c->d_mod,
                  scalar_tab(c, v, level), c->logN, level, total);
    return g.rc();
}

extern "C" int ckksmi_mod_drop(ckksmi_ctx *c, const uint64_t *a, int level_in, int level_out, uint64_t *out, int batch, void *stream) {
    int rc = ct_args_ok(c, level_in, batch);
    if (rc) return rc;
    if (level_out < 1 || level_out > level_in) return CKKSMI_ELEVEL;
    if (!a || !out || a == out) return CKKSMI_EINVAL;
    if (batch == 0) return CKKSMI_OK;
    Guard g(c);
    const size_t total = (size_t)batch * 2 * level_out * c->N;
    KL(c, CKKSMI_K_ELEMWISE, (double)batch * 2 * level_out, mod_drop_kernel, dim3(ew_blocks(total)), dim3(EW_THREADS), S(stream), (const u64d *)a, (u64d *)out, c->logN, level_in,
                  level_out, total);
    return g.rc();
}

extern "C" int ckksmi_hmul(ckksmi_ctx *c, const uint64_t *a, const uint64_t *b, uint64_t *d, int level, int batch, void *stream) {
    int rc = ct_args_ok(c, level, batch);
    if (rc) return rc;
    if (!a || !b || !d || !al16(a) || !al16(b) || !al16(d)) return CKKSMI_EINVAL;
    if (batch == 0) return CKKSMI_OK;
    Guard g(c);
    launch_tensor(c, a, b, d, level, batch, S(stream));
    return g.rc();
}

extern "C" int ckksmi_workspace_bytes(const ckksmi_ctx *c, int op, int level, int batch, size_t *bytes) {
    if (!c || !bytes || batch < 0) return CKKSMI_EINVAL;
    if (level < 1 || level > c->n_q) return CKKSMI_ELEVEL;
    const size_t N = c->N;
    size_t per = 0;
    switch (op) {
        case CKKSMI_OP_RELIN: per = ks_words_per_item(c, level); break;
        case CKKSMI_OP_RESCALE:
            if (level < 2) return CKKSMI_ELEVEL;
            per = rescale_words_per_item(c, level);
            break;
        case CKKSMI_OP_MUL_SCALAR_RESCALE:
            if (level < 2) return CKKSMI_ELEVEL;
            per = rescale_words_per_item(c, level) + 4 * (size_t)level * N;
            break;
        case CKKSMI_OP_HMUL_RELIN_RESCALE:
            if (level < 2) return CKKSMI_ELEVEL;
            per = 5 * (size_t)level * N + std::max(ks_words_per_item(c, level), rescale_words_per_item(c, level));
            break;
        case CKKSMI_OP_ROTATE: per = 2 * (size_t)level * N + ks_words_per_item(c, level); break;
        case CKKSMI_OP_CONV2D_MAC:
            *bytes = (size_t)batch * level * sizeof(WMul);
            return CKKSMI_OK;
        default: return CKKSMI_EINVAL;
    }
    if ((op == CKKSMI_OP_RELIN || op == CKKSMI_OP_HMUL_RELIN_RESCALE || op == CKKSMI_OP_ROTATE) && c->k == 0) return CKKSMI_EUNSUPPORTED;
    *bytes = per * 8 * (size_t)batch;
    return CKKSMI_OK;
}

extern "C" int ckksmi_relin(ckksmi_ctx *c, const uint64_t *d, const uint64_t *evk, uint64_t *out, int level, int batch, void *ws,
                            size_t ws_bytes, void *stream) {
    int rc = ct_args_ok(c, level, batch);
    if (rc) return rc;
    if (c->k == 0) return CKKSMI_EUNSUPPORTED;
    if (!d || !evk || !out || (!ws && batch) || !al16(d) || !al16(evk) || !al16(out) || !al16(ws)) return CKKSMI_EINVAL;
    if (batch == 0) return CKKSMI_OK;
    const size_t N = c->N, per = ks_words_per_item(c, level);
    const int chunk = sweep_items(ws_bytes, per, batch);
    if (chunk < 1) return CKKSMI_EWORKSPACE;
    Guard g(c);
    KeyTab K;
    memset(&K, 0, sizeof(K));
    K.key[0] = (const u64d *)evk;
    for (int b0 = 0; b0 < batch; b0 += chunk) {
        const int items = std::min(chunk, batch - b0);
        const u64 *di = d + (size_t)b0 * 3 * level * N;
        ks_core(c, di + (size_t)2 * level * N, (size_t)3 * level * N, K, items, level, di, (size_t)3 * level * N, (size_t)level * N, 1,
                out + (size_t)b0 * 2 * level * N, (u64 *)ws, S(stream));
    }
    return g.rc();
}

extern "C" int ckksmi_rescale(ckksmi_ctx *c, const uint64_t *a, uint64_t *out, int level, int batch, void *ws, size_t ws_bytes,
                              void *stream) {
    int rc = ct_args_ok(c, level, batch);
    if (rc) return rc;
    if (level < 2) return CKKSMI_ELEVEL;
    if (!a || !out || a == out || (!ws && batch) || !al16(a) || !al16(out) || !al16(ws)) return CKKSMI_EINVAL;
    if (batch == 0) return CKKSMI_OK;
    const size_t N = c->N, per = rescale_words_per_item(c, level);
    const int chunk = sweep_items(ws_bytes, per, batch);
    if (chunk < 1) return CKKSMI_EWORKSPACE;
    Guard g(c);
    for (int b0 = 0; b0 < batch; b0 += chunk) {
        const int items = std::min(chunk, batch - b0);
        rescale_core(c, a + (size_t)b0 * 2 * level * N, out + (size_t)b0 * 2 * (level - 1) * N, items, level, (u64 *)ws, S(stream));
    }
    return g.rc();
}

// The same sweeps as ckksmi_rescale over the GPU's static scratch array instead of a caller's workspace.  Nothing on this
// path allocates: no hipMalloc / hipFree, no events (profiling records none here), no containers.
extern "C" int ckksmi_rescale_static(ckksmi_ctx *c, const uint64_t *a, uint64_t *out, int level, int batch, void *stream) {
    int rc = ct_args_ok(c, level, batch);
    if (rc) return rc;
    if (level < 2) return CKKSMI_ELEVEL;
    if (!a || !out || a == out || !al16(a) || !al16(out)) return CKKSMI_EINVAL;
    if (batch == 0) return CKKSMI_OK;
    const size_t N = c->N, per = rescale_words_per_item(c, level);
    // the static array must hold one item's intermediates; more items than fit are swept in chunks
    if (per * 8 > (size_t)CKKSMI_STATIC_SCRATCH_BYTES) return CKKSMI_EWORKSPACE;
    u64 *ws = c->device < kMaxDevices ? (u64 *)g_scratch_ptr[c->device] : nullptr;
    if (!ws) return CKKSMI_EUNSUPPORTED;
    const int chunk = sweep_items((size_t)CKKSMI_STATIC_SCRATCH_BYTES, per, batch);
    const bool was_profiling = c->prof_on;
    c->prof_on = false;  // timing events are allocations
    Guard g(c);
    for (int b0 = 0; b0 < batch; b0 += chunk) {
        const int items = std::min(chunk, batch - b0);
        rescale_core(c, a + (size_t)b0 * 2 * level * N, out + (size_t)b0 * 2 * (level - 1) * N, items, level, ws, S(stream));
    }
    c->prof_on = was_profiling;
    return g.rc();
}

extern "C" int ckksmi_mul_scalar_rescale(ckksmi_ctx *c, const uint64_t *a, int64_t v, const uint64_t *addend, uint64_t *out, int level_in,
                                         int level, int batch, void *ws, size_t ws_bytes, void *stream) {
    int rc = ct_args_ok(c, level, batch);
    if (rc) return rc;
    if (level < 2 || level_in < level || level_in > c->n_q) return CKKSMI_ELEVEL;
    if (!a || !out || a == out || (!ws && batch) || !al16(a) || !al16(out) || !al16(ws) || !al16(addend)) return CKKSMI_EINVAL;
    if (batch == 0) return CKKSMI_OK;
    const size_t N = c->N, per = rescale_words_per_item(c, level) + 4 * (size_t)level * N;
    const int chunk = sweep_items(ws_bytes, per, batch);
    if (chunk < 1) return CKKSMI_EWORKSPACE;
    Guard g(c);
    hipStream_t st = S(stream);
    for (int b0 = 0; b0 < batch; b0 += chunk) {
        const int items = std::min(chunk, batch - b0);
        const u64 *ain = a + (size_t)b0 * 2 * level_in * N;
        u64 *o = out + (size_t)b0 * 2 * (level - 1) * N;
        const u64 *add = addend ? addend + (size_t)b0 * 2 * (level - 1) * N : nullptr;
        if (c->fused) {
            scalar_rescale_fused(c, ain, v, add, o, items, level_in, level, (u64 *)ws, st);
        } else {
            // the steps as they are (modulus drop, scalar product, rescale): the product goes through the workspace
            u64 *prod = (u64 *)ws;
            const size_t total = (size_t)items * 2 * level * N;
            const u64 *src = ain;
            if (level_in != level) {
                KL(c, CKKSMI_K_ELEMWISE, (double)items * 2 * level, mod_drop_kernel, dim3(ew_blocks(total)), dim3(EW_THREADS), st, (const u64d *)ain,
                   (u64d *)prod, c->logN, level_in, level, total);
                src = prod;
            }
            KL(c, CKKSMI_K_ELEMWISE, (double)items * 2 * level, mul_scalar_kernel, dim3(ew_blocks(total)), dim3(EW_THREADS), st, (const u64d *)src,
               (u64d *)prod, c->d_mod, scalar_tab(c, v, level), c->logN, level, total);
            if (add) {
                // the addend may be the output buffer itself: the quotient goes through the workspace
                u64 *res = prod + total + (size_t)items * rescale_words_per_item(c, level);
                const size_t tout = (size_t)items * 2 * (level - 1) * N;
                rescale_core(c, prod, res, items, level, prod + total, st);
                KL(c, CKKSMI_K_ELEMWISE, (double)items * 2 * (level - 1), addsub_kernel, dim3(ew_blocks(tout)), dim3(EW_THREADS), st, (const u64d *)res,
                   (const u64d *)add, (u64d *)o, c->d_mod, c->logN, level - 1, tout, 0);
            } else {
                rescale_core(c, prod, o, items, level, prod + total, st);
            }
        }
    }
    return g.rc();
}

static int hmul_relin_rescale_impl(ckksmi_ctx *c, const uint64_t *a, const uint64_t *b, const uint64_t *evk, uint64_t *out, int level, int batch,
                                  void *ws, size_t ws_bytes, void *stream, bool merged, int terms = 1) {
    int rc = ct_args_ok(c, level, batch);
    if (rc) return rc;
    if (terms < 1) return CKKSMI_EINVAL;
    if (c->k == 0 || (merged && !c->merged_ok)) return CKKSMI_EUNSUPPORTED;
    if (level < 2) return CKKSMI_ELEVEL;
    if (!a || !b || !evk || !out || (!ws && batch) || !al16(a) || !al16(b) || !al16(evk) || !al16(out) || !al16(ws)) return CKKSMI_EINVAL;
    if (batch == 0) return CKKSMI_OK;
    const size_t N = c->N;
    const size_t per = 5 * (size_t)level * N + std::max(ks_words_per_item(c, level), rescale_words_per_item(c, level));
    const int chunk = sweep_items(ws_bytes, per, batch);
    if (chunk < 1) return CKKSMI_EWORKSPACE;
    Guard g(c);
    KeyTab K;
    memset(&K, 0, sizeof(K));
    K.key[0] = (const u64d *)evk;
    for (int b0 = 0; b0 < batch; b0 += chunk) {
        const int items = std::min(chunk, batch - b0);
        u64 *d = (u64 *)ws;                              // [items][3][level][N]
        u64 *r = d + (size_t)items * 3 * level * N;      // [items][2][level][N]
        u64 *rest = r + (size_t)items * 2 * level * N;
        // register-tiled sizes: the tensor kernel takes d2 through the inverse row pass on the way (its output lands where
        // the key switch expects it: the start of its workspace)
        const size_t in0 = (size_t)b0 * terms * 2 * level * N;
        u64 *o = out + (size_t)b0 * 2 * (level - 1) * N;
        if (!c->fused) {
            launch_tensor(c, a + in0, b + in0, d, level, items, S(stream), terms);
            if (merged) {
                ks_core(c, d + (size_t)2 * level * N, (size_t)3 * level * N, K, items, level, d, (size_t)3 * level * N, (size_t)level * N, 1, o, rest,
                        S(stream), true);
            } else {
                ks_core(c, d + (size_t)2 * level * N, (size_t)3 * level * N, K, items, level, d, (size_t)3 * level * N, (size_t)level * N, 1, r, rest,
                        S(stream));
                rescale_core(c, r, o, items, level, rest, S(stream));
            }
            continue;
        }
        // the tensor is never written: its third component goes through the inverse row pass on the way, the inner product forms
        // what it needs of all three from the operands
        launch_tensor_rows(c, a + in0, b + in0, rest, level, items, S(stream), terms);
        if (merged || one_conversion_tail_ok(c)) {
            // one division by P*q_{level-1} of (accumulators + P*(d0, d1)), or ModDown + add + rescale as one conversion
            ks_core_fused(c, nullptr, 0, K, items, level, nullptr, 0, 0, 1, o, rest, S(stream), !merged, merged, nullptr, a + in0, b + in0, terms);
        } else {
            ks_core_fused(c, nullptr, 0, K, items, level, nullptr, 0, 0, 1, r, rest, S(stream), false, false, nullptr, a + in0, b + in0, terms);
            rescale_core(c, r, o, items, level, rest, S(stream));
        }
    }
    return g.rc();
}

extern "C" int ckksmi_hmul_relin_rescale(ckksmi_ctx *c, const uint64_t *a, const uint64_t *b, const uint64_t *evk, uint64_t *out, int level,
                                         int batch, void *ws, size_t ws_bytes, void *stream) {
    return hmul_relin_rescale_impl(c, a, b, evk, out, level, batch, ws, ws_bytes, stream, false);
}

extern "C" int ckksmi_hmul_sum_relin_rescale(ckksmi_ctx *c, const uint64_t *a, const uint64_t *b, int terms, const uint64_t *evk, uint64_t *out,
                                             int level, int batch, void *ws, size_t ws_bytes, void *stream) {
    return hmul_relin_rescale_impl(c, a, b, evk, out, level, batch, ws, ws_bytes, stream, false, terms);
}

extern "C" int ckksmi_hmul_relin_rescale_merged(ckksmi_ctx *c, const uint64_t *a, const uint64_t *b, const uint64_t *evk, uint64_t *out, int level,
                                                int batch, void *ws, size_t ws_bytes, void *stream) {
    return hmul_relin_rescale_impl(c, a, b, evk, out, level, batch, ws, ws_bytes, stream, true);
}

extern "C" int ckksmi_rotate(ckksmi_ctx *c, const uint64_t *a, const int *rot, uint64_t *out, int level, int batch, void *ws,
                             size_t ws_bytes, void *stream) {
    int rc = ct_args_ok(c, level, batch);
    if (rc) return rc;
    if (c->k == 0) return CKKSMI_EUNSUPPORTED;
    if (!a || !rot || !out || a == out || (!ws && batch) || !al16(a) || !al16(out) || !al16(ws)) return CKKSMI_EINVAL;
    if (batch == 0) return CKKSMI_OK;
    // every rotation needs its key before anything is enqueued
    std::vector<int> key_of(batch);
    for (int i = 0; i < batch; i++) {
        const int r = norm_rot(c, rot[i]);
        int found = -1;
        for (size_t e = 0; e < c->galois.size(); e++)
            if (c->galois[e].first == r) found = (int)e;
        if (found < 0) return CKKSMI_ENOKEY;
        key_of[i] = found;
    }
    const size_t N = c->N;
    const size_t per = 2 * (size_t)level * N + ks_words_per_item(c, level);
    const int chunk = sweep_items(ws_bytes, per, batch);
    if (chunk < 1) return CKKSMI_EWORKSPACE;
    Guard g(c);
    int b0 = 0;
    while (b0 < batch) {
        // longest run from b0 that fits the sweep and addresses at most CKKSMI_MAX_KEYS distinct keys
        KeyTab K;
        GaloisTab G;
        memset(&K, 0, sizeof(K));
        memset(&G, 0, sizeof(G));
        int used[CKKSMI_MAX_KEYS], n_used = 0, items = 0;
        while (b0 + items < batch && items < chunk) {
            const int kidx = key_of[b0 + items];
            int slot = -1;
            for (int u = 0; u < n_used; u++)
                if (used[u] == kidx) slot = u;
            if (slot < 0) {
                if (n_used == CKKSMI_MAX_KEYS) break;
                slot = n_used;
                used[n_used++] = kidx;
                K.key[slot] = (const u64d *)c->galois[kidx].second;
            }
            K.slot[items] = (unsigned char)slot;
            G.g[items] = (unsigned)galois_element_of(c, rot[b0 + items]);
            items++;
        }
        u64 *sig = (u64 *)ws;  // [items][2][level][N]
        u64 *rest = sig + (size_t)items * 2 * level * N;
        const size_t total = (size_t)items * 2 * level * N;
        if (c->fused) {
            // register-tiled sizes: no rotated copy is written; the kernels that read c1 (inverse row pass, the own digit's
            // term of the inner product) and c0 (the addend) read them through the automorphism
            const u64 *ai = a + (size_t)b0 * 2 * level * N;
            ks_core_fused(c, ai + (size_t)level * N, (size_t)2 * level * N, K, items, level, ai, (size_t)2 * level * N, 0, 0,
                          out + (size_t)b0 * 2 * level * N, rest, S(stream), false, false, nullptr, nullptr, nullptr, 1, &G);
            b0 += items;
            continue;
        }
        KL(c, CKKSMI_K_AUTOMORPH, (double)items * 2 * level, automorphism_kernel, dim3(ew_blocks(total)), dim3(EW_THREADS), S(stream), (const u64d *)(a + (size_t)b0 * 2 * level * N),
                      (u64d *)sig, G, c->logN, 2 * level, total);
        ks_core(c, sig + (size_t)level * N, (size_t)2 * level * N, K, items, level, sig, (size_t)2 * level * N, 0, 0,
                out + (size_t)b0 * 2 * level * N, rest, S(stream));
        b0 += items;
    }
    return g.rc();
}

// ------------------------------------------------------------------ device-side encoding and encryption
extern "C" int ckksmi_encode_device(ckksmi_ctx *c, const double *re, const double *im, double scale, int level, int batch, uint64_t *pt, void *ws,
                                    size_t ws_bytes, void *stream) {
    int rc = ct_args_ok(c, level, batch);
    if (rc) return rc;
    if (!re || !pt || !(scale > 0) || (!ws && batch) || !al16(pt) || !al16(ws) || ((uintptr_t)re & 7u) || ((uintptr_t)im & 7u)) return CKKSMI_EINVAL;
    if (c->logN < 1) return CKKSMI_EUNSUPPORTED;
    if (batch == 0) return CKKSMI_OK;
    const size_t N = c->N;
    if (ws_bytes < (size_t)batch * N * 16) return CKKSMI_EWORKSPACE;
    Guard g(c);
    hipStream_t st = S(stream);
    EncodeArgs A;
    A.re = re; A.im = im; A.cbuf = (double2 *)ws; A.slot_exp = c->d_slot_exp; A.ctw = (const double2 *)c->d_ctw; A.logN = c->logN;
    // every call takes its own overflow word (round-robin over CKKSMI_FLAG_SLOTS), so calls in flight on different streams
    // of one context do not share one
    int *flag_word = c->d_flag + (c->flag_next.fetch_add(1) % CKKSMI_FLAG_SLOTS);
    A.flag = flag_word;
    A.LA = la_for(c->logN);
    const unsigned N1 = 1u << A.LA, N2 = (unsigned)(N >> A.LA);
    const unsigned R = N2 >= CFFT_TILE ? 1u : CFFT_TILE / N2;
    KL(c, CKKSMI_K_ENCODE, (double)batch, encode_scatter_kernel, dim3(ew_blocks(N / 2), batch), dim3(EW_THREADS), st, A);
    KL(c, CKKSMI_K_ENCODE, (double)batch, cfft_inv_kernel<false>, dim3(batch, (N1 + R - 1) / R), dim3(NTT_THREADS), st, A);
    if (A.LA) KL(c, CKKSMI_K_ENCODE, (double)batch, cfft_inv_kernel<true>, dim3(batch, N2 / NTT_TC), dim3(NTT_THREADS), st, A);
    const size_t total = (size_t)batch * N;
    KL(c, CKKSMI_K_ENCODE, (double)batch, encode_round_kernel, dim3(ew_blocks(total)), dim3(EW_THREADS), st, (const double2 *)ws, scale / (double)N,
       (u64d *)pt, c->d_mod, c->logN, level, total, flag_word);
    int idx[CKKSMI_MAX_MODULI];
    for (int i = 0; i < level; i++) idx[i] = i;
    launch_ntt(c, true, pt, pt, table_map(idx, level, (size_t)level * N, (size_t)level * N), batch, st);
    int flag = 0;
    if (hipMemcpyAsync(&flag, flag_word, sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess || hipStreamSynchronize(st) != hipSuccess)
        return CKKSMI_EDEVICE;
    if (flag) return CKKSMI_EINVAL;
    return g.rc();
}

extern "C" int ckksmi_encrypt_device(ckksmi_ctx *c, const uint64_t *pk, const uint64_t *pt, const int64_t *r, const int64_t *e0, const int64_t *e1,
                                     int level, int batch, uint64_t *ct, void *ws, size_t ws_bytes, void *stream) {
    int rc = ct_args_ok(c, level, batch);
    if (rc) return rc;
    if (!pk || !pt || !r || !e0 || !e1 || !ct || (!ws && batch) || !al16(pk) || !al16(pt) || !al16(ct) || !al16(ws) || ((uintptr_t)r & 7u) ||
        ((uintptr_t)e0 & 7u) || ((uintptr_t)e1 & 7u))
        return CKKSMI_EINVAL;
    if (batch == 0) return CKKSMI_OK;
    const size_t N = c->N;
    const size_t per = 3 * (size_t)level * N * 8;
    const int chunk = (int)std::min<size_t>((size_t)batch, ws_bytes / per);
    if (chunk < 1) return CKKSMI_EWORKSPACE;
    Guard g(c);
    hipStream_t st = S(stream);
    int idx[CKKSMI_MAX_MODULI];
    for (int i = 0; i < level; i++) idx[i] = i;
    for (int b0 = 0; b0 < batch; b0 += chunk) {
        const int items = std::min(chunk, batch - b0);
        u64 *small = (u64 *)ws;  // [items][3][level][N]: r, e0, e1
        const int64_t *src[3] = {r, e0, e1};
        if (c->fused) {
            // register-tiled sizes: the column pass reads the small coefficients themselves, the row pass forms the ciphertext
            NttV2Args V;
            memset(&V, 0, sizeof(V));
            V.modc = c->d_mod; V.tw = c->d_tww_fwd; V.logN = c->logN; V.p51 = c->p51mask; V.items = items;
            V.map = table_map(idx, level, N, (size_t)3 * level * N);  // source: one int64 polynomial per item
            const unsigned tiles = (unsigned)(N / 4096);
            const unsigned zc = zchunks_for(c, tiles * level, items, V.items_per_z);
            for (int which = 0; which < 3; which++) {
                V.src = (const u64d *)(src[which] + (size_t)b0 * N);
                V.dst = (u64d *)(small + (size_t)which * level * N);
                KL(c, CKKSMI_K_ENCRYPT, (double)items * level, ntt_v2_fwd_cols_small_kernel, dim3(tiles, level, zc), dim3(V2_THREADS), st, V);
            }
            EncryptRowsArgs E;
            E.mid = (const u64d *)small; E.pk = (const u64d *)pk; E.pt = (const u64d *)(pt + (size_t)b0 * level * N);
            E.ct = (u64d *)(ct + (size_t)b0 * 2 * level * N); E.modc = c->d_mod; E.tw = c->d_tww_fwd; E.logN = c->logN; E.level = level;
            E.n_q = c->n_q; E.items = items; E.p51 = c->p51mask;
            const unsigned xc = zchunks_for(c, tiles * level, items, E.items_per_x);
            KL(c, CKKSMI_K_ENCRYPT, (double)items * level, encrypt_rows_kernel, dim3(xc, tiles, level), dim3(V2_THREADS), st, E);
            continue;
        }
        const size_t rows_total = (size_t)items * N;
        for (int which = 0; which < 3; which++)
            KL(c, CKKSMI_K_ENCRYPT, (double)items * level, small_to_rns_kernel, dim3(ew_blocks(rows_total)), dim3(EW_THREADS), st,
               (const long long *)(src[which] + (size_t)b0 * N), (u64d *)(small + (size_t)which * level * N),
               (unsigned long long)((size_t)3 * level * N), c->d_mod, c->logN, level, rows_total);
        launch_ntt(c, true, small, small, table_map(idx, level, (size_t)level * N, (size_t)level * N), (size_t)items * 3, st);
        const size_t total = (size_t)items * level * N;
        KL(c, CKKSMI_K_ENCRYPT, (double)items * level, encrypt_combine_kernel, dim3(ew_blocks(total)), dim3(EW_THREADS), st, (const u64d *)small,
           (const u64d *)pk, (const u64d *)(pt + (size_t)b0 * level * N), (u64d *)(ct + (size_t)b0 * 2 * level * N), c->d_mod, c->logN, level,
           c->n_q, total);
    }
    return g.rc();
}

extern "C" int ckksmi_sample_device(ckksmi_ctx *c, int kind, double sigma, uint64_t seed, uint64_t first_index, int rows, int64_t *out, void *stream) {
    if (!dev_ok(c)) return CKKSMI_EDEVICE;
    if ((kind != CKKSMI_SAMPLE_TERNARY && kind != CKKSMI_SAMPLE_GAUSSIAN) || rows < 0 || (!out && rows) || ((uintptr_t)out & 7u) ||
        (kind == CKKSMI_SAMPLE_GAUSSIAN && !(sigma > 0.0 && sigma < 64.0)))
        return CKKSMI_EINVAL;
    if (rows == 0) return CKKSMI_OK;
    Guard g(c);
    SampleArgs A;
    memset(&A, 0, sizeof(A));
    A.out = (long long *)out; A.seed = seed; A.first_index = first_index; A.kind = kind; A.logN = c->logN; A.total = (size_t)rows * c->N;
    if (kind == CKKSMI_SAMPLE_GAUSSIAN)
        for (int k = 0; k < SAMPLE_K; k++) {
            // P(|X| <= k) = erf((k + 1/2) / (sigma sqrt 2)) through the complementary function: the tail keeps its relative accuracy
            const long double tail = erfcl(((long double)k + 0.5L) / ((long double)sigma * sqrtl(2.0L))) * 18446744073709551616.0L;
            A.T[k] = tail >= 1.0L ? (unsigned long long)0 - (unsigned long long)ceill(tail) : ~0ull;
        }
    KL(c, CKKSMI_K_ENCRYPT, (double)rows, sample_kernel, dim3(ew_blocks(A.total)), dim3(EW_THREADS), S(stream), A);
    return g.rc();
}

static size_t hoisted_words_per_item(const ckksmi_ctx *c, int level, int R) {
    const size_t N = c->N, E = level + c->k, beta = (level + c->alpha - 1) / c->alpha;
    // sigma_r(c0) + lifted digits + R accumulator pairs + R conversion results
    return N * ((size_t)R * level + (size_t)level + beta * E + (size_t)R * (2 * E + 2 * (size_t)level));
}

extern "C" int ckksmi_rotate_hoisted_workspace_bytes(const ckksmi_ctx *c, int level, int batch, int n_rot, size_t *bytes) {
    if (!c || !bytes || level < 1 || level > c->n_q || batch < 0 || n_rot < 1 || n_rot > CKKSMI_MAX_KEYS) return CKKSMI_EINVAL;
    const size_t items = (size_t)(batch < CKKSMI_MAX_ITEMS ? batch : CKKSMI_MAX_ITEMS);
    *bytes = items * hoisted_words_per_item(c, level, n_rot) * 8;
    return CKKSMI_OK;
}

extern "C" int ckksmi_rotate_hoisted(ckksmi_ctx *c, const uint64_t *a, const int *rot, int n_rot, uint64_t *out, int level, int batch, void *ws,
                                     size_t ws_bytes, void *stream) {
    int rc = ct_args_ok(c, level, batch);
    if (rc) return rc;
    if (c->k == 0) return CKKSMI_EUNSUPPORTED;
    if (!a || !rot || !out || a == out || n_rot < 1 || n_rot > CKKSMI_MAX_KEYS || (!ws && batch) || !al16(a) || !al16(out) || !al16(ws))
        return CKKSMI_EINVAL;
    HoistPlan H;
    memset(&H, 0, sizeof(H));
    H.R = n_rot;
    for (int r = 0; r < n_rot; r++) {
        const int nr = norm_rot(c, rot[r]);
        int found = -1;
        for (size_t e = 0; e < c->galois.size(); e++)
            if (c->galois[e].first == nr) found = (int)e;
        if (found < 0) return CKKSMI_ENOKEY;
        H.key[r] = c->galois[found].second;
        H.g[r] = (unsigned)galois_element_of(c, rot[r]);
        H.ginv[r] = (unsigned)hm::powmod(H.g[r], c->N - 1, 2 * c->N);  // the units mod 2N have order N
    }
    if (batch == 0) return CKKSMI_OK;
    const size_t N = c->N;
    const int chunk = sweep_items(ws_bytes, hoisted_words_per_item(c, level, n_rot), batch);
    if (chunk < 1) return CKKSMI_EWORKSPACE;
    Guard g(c);
    KeyTab K;
    memset(&K, 0, sizeof(K));
    for (int b0 = 0; b0 < batch; b0 += chunk) {
        const int items = std::min(chunk, batch - b0);
        const u64 *ain = a + (size_t)b0 * 2 * level * N;
        u64 *sig = (u64 *)ws;  // [items][R][level][N]
        u64 *rest = sig + (size_t)items * n_rot * level * N;
        HoistArgs HA;
        memset(&HA, 0, sizeof(HA));
        HA.logN = c->logN; HA.level = level; HA.R = n_rot;
        for (int r = 0; r < n_rot; r++) HA.g[r] = H.g[r];
        const size_t total = (size_t)items * n_rot * level * N;
        // register-tiled sizes: the last pass reads sigma_r(c0) from the input through the automorphism; otherwise it is written here
        if (!c->fused)
            KL(c, CKKSMI_K_AUTOMORPH_BCAST, (double)items * n_rot * level, automorphism_bcast_kernel, dim3(ew_blocks(total)), dim3(EW_THREADS), S(stream),
               (const u64d *)ain, (unsigned long long)((size_t)2 * level * N), (u64d *)sig, HA, total);
        H.sig = sig; H.c0 = ain; H.c0_stride = (size_t)2 * level * N;
        ks_core(c, ain + (size_t)level * N, (size_t)2 * level * N, K, items, level, nullptr, 0, 0, 0, out + (size_t)b0 * n_rot * 2 * level * N, rest,
                S(stream), false, &H);
    }
    return g.rc();
}

namespace {
// Which multiply-accumulate kernel a layer shape can use, and the workspace the matrix-core ones need.
struct MacShape {
    bool mfma_ok;
    bool resident;  // few taps: the kernel that keeps the weight digits in LDS
    bool strip;     // ... and a narrow window: four positions (TY x TX) share a strip of the image staged in LDS
    int TY, TX, SR, SC;  // strip rows per channel, pixels per strip row
    int quad;       // its last step covers at most 16 taps, as a quad step
    int Kb, Mg;     // steps (64 taps, or the quad step), 32-channel groups
    size_t afrag_bytes, taps_bytes, off_bytes, tapoff_bytes, wsum_bytes, mfma_bytes;
};
MacShape mac_shape(const ckksmi_ctx *c, int C, int O, int kh, int kw, int stride, int out_rows, int Wo, int level) {
    MacShape s;
    const long long K = (long long)C * kh * kw;
    s.Kb = (int)((K + 63) / 64);
    s.resident = s.Kb <= MM_RES_STEPS;
    s.quad = (s.resident && K % 64 != 0 && K % 64 <= 16) ? 1 : 0;
    // the four waves' positions: 2 x 2 or 1 x 4, whichever leaves fewer waves without a position (then the smaller strip)
    s.strip = false;
    s.TY = 1; s.TX = MM_STRIP_POS; s.SR = kh; s.SC = kw + (MM_STRIP_POS - 1) * stride;
    if (s.Kb <= MM_STRIP_STEPS && c->N >= 16 && kh + stride < 256 && kw + 3LL * stride < 65536) {
        long long best = -1;
        for (int ty = 1; ty <= 2; ty++) {
            const int tx = MM_STRIP_POS / ty;
            const long long sr = kh + (ty - 1) * stride, sc = kw + (tx - 1) * stride, ln = (long long)C * sr * sc;
            if (ln > MM_STRIP_LINES) continue;
            const long long slots = (long long)((out_rows + ty - 1) / ty) * ((Wo + tx - 1) / tx);
            const long long cost = slots * 1024 + ln;
            if (best < 0 || cost < best) { best = cost; s.strip = true; s.TY = ty; s.TX = tx; s.SR = (int)sr; s.SC = (int)sc; }
        }
    }
    s.Mg = (O + MM_CH - 1) / MM_CH;
    s.afrag_bytes = (size_t)level * s.Kb * s.Mg * MM_FRAG * 16;
    s.taps_bytes = 2 * (size_t)s.Kb * 64 * sizeof(TapEnt);
    s.off_bytes = (size_t)s.Kb * 64 * sizeof(unsigned long long);
    s.tapoff_bytes = (size_t)s.Kb * 64 * sizeof(unsigned);
    s.wsum_bytes = (size_t)level * s.Mg * MM_CH * sizeof(double);
    s.mfma_bytes = s.afrag_bytes + s.taps_bytes + s.off_bytes + s.tapoff_bytes + s.wsum_bytes;
    // below 8 output channels most of a 32-channel group would multiply zeros: the vector kernel is faster there
    s.mfma_ok = c->N >= MM_WORDS && O >= 8 && K <= MM_KMAX - 63;
    return s;
}
}  // namespace

extern "C" int ckksmi_conv2d_mac_rows(ckksmi_ctx *c, const uint64_t *in, const int64_t *w, int C, int H, int W, int O, int kh, int kw,
                                      int stride, int pad, int in_row0, int in_rows, int out_row0, int out_rows, uint64_t *out, int level,
                                      void *ws, size_t ws_bytes, void *stream) {
    if (!c) return CKKSMI_EINVAL;
    if (!dev_ok(c)) return CKKSMI_EDEVICE;
    if (level < 1 || level > c->n_q) return CKKSMI_ELEVEL;
    if (!in || !w || !out || !ws || in == out) return CKKSMI_EINVAL;
    if (!al16(in) || !al16(out) || !al16(ws)) return CKKSMI_EINVAL;
    if (C < 1 || H < 1 || W < 1 || O < 1 || kh < 1 || kw < 1 || stride < 1 || pad < 0) return CKKSMI_EINVAL;
    if (H + 2 * pad < kh || W + 2 * pad < kw) return CKKSMI_EINVAL;
    const int Ho = (H + 2 * pad - kh) / stride + 1, Wo = (W + 2 * pad - kw) / stride + 1;
    if (out_row0 < 0 || out_rows < 1 || out_row0 > Ho - out_rows) return CKKSMI_EINVAL;
    if (in_row0 < 0 || in_rows < 1 || in_row0 > H - in_rows) return CKKSMI_EINVAL;
    // every image row that a tap of the requested output rows can touch must lie inside the strip
    const long long first = std::max(0LL, (long long)out_row0 * stride - pad);
    const long long last = std::min((long long)H - 1, (long long)(out_row0 + out_rows - 1) * stride - pad + kh - 1);
    if (first <= last && (first < in_row0 || last >= (long long)in_row0 + in_rows)) return CKKSMI_EINVAL;
    const size_t n_weights = (size_t)O * C * kh * kw;
    Guard g(c);
    MacShape ms = mac_shape(c, C, O, kh, kw, stride, out_rows, Wo, level);
    if (ms.mfma_ok && ws_bytes >= ms.mfma_bytes && (size_t)C * in_rows * W < MM_TAP_DELTA_MAX && kh <= MM_TAP_KMAX && kw <= MM_TAP_KMAX) {
        const unsigned positions = (unsigned)(out_rows * Wo);
        // resident kernel: each workgroup takes `run` positions of a 64-word block, nrun workgroups share the block;
        // strip kernel: `run` tiles (four positions of a row) of a 16-word block
        const int spr = (Wo + ms.TX - 1) / ms.TX;
        const unsigned units_per_block = ms.strip ? (unsigned)(((out_rows + ms.TY - 1) / ms.TY) * spr) : positions;
        // long runs amortise the weight digits and keep the staging pipeline full (64 tiles, or 8 positions where every
        // wave loads its own words); short ones where the layer would otherwise give the chip too few workgroups
        const size_t blocks = (size_t)(c->N / (ms.strip ? 16 : MM_WORDS)) * 2 * level;
        const size_t target = (size_t)std::max(1, c->ntt_target_wgs / 2);
        const unsigned want_nrun = (unsigned)std::min<size_t>(units_per_block, (target + blocks - 1) / blocks);
        const unsigned run = std::max(1u, std::min(ms.strip ? 64u : 8u, units_per_block / std::max(1u, want_nrun)));
        const unsigned nrun = (units_per_block + run - 1) / run;
        const size_t real = ms.strip      ? (size_t)nrun * (c->N / 16) * 2 * level
                            : ms.resident ? (size_t)nrun * (c->N / MM_WORDS) * 2 * level
                                          : (size_t)positions * ms.Mg * (c->N / MM_WORDS) * 2 * level;
        const size_t xdim = (real + 7) / 8 * 8;
        if (xdim > 0x7fffffffu) return CKKSMI_EUNSUPPORTED;
        char *wp = (char *)ws;  // every part is a multiple of 16 bytes
        v4i *afrag = (v4i *)wp; wp += ms.afrag_bytes;
        TapEnt *taps = (TapEnt *)wp; wp += ms.taps_bytes;
        unsigned long long *off64 = (unsigned long long *)wp; wp += ms.off_bytes;
        unsigned *tapoff = (unsigned *)wp; wp += ms.tapoff_bytes;
        double *wsum = (double *)wp;
        const size_t prep = std::max(std::max(ms.afrag_bytes / 16, (size_t)ms.Kb * 64), (size_t)level * ms.Mg * MM_CH);
        KL(c, CKKSMI_K_MACPREP_MFMA, 1, mac_prepare_mfma_kernel, dim3(ew_blocks(prep)), dim3(EW_THREADS), S(stream), (const long long *)w, afrag, taps,
                      off64, tapoff, ms.SR, ms.SC, wsum, c->d_mod, level, c->logN, O, C, kh, kw, in_rows, W, ms.Kb, ms.Mg, ms.quad);
        MacMfmaArgs A;
        A.in = (const u64d *)in; A.out = (u64d *)out; A.afrag = afrag; A.taps = taps; A.off64 = off64; A.tapoff = tapoff; A.wsum = wsum; A.modc = c->d_mod;
        A.pow24 = c->d_pow24;
        A.logN = c->logN; A.level = level; A.C = C; A.H = H; A.W = W; A.O = O; A.kh = kh; A.kw = kw; A.stride = stride; A.pad = pad; A.Wo = Wo;
        A.in_row0 = in_row0; A.in_rows = in_rows; A.out_row0 = out_row0; A.out_rows = out_rows; A.Kb = ms.Kb; A.Mg = ms.Mg; A.quad = ms.quad;
        A.positions = positions; A.nrun = nrun; A.run = run; A.TY = ms.TY; A.TX = ms.TX; A.SR = ms.SR; A.SC = ms.SC; A.spr = spr; A.total_wgs = xdim; A.real_wgs = real;
        const double units = (double)O * out_rows * Wo * 2 * level;
        if (ms.strip) {
            const dim3 grid((unsigned)xdim), block(256);
#define MAC_STRIP(KB, Q)                                                                                                            \
    do {                                                                                                                            \
        if (ms.TY == 1) KL(c, CKKSMI_K_MAC_MFMA_STRIP, units, (conv_mac_mfma_strip_kernel<KB, Q, 1>), grid, block, S(stream), A);   \
        else KL(c, CKKSMI_K_MAC_MFMA_STRIP, units, (conv_mac_mfma_strip_kernel<KB, Q, 2>), grid, block, S(stream), A);              \
    } while (0)
            switch (ms.Kb * 2 + ms.quad) {
                case 2: MAC_STRIP(1, false); break;
                case 3: MAC_STRIP(1, true); break;
                case 4: MAC_STRIP(2, false); break;
                default: MAC_STRIP(2, true); break;
            }
#undef MAC_STRIP
        } else if (ms.resident) {
            const dim3 grid((unsigned)xdim), block(256);
#define MAC_RES(KB, Q) KL(c, CKKSMI_K_MAC_MFMA_RES, units, (conv_mac_mfma_resident_kernel<KB, Q>), grid, block, S(stream), A)
            switch (ms.Kb * 2 + ms.quad) {
                case 2: MAC_RES(1, false); break;
                case 3: MAC_RES(1, true); break;
                case 4: MAC_RES(2, false); break;
                case 5: MAC_RES(2, true); break;
                case 6: MAC_RES(3, false); break;
                case 7: MAC_RES(3, true); break;
                case 8: MAC_RES(4, false); break;
                default: MAC_RES(4, true); break;
            }
#undef MAC_RES
        } else
            KL(c, CKKSMI_K_MAC_MFMA, units, conv_mac_mfma_kernel, dim3((unsigned)xdim), dim3(256), S(stream), A);
        return g.rc();
    }
    if (ws_bytes < n_weights * level * sizeof(WMul)) return CKKSMI_EWORKSPACE;
    const size_t zdim = (size_t)out_rows * Wo * ((O + MAC_OC - 1) / MAC_OC);
    if (zdim > 0x7fffffffu || ew_blocks(c->N) > 65535) return CKKSMI_EUNSUPPORTED;
    KL(c, CKKSMI_K_MACPREP, 1, mac_prepare_kernel, dim3(ew_blocks(n_weights * level)), dim3(EW_THREADS), S(stream), (const long long *)w, (WMul *)ws,
                  c->d_mod, level, n_weights);
    MacArgs A;
    A.in = (const u64d *)in; A.out = (u64d *)out; A.wtab = (const WMul *)ws; A.modc = c->d_mod;
    A.logN = c->logN; A.level = level;
    A.C = C; A.H = H; A.W = W; A.O = O; A.kh = kh; A.kw = kw; A.stride = stride; A.pad = pad; A.Ho = Ho; A.Wo = Wo;
    A.in_row0 = in_row0; A.in_rows = in_rows; A.out_row0 = out_row0; A.out_rows = out_rows;
    KL(c, CKKSMI_K_MAC, (double)O * out_rows * Wo * 2 * level, conv_mac_kernel, dim3((unsigned)zdim, ew_blocks(c->N), 2 * level), dim3(EW_THREADS), S(stream), A);
    return g.rc();
}

extern "C" int ckksmi_conv2d_workspace_bytes(const ckksmi_ctx *c, int C, int O, int kh, int kw, int level, size_t *bytes) {
    if (!c || !bytes || C < 1 || O < 1 || kh < 1 || kw < 1) return CKKSMI_EINVAL;
    if (level < 1 || level > c->n_q) return CKKSMI_ELEVEL;
    const MacShape ms = mac_shape(c, C, O, kh, kw, 1, 1, 1, level);
    const size_t valu = (size_t)O * C * kh * kw * level * sizeof(WMul);
    *bytes = ms.mfma_ok ? std::max(valu, ms.mfma_bytes) : valu;
    return CKKSMI_OK;
}

extern "C" int ckksmi_conv2d_mac(ckksmi_ctx *c, const uint64_t *in, const int64_t *w, int C, int H, int W, int O, int kh, int kw, int stride,
                                 int pad, uint64_t *out, int level, void *ws, size_t ws_bytes, void *stream) {
    if (H < 1 || kh < 1 || stride < 1 || pad < 0 || H + 2 * pad < kh) return CKKSMI_EINVAL;
    const int Ho = (H + 2 * pad - kh) / stride + 1;
    return ckksmi_conv2d_mac_rows(c, in, w, C, H, W, O, kh, kw, stride, pad, 0, H, 0, Ho, out, level, ws, ws_bytes, stream);
}

extern "C" int ckksmi_sum_pool2d(ckksmi_ctx *c, const uint64_t *in, int C, int H, int W, int k, int pad, uint64_t *out, int level,
                                 void *stream) {
    if (!c) return CKKSMI_EINVAL;
    if (!dev_ok(c)) return CKKSMI_EDEVICE;
    if (level < 1 || level > c->n_q) return CKKSMI_ELEVEL;
    if (!in || !out || in == out) return CKKSMI_EINVAL;
    if (C < 1 || H < 1 || W < 1 || k < 1 || k > 16 || pad < 0 || pad >= k || H + 2 * pad < k || W + 2 * pad < k) return CKKSMI_EINVAL;
    const int Ho = (H + 2 * pad) / k, Wo = (W + 2 * pad) / k;
    const size_t total = (size_t)C * Ho * Wo * 2 * level * c->N;
    if (ew_blocks(total) > 0x7fffffffu) return CKKSMI_EUNSUPPORTED;
    Guard g(c);
    KL(c, CKKSMI_K_ELEMWISE, (double)C * Ho * Wo * 2 * level, sum_pool_kernel, dim3(ew_blocks(total)), dim3(EW_THREADS), S(stream), (const u64d *)in,
                  (u64d *)out, c->d_mod, c->logN, level, H, W, k, pad, Ho, Wo, total);
    return g.rc();
}

extern "C" int ckksmi_fc_mac(ckksmi_ctx *c, const uint64_t *in, const int64_t *w, int F, int O, uint64_t *out, int level, void *ws,
                             size_t ws_bytes, void *stream) {
    return ckksmi_conv2d_mac(c, in, w, F, 1, 1, O, 1, 1, 1, 0, out, level, ws, ws_bytes, stream);
}

// ------------------------------------------------------------------ per-kernel timing
extern "C" int ckksmi_profile_enable(ckksmi_ctx *c, int on) {
    if (!c) return CKKSMI_EINVAL;
    if (!dev_ok(c)) return CKKSMI_EDEVICE;
    for (ProfRec &r : c->prof) { (void)hipEventDestroy((hipEvent_t)r.start); (void)hipEventDestroy((hipEvent_t)r.stop); }
    c->prof.clear();
    c->prof_on = on != 0;
    return CKKSMI_OK;
}

extern "C" int ckksmi_profile_read(ckksmi_ctx *c, int kernel_class, double *total_ms, long long *launches, double *units) {
    if (!c || kernel_class < 0 || kernel_class >= CKKSMI_K_COUNT) return CKKSMI_EINVAL;
    if (!dev_ok(c)) return CKKSMI_EDEVICE;
    double ms = 0, u = 0;
    long long n = 0;
    for (ProfRec &r : c->prof) {
        if (r.kid != kernel_class) continue;
        if (hipEventSynchronize((hipEvent_t)r.stop) != hipSuccess) return CKKSMI_EDEVICE;
        float dt = 0;
        if (hipEventElapsedTime(&dt, (hipEvent_t)r.start, (hipEvent_t)r.stop) != hipSuccess) return CKKSMI_EDEVICE;
        ms += dt;
        u += r.units;
        n++;
    }
    if (total_ms) *total_ms = ms;
    if (launches) *launches = n;
    if (units) *units = u;
    return CKKSMI_OK;
}

extern "C" int ckksmi_tune(ckksmi_ctx *c, int knob, int value) {
    if (!c || knob != CKKSMI_TUNE_TARGET_WGS || value < 1) return CKKSMI_EINVAL;
    c->ntt_target_wgs = value;
    return CKKSMI_OK;
}

extern "C" const char *ckksmi_kernel_class_name(const ckksmi_ctx *c, int kernel_class) {
    static const char *names[CKKSMI_K_COUNT] = {"ntt_fwd_kernel<true>", "ntt_fwd_kernel<false>", "ntt_inv_kernel<false>", "ntt_inv_kernel<true>",
                                                "tensor_kernel", "modup_kernel", "inner_product_kernel", "divround_conv_kernel",
                                                "divround_final_kernel", "automorphism_kernel", "mac_prepare_kernel", "conv_mac_kernel",
                                                "elementwise kernels", "modup_cols_kernel", "modup_cols_kernel", "rows_inner_kernel",
                                                "rows_final_kernel", "modup_cols_kernel", "conv_mac_mfma_kernel", "mac_prepare_mfma_kernel", "ntt_wg_kernel", "tensor_rows_kernel",
                                                "axpy_limb_kernel", "modup_cols_kernel", "inner_product_hoisted_tile_kernel", "automorphism_bcast_kernel",
                                                "encoding kernels", "encryption kernels", "modup_cols_kernel", "conv_mac_mfma_resident_kernel", "conv_mac_mfma_strip_kernel"};
    if (kernel_class < 0 || kernel_class >= CKKSMI_K_COUNT) return "";
    if (c && kernel_class == CKKSMI_K_INNER_HOISTED && !hoisted_tile_ok(c, c->beta_top)) return "inner_product_hoisted_kernel";
    if (c && c->logN >= 12 && c->logN <= 16) {
        static const char *v2[4] = {"ntt_v2_kernel<false, true>", "ntt_v2_kernel<false, false>", "ntt_v2_kernel<true, false>",
                                    "ntt_v2_kernel<true, true>"};
        if (kernel_class < 4) return v2[kernel_class];
        // the conversion kernels are instantiated per (size, source limbs, mode): report the symbol that runs
        static thread_local char buf[64];
        const int q = c->logN - 12;
        if (kernel_class == CKKSMI_K_CONV_COLS_MODUP) { snprintf(buf, sizeof(buf), "modup_cols_kernel<%d, %d, 0>", q, c->alpha); return buf; }
        if (kernel_class == CKKSMI_K_CONV_COLS_DIV) { snprintf(buf, sizeof(buf), "modup_cols_kernel<%d, %d, 1>", q, c->k); return buf; }
        if (kernel_class == CKKSMI_K_CONV_COLS_RESCALE) { snprintf(buf, sizeof(buf), "modup_cols_kernel<%d, 1, 1>", q); return buf; }
        if (kernel_class == CKKSMI_K_CONV_COLS_TAIL) { snprintf(buf, sizeof(buf), "modup_cols_kernel<%d, %d, 3>", q, c->k + 1); return buf; }
        if (kernel_class == CKKSMI_K_CONV_COLS_MERGED) { snprintf(buf, sizeof(buf), "modup_cols_kernel<%d, %d, 2>", q, c->k + 1); return buf; }
    }
    return names[kernel_class];
}

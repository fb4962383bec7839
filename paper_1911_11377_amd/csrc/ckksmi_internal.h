// Internal declarations shared by the host code and the kernel launchers.
#pragma once
#include <atomic>
#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/ckksmi.h"
#include "../../include/ckksmi_profile.h"

typedef uint64_t u64;
typedef int64_t i64;
typedef unsigned __int128 u128;

#define CKKSMI_MAX_SPECIAL 4
#define CKKSMI_MAX_ALPHA 4
#define CKKSMI_MAX_MODULI 72
#define CKKSMI_MAX_KEYS 64     // distinct switching keys one launch can address (tables of pointers travel as kernel arguments)
#define CKKSMI_FLAG_SLOTS 64    // overflow words of the device encoder: calls in flight at once on one context
#define CKKSMI_MAX_ITEMS 256   // items per key-switch sweep (per-item tables travel as kernel arguments)

// ---- host integer helpers (host_math.cpp) ----
namespace hm {
inline u64 mulmod(u64 a, u64 b, u64 q) { return (u64)((u128)a * b % q); }
inline u64 addmod(u64 a, u64 b, u64 q) { u64 s = a + b; return s >= q ? s - q : s; }
inline u64 submod(u64 a, u64 b, u64 q) { return a >= b ? a - b : a + q - b; }
u64 powmod(u64 a, u64 e, u64 q);
u64 invmod(u64 a, u64 q);
u64 signed_mod(i64 v, u64 q);
bool is_prime(u64 n);
bool find_primes(int bits, int logN, int count, const std::vector<u64> &taken, std::vector<u64> &out);
u64 find_psi(u64 q, int logN);
inline u64 brev(u64 x, int bits) { u64 r = 0; for (int i = 0; i < bits; i++) { r = (r << 1) | (x & 1); x >>= 1; } return r; }
}  // namespace hm

// A multiplicand w prepared for the floating-point modular product: the balanced
// representative of w (|w| <= p/2) and the rounded quotient w/p.
struct WMul { double w, wp; };

// Per-modulus constants used by every kernel.
struct ModConst { double p, pinv; };

// Constants of one DivRound (ModDown over the special primes, or rescale by one q).
struct DivRoundHost {
    int nb = 0;
    int b_idx[CKKSMI_MAX_SPECIAL];
    std::vector<double> hb;     // [nb]      floor(Bbar/2) mod b_m
    std::vector<WMul> invb;     // [nb]      (Bbar/b_m)^-1 mod b_m
    std::vector<WMul> conv;     // [nb][T]   (Bbar/b_m) mod c
    std::vector<double> hc;     // [T]       floor(Bbar/2) mod c
    std::vector<WMul> Binv;     // [T]       Bbar^-1 mod c
    std::vector<double> Bmod;   // [T]       Bbar mod c
};

struct DivRoundDev {
    int nb;
    int b_idx[CKKSMI_MAX_SPECIAL];
    double hb[CKKSMI_MAX_SPECIAL];
    WMul invb[CKKSMI_MAX_SPECIAL];
    const WMul *conv;  // device [nb][T]
    const double *hc;  // device [T]
    const WMul *Binv;  // device [T]
    // exact form (conversion overshoot removed): 1/b_m as a double, Bbar mod c
    double invb_f[CKKSMI_MAX_SPECIAL];
    const double *Bmod;  // device [T]
};

// Last-stage constants of an inverse transform that also multiplies by a constant c and adds a
// constant to every coefficient: ninv = c/N, wlast = c*psi^-brev(1)/N, result + cadd.
struct FinConst { WMul ninv, wlast; double cadd, pad; };

// bit t set: modulus t is >= 2^50 (tighter lazy-reduction schedule).  Travels in kernel arguments so that the choice
// of code path does not wait for a memory load.
struct P51Mask { unsigned long long w[2]; };

struct ProfRec { int kid; double units; void *start, *stop; };

struct ckksmi_ctx {
    bool prof_on = false;
    int ntt_target_wgs = 8192;  // workgroups a transform launch aims for before it starts looping over items (ckksmi_tune)
    std::vector<ProfRec> prof;

    int logN = 0, n_q = 0, k = 0, alpha = 1, T = 0, beta_top = 0;
    u64 N = 0;
    int device = -1;
    int last_hip_error = 0;
    std::vector<u64> mod, psi;

    // host transform tables (integer): psi powers in bit-reversed order
    std::vector<std::vector<u64>> h_fwd, h_inv;  // [T][N]
    std::vector<u64> h_ninv;                     // [T]

    // ---- device tables ----
    ModConst *d_mod = nullptr;   // [T]
    WMul *d_pow24 = nullptr;     // [T] 2^24 mod p (matrix-core MAC: recombination of the digit diagonals)
    WMul *d_tw_fwd = nullptr;    // [T][N]  psi^brev(x), x in [1,N)
    WMul *d_tw_inv = nullptr;    // [T][N]  psi^-brev(x); entry 0 holds N^-1
    WMul *d_tw_inv_last = nullptr;  // [T]   psi^-brev(1) * N^-1  (last inverse stage)
    WMul *d_tw_ninv = nullptr;      // [T]   N^-1
    double *d_tww_fwd = nullptr;    // [T][N] balanced twiddles only (register-tiled kernels recompute w/p)
    double *d_tww_inv = nullptr;    // [T][N]
    // ModUp: digit j, number of limbs present nd (1..alpha), source a, target t
    WMul *d_modup_inv = nullptr; // [beta_top][alpha][alpha]
    WMul *d_modup_c = nullptr;   // [beta_top][alpha][alpha][T]
    // DivRound tables: index 0 = ModDown over specials, 1 + i = rescale dropping q_i
    std::vector<DivRoundDev> divround;
    std::vector<void *> dev_allocs;

    // fused path (N = 2^16): last-stage constants of the inverse transforms that produce conversion inputs
    FinConst *d_fin_modup = nullptr;    // [n_q + 1][n_q]  level, limb
    FinConst *d_fin_moddown = nullptr;  // [k]
    FinConst *d_fin_rescale = nullptr;  // [n_q]  dropped limb
    unsigned *d_slot_exp = nullptr;     // [N/2] 5^k mod 2N (device-side encoding)
    void *d_ctw = nullptr;              // [N] complex doubles zeta^-brev(x), zeta = exp(i*pi/N)
    int *d_flag = nullptr;              // CKKSMI_FLAG_SLOTS words: one is raised by a kernel that meets an unencodable value
    std::atomic<unsigned> flag_next{0}; // the next call's word
    FinConst *d_fin_tail = nullptr;     // [n_q + 1][CKKSMI_MAX_SPECIAL]  level, {plain inverse of q_{level-1}, ModDown's constants}
    FinConst *d_fin_merged = nullptr;   // [n_q + 1][CKKSMI_MAX_SPECIAL]  level, member of {q_{level-1}, p_0 ..}
    std::vector<DivRoundDev> divround_merged;  // [n_q + 1] by level; nb == 0 where unavailable
    std::vector<WMul> h_pmod;           // [T] P mod q_i (zero for the special primes)
    std::vector<WMul> h_Pinv;           // [T] P^-1 mod q_i
    WMul *d_pmod = nullptr;             // device copy (k > 0)
    bool merged_ok = false;             // merged division available: k > 0 and k + 1 <= CKKSMI_MAX_SPECIAL
    P51Mask p51mask = {{0, 0}};
    bool fused = false;  // 2^12 <= N <= 2^16: register-tiled passes with the limb-wise steps fused into them

    // registered Galois keys
    std::vector<std::pair<int, const u64 *>> galois;

    ModConst h_modc[CKKSMI_MAX_MODULI];
};

// host_math.cpp
WMul make_wmul(u64 w, u64 p);
void build_host_tables(ckksmi_ctx *c);
void host_ntt(const ckksmi_ctx *c, int t, u64 *a);
void host_intt(const ckksmi_ctx *c, int t, u64 *a);
DivRoundHost make_divround(const ckksmi_ctx *c, const std::vector<int> &bidx);
void make_modup_tables(const ckksmi_ctx *c, std::vector<WMul> &inv, std::vector<WMul> &cc);

// device side (ckksmi_device.hip)
int dev_upload_tables(ckksmi_ctx *c);
void dev_free_tables(ckksmi_ctx *c);

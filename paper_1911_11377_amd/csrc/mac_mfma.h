// Convolution / fully-connected multiply-accumulate on the matrix cores.
//
// out[o, pos, word] = sum_tap W[o, tap] * in[tap(pos), word]  (mod p) is a dense contraction over the taps: per prime
// an (O x K) integer weight matrix times a (K x words) matrix of ciphertext words, the same weight matrix for every
// word and every output position.  The operands are 50-bit, the matrix cores multiply 8-bit integers, so both sides
// are written in balanced base-256 digits,
//     x = sum_i x_i 256^i,  w = sum_j w_j 256^j,  x_i, w_j in [-128, 127],  7 digits each (|value| < 2^55),
// and the product sum becomes 49 int8 contractions whose int32 results are added on the 13 diagonals d = i + j:
//     sum_tap x*w = sum_d 256^d * D_d,   D_d = sum_{i+j=d} sum_tap x_i w_j.
// Everything is exact: |x_i w_j| <= 2^14, a diagonal holds at most 7 digit pairs, so K <= 16384 taps keep |D_d| < 2^31.
// The digits cost nothing to extract: adding 0x80 to every byte of the 64-bit word propagates the carries, and the
// bytes of the sum, each with its top bit flipped, are the balanced digits (byte i = digit i).
//
// Instruction: v_mfma_i32_16x16x64_i8.  Lane l supplies 16 bytes of A (row l%16, k-group l/16) and 16 bytes of B
// (column l%16, same k-group) and holds D[row 4*(l/16)+r][column l%16], r < 4.  Which 16 of the 64 k-indices a k-group
// covers is free as long as A and B agree; here k-group g, byte t is tap kb*64 + 16*g + t.
//
// Workgroup = 4 waves; wave w owns 16 consecutive words, all waves share the A fragments (32 output channels x 64 taps
// x 7 digits = 14 KB per k-step) through LDS.  Per k-step a lane loads the 16 words (its word, its k-group's taps),
// turns them into digits, transposes them bytewise into the 7 B fragments and issues 7 x 7 x 2 MFMAs.
#pragma once

#define MM_WORDS 64    // words per workgroup
#define MM_MB 2        // 16-channel blocks per workgroup
#define MM_CH (16 * MM_MB)
#define MM_DIG 7       // base-256 digits per operand
#define MM_KMAX 16384  // taps (padded) that keep the int32 diagonals exact
#define MM_BIAS 0x0080808080808080ull

#ifdef CKKSMI_EMULATE
typedef int v4i __attribute__((vector_size(16)));
v4i emu_mfma_i32_16x16x64_i8(v4i a, v4i b, v4i c);
static inline unsigned emu_perm_b32(unsigned hi, unsigned lo, unsigned sel) {
    const unsigned long long v = ((unsigned long long)hi << 32) | lo;
    unsigned r = 0;
    for (int i = 0; i < 4; i++) r |= (unsigned)((v >> (8 * ((sel >> (8 * i)) & 7))) & 0xff) << (8 * i);
    return r;
}
#define MM_MFMA(a, b, c) emu_mfma_i32_16x16x64_i8(a, b, c)
#define MM_PERM(hi, lo, sel) emu_perm_b32(hi, lo, sel)
#else
typedef int v4i __attribute__((ext_vector_type(4)));
#define MM_MFMA(a, b, c) __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0)
#define MM_PERM(hi, lo, sel) __builtin_amdgcn_perm(hi, lo, sel)
#endif

// One tap packed in 32 bits: bits 0..21 (c*in_rows + u)*W + v = ciphertext index relative to the window origin,
// bits 22..26 kernel row u, bits 27..31 kernel column v; u = 31 marks a padding entry beyond the last tap.
// A second table holds delta * 2*level (the tap's limb-row offset) for windows that lie wholly inside the image, where
// no tap needs a bounds check; entries beyond the last tap are 0 there: their weights are zero, any word will do.
typedef unsigned TapEnt;
#define MM_TAP_DELTA_MAX (1u << 22)
#define MM_TAP_KMAX 30  // largest kernel height / width

struct MacMfmaArgs {
    const u64d *in;       // [C][in_rows][W] ciphertexts
    u64d *out;            // [O][out_rows][Wo]
    const v4i *afrag;     // [level][Kb][Mg][MM_MB][MM_DIG][64 lanes] 16-byte A fragments
    const TapEnt *taps;   // [2][Kb*64]: packed entries, then premultiplied offsets
    const ModConst *modc;
    const WMul *pow24;    // 2^24 mod p per modulus
    int logN, level;
    int H, W, O, kh, kw, stride, pad, Wo;
    int in_row0, in_rows, out_row0, out_rows;
    int Kb, Mg;
    unsigned positions;                  // out_rows * Wo
    unsigned long long total_wgs, real_wgs;  // grid size (multiple of 8) and the number of real workgroups
};

// One thread per 16-byte A fragment chunk, plus the tap table.
__global__ __launch_bounds__(EW_THREADS) void mac_prepare_mfma_kernel(const long long *w, v4i *afrag, TapEnt *taps, const ModConst *modc, int level,
                                                                      int O, int C, int kh, int kw, int in_rows, int W, int Kb, int Mg) {
    const size_t idx = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    const int K = C * kh * kw;
    if (idx < (size_t)Kb * 64) {
        const int k = (int)idx;
        TapEnt e = 31u << 22;
        if (k < K) {
            const unsigned c = k / (kh * kw), u = (k / kw) % kh, v = k % kw;
            e = ((c * in_rows + u) * W + v) | (u << 22) | (v << 27);
        }
        taps[k] = e;
        taps[(size_t)Kb * 64 + k] = k < K ? (e & (MM_TAP_DELTA_MAX - 1)) * (unsigned)(2 * level) : 0u;
    }
    const size_t total = (size_t)level * Kb * Mg * MM_MB * MM_DIG * 64;
    if (idx >= total) return;
    size_t r = idx;
    const int lane = (int)(r % 64); r /= 64;
    const int j = (int)(r % MM_DIG); r /= MM_DIG;
    const int mb = (int)(r % MM_MB); r /= MM_MB;
    const int mg = (int)(r % Mg); r /= Mg;
    const int kb = (int)(r % Kb); r /= Kb;
    const int i = (int)r;
    const long long q = (long long)modc[i].p;
    const int m = (mg * MM_MB + mb) * 16 + lane % 16;
    unsigned bytes[4] = {0, 0, 0, 0};
    for (int t = 0; t < 16; t++) {
        const int k = kb * 64 + 16 * (lane / 16) + t;
        long long bal = 0;
        if (m < O && k < K) {
            bal = w[(size_t)m * K + k] % q;  // (-q, q)
            if (bal > q / 2) bal -= q;
            if (bal < -(q / 2)) bal += q;
        }
        const unsigned long long dig = ((unsigned long long)bal + MM_BIAS) ^ MM_BIAS;
        bytes[t / 4] |= (unsigned)((dig >> (8 * j)) & 0xff) << (8 * (t % 4));
    }
    v4i f;
    f[0] = (int)bytes[0]; f[1] = (int)bytes[1]; f[2] = (int)bytes[2]; f[3] = (int)bytes[3];
    afrag[idx] = f;
}

// 4x4 byte transpose: a[t] holds digits (bytes) j0..j0+3 of tap t; out[j] = those digits of taps 0..3
__device__ __forceinline__ void transpose4(const unsigned (&a)[4], unsigned (&o)[4]) {
    const unsigned p01l = MM_PERM(a[1], a[0], 0x05010400u), p01h = MM_PERM(a[1], a[0], 0x07030602u);
    const unsigned p23l = MM_PERM(a[3], a[2], 0x05010400u), p23h = MM_PERM(a[3], a[2], 0x07030602u);
    o[0] = MM_PERM(p23l, p01l, 0x05040100u);
    o[1] = MM_PERM(p23l, p01l, 0x07060302u);
    o[2] = MM_PERM(p23h, p01h, 0x05040100u);
    o[3] = MM_PERM(p23h, p01h, 0x07060302u);
}

// Request the 16 words of one k-step (taps kb*64 + 16g + t of this lane's word) from their tap entries, and this
// thread's share of the step's A fragments.  INTERIOR: the window lies inside the image, the entries are limb-row
// offsets and every load is valid.  Otherwise a tap on padding reads limb row 0 of the strip instead (always valid) and
// is zeroed when the digits are formed: bit t of the returned mask says tap t is real.
#define MM_ACHUNKS ((MM_MB * MM_DIG * 64 + 255) / 256)
template <bool INTERIOR>
__device__ __forceinline__ unsigned mm_issue_loads(const MacMfmaArgs &A, const TapEnt (&ent)[16], int iy0, int ix0, int origin, const u64d *inw,
                                                   const v4i *asrc, unsigned tid, u64d (&x)[16], v4i (&ap)[MM_ACHUNKS]) {
    unsigned mask = 0;
    const unsigned twoL = 2u * (unsigned)A.level;
#pragma unroll
    for (int t = 0; t < 16; t++) {
        const unsigned e = ent[t];
        unsigned row;  // limb row of the tap's ciphertext: ciphertext index * 2*level, below 2^30
        if (INTERIOR) {
            row = e + (unsigned)origin * twoL;
        } else {
            const int iy = iy0 + (int)((e >> 22) & 31u), ix = ix0 + (int)(e >> 27);
            const bool ok = (unsigned)iy < (unsigned)A.H && (unsigned)ix < (unsigned)A.W;
            row = ok ? __umul24((unsigned)(origin + (int)(e & (MM_TAP_DELTA_MAX - 1))), twoL) : 0u;
            mask |= ok ? 1u << t : 0u;
        }
        x[t] = inw[(size_t)row << A.logN];
    }
#pragma unroll
    for (int e = 0; e < MM_ACHUNKS; e++) {
        const unsigned idx = tid + 256u * e;
        ap[e] = asrc[idx < MM_MB * MM_DIG * 64 ? idx : 0];
    }
    return mask;
}

// grid: 1-D, `total` workgroups rounded up to a multiple of 8.  Workgroups go to the 8 XCDs round-robin by linear id and
// each XCD has its own L2, so the id is first turned into v = (id % 8) * (total / 8) + id / 8: every XCD then walks a
// contiguous range of v, in which the channel group is the fastest index, then the output position, then the word
// block, then the limb -- consecutive workgroups of one XCD read the same input words (other channels, overlapping
// windows) and find them in its L2.
template <bool INTERIOR>
__device__ __forceinline__ void conv_mac_mfma_body(const MacMfmaArgs &A, v4i *a_lds, unsigned mg, unsigned pos, unsigned wb, unsigned lc);

__global__ __launch_bounds__(256, 2) void conv_mac_mfma_kernel(MacMfmaArgs A) {
    __shared__ v4i a_lds[MM_MB * MM_DIG * 64];
    const unsigned N = 1u << A.logN;
    const size_t per_xcd = A.total_wgs / 8;
    size_t v = (size_t)(blockIdx.x % 8u) * per_xcd + blockIdx.x / 8u;
    if (v >= A.real_wgs) return;  // uniform for the workgroup
    const unsigned mg = (unsigned)(v % (unsigned)A.Mg); v /= (unsigned)A.Mg;
    const unsigned pos = (unsigned)(v % A.positions); v /= A.positions;
    const unsigned wb = (unsigned)(v % (N / MM_WORDS)); v /= (N / MM_WORDS);
    const unsigned lc = (unsigned)v;
    const int oyl = (int)(pos / (unsigned)A.Wo), ox = (int)(pos % (unsigned)A.Wo);
    const int iy0 = (A.out_row0 + oyl) * A.stride - A.pad, ix0 = ox * A.stride - A.pad;
    if (iy0 >= 0 && iy0 + A.kh <= A.H && ix0 >= 0 && ix0 + A.kw <= A.W)
        conv_mac_mfma_body<true>(A, a_lds, mg, pos, wb, lc);
    else
        conv_mac_mfma_body<false>(A, a_lds, mg, pos, wb, lc);
}

template <bool INTERIOR>
__device__ __forceinline__ void conv_mac_mfma_body(const MacMfmaArgs &A, v4i *a_lds, unsigned mg, unsigned pos, unsigned wb, unsigned lc) {
    const unsigned N = 1u << A.logN;
    const unsigned tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const unsigned i = lc % (unsigned)A.level;
    const int oyl = (int)(pos / (unsigned)A.Wo), ox = (int)(pos % (unsigned)A.Wo);
    const int iy0 = (A.out_row0 + oyl) * A.stride - A.pad, ix0 = ox * A.stride - A.pad;
    const int origin = (iy0 - A.in_row0) * A.W + ix0;
    const size_t ctw = (size_t)2 * A.level * N;
    const unsigned n = wb * MM_WORDS + wave * 16 + (lane & 15);
    const unsigned g = lane >> 4;
    const u64d *inw = A.in + (size_t)lc * N + n;
    const size_t astep = (size_t)A.Mg * (MM_MB * MM_DIG * 64);
    const v4i *asrc = A.afrag + ((size_t)i * A.Kb * A.Mg + mg) * (MM_MB * MM_DIG * 64);

    v4i acc[2 * MM_DIG - 1][MM_MB];
#pragma unroll
    for (int d = 0; d < 2 * MM_DIG - 1; d++)
#pragma unroll
        for (int mb = 0; mb < MM_MB; mb++) acc[d][mb] = v4i{0, 0, 0, 0};

    // the tap entries run two steps ahead of the matrix work, the words and A fragments one step ahead
    u64d x[16];
    v4i ap[MM_ACHUNKS];
    TapEnt ent[16];
    const TapEnt *tp = A.taps + (INTERIOR ? (size_t)A.Kb * 64 : 0) + 16 * g;
#pragma unroll
    for (int t = 0; t < 16; t++) ent[t] = tp[t];
    unsigned mask = mm_issue_loads<INTERIOR>(A, ent, iy0, ix0, origin, inw, asrc, tid, x, ap);
    if (A.Kb > 1) {
#pragma unroll
        for (int t = 0; t < 16; t++) ent[t] = tp[64 + t];
    }
    for (int kb = 0; kb < A.Kb; kb++) {
        __syncthreads();  // the previous step's readers of the A fragments are done
#pragma unroll
        for (int e = 0; e < MM_ACHUNKS; e++) {
            const unsigned idx = tid + 256u * e;
            if (idx < MM_MB * MM_DIG * 64) a_lds[idx] = ap[e];
        }
        __syncthreads();
        // digits, then bytewise transpose into the B fragments: bf[d] = digit d of the 16 taps
        unsigned lo[16], hi[16];
#pragma unroll
        for (int t = 0; t < 16; t++) {
            const u64d dg = (INTERIOR || ((mask >> t) & 1u)) ? (x[t] + MM_BIAS) ^ MM_BIAS : 0ull;
            lo[t] = (unsigned)dg;
            hi[t] = (unsigned)(dg >> 32);
        }
        v4i bf[8];
#pragma unroll
        for (int q4 = 0; q4 < 4; q4++) {
            unsigned a4[4], o4[4];
#pragma unroll
            for (int t = 0; t < 4; t++) a4[t] = lo[4 * q4 + t];
            transpose4(a4, o4);
#pragma unroll
            for (int d = 0; d < 4; d++) bf[d][q4] = (int)o4[d];
#pragma unroll
            for (int t = 0; t < 4; t++) a4[t] = hi[4 * q4 + t];
            transpose4(a4, o4);
#pragma unroll
            for (int d = 0; d < 4; d++) bf[4 + d][q4] = (int)o4[d];
        }
        // the next step's operands are requested before this step's matrix work so that their latency hides behind it
        if (kb + 1 < A.Kb) {
            mask = mm_issue_loads<INTERIOR>(A, ent, iy0, ix0, origin, inw, asrc + (size_t)(kb + 1) * astep, tid, x, ap);
            if (kb + 2 < A.Kb) {
#pragma unroll
                for (int t = 0; t < 16; t++) ent[t] = tp[(kb + 2) * 64 + t];
            }
        }
        SCHED_FENCE();
#pragma unroll
        for (int j = 0; j < MM_DIG; j++) {
            v4i af[MM_MB];
#pragma unroll
            for (int mb = 0; mb < MM_MB; mb++) af[mb] = a_lds[(mb * MM_DIG + j) * 64 + lane];
#pragma unroll
            for (int d = 0; d < MM_DIG; d++)
#pragma unroll
                for (int mb = 0; mb < MM_MB; mb++) acc[d + j][mb] = MM_MFMA(af[mb], bf[d], acc[d + j][mb]);
        }
    }

    // value = sum_d 256^d D_d: three diagonals combine exactly in a double (< 2^48), the groups by Horner in 2^24
    const ModConst mc = A.modc[i];
    const WMul P24 = A.pow24[i];
#pragma unroll
    for (int mb = 0; mb < MM_MB; mb++)
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const int m = (int)(mg * MM_MB + mb) * 16 + 4 * (int)g + r;
            double grp[5];
#pragma unroll
            for (int q = 0; q < 4; q++)
                grp[q] = fma(65536.0, (double)acc[3 * q + 2][mb][r], fma(256.0, (double)acc[3 * q + 1][mb][r], (double)acc[3 * q][mb][r]));
            grp[4] = (double)acc[12][mb][r];
            double v = grp[4];
#pragma unroll
            for (int q = 3; q >= 0; q--) v = mulmod_w(v, P24.w, P24.wp, mc.p) + grp[q];
            if (m < A.O)
                A.out[(((size_t)m * A.out_rows + oyl) * A.Wo + ox) * ctw + (size_t)lc * N + n] = d2u(canon(v, mc.p, mc.pinv));
        }
}

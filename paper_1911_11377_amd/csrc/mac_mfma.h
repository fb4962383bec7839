// Convolution / fully-connected multiply-accumulate on the matrix cores.
//
// out[o, pos, word] = sum_tap W[o, tap] * in[tap(pos), word]  (mod p) is a dense contraction over the taps: per prime
// an (O x K) integer weight matrix times a (K x words) matrix of ciphertext words, the same weight matrix for every
// word and every output position.  The operands are 50-bit, the matrix cores multiply signed 8-bit integers, so both
// sides are written in base-256 digits in [-128, 127], 7 each:
//     w = sum_j w_j 256^j   balanced digits of the balanced weight (add 0x80 to every byte, the carries propagate, flip
//                           the top bit of every byte; once per layer, in the preparation kernel),
//     x = B + sum_i x_i 256^i,   x_i = (byte i of x) - 128 = the byte with its top bit flipped,  B = sum_i 128 * 256^i
// (no carries on this side: one XOR per half word in the inner loop).  The product sum becomes 49 int8 contractions
// whose int32 results are added on the 13 diagonals d = i + j:
//     sum_tap x*w = sum_d 256^d * D_d + B * sum_tap w,    D_d = sum_{i+j=d} sum_tap x_i w_j.
// The last term is a constant per output channel and modulus (`wsum`, made together with the weight digits).  A tap that
// falls on padding is given x = 0, i.e. every digit -128, which the constant cancels.
// Everything is exact: |x_i w_j| <= 2^14, a diagonal holds at most 7 digit pairs, so K <= 16384 taps keep |D_d| < 2^31.
//
// Instruction: v_mfma_i32_16x16x64_i8.  Lane l supplies 16 bytes of A (row l%16, k-group l/16) and 16 bytes of B
// (column l%16, same k-group) and holds D[row 4*(l/16)+r][column l%16], r < 4.  Which 16 of the 64 k-indices a k-group
// covers is free as long as A and B agree.
//   full step  : k-group g, byte t is tap 64*kb + 16*g + t; 7 x 7 digit pairs = 49 instructions per 16 channels.
//   quad step  : the last 16 (or fewer) taps of a layer whose tap count leaves a remainder of at most 16.  All four
//                k-groups carry the SAME 16 taps and differ in the digits instead: group g supplies digit i0 - g of the
//                weights (fragment i0) and digit r + g of the words (fragment r: the word shifted right by g bytes before
//                its bytes are transposed), so one instruction adds four digit pairs of diagonal i0 + r.  The pairs of a
//                diagonal d are covered by fragments i0 = min(6, d), min(6, d) - 4, ... down to max(0, d - 6); pairs a
//                fragment reaches beyond the diagonal's ends have a zero digit on one side.  18 instructions instead of 49.
//
// Three kernels.  All: workgroup = 4 waves, a wave works on 16 consecutive words, 32 output channels per workgroup, the A
// fragments (weight digits, 14 KB per step) are shared through LDS; per step a lane takes the 16 words of its taps,
// flips the top bits, transposes the bytes into the 7 B fragments (v_perm_b32) and issues the matrix instructions.
//   conv_mac_mfma_kernel          any tap count: one output position per workgroup, the A fragments stream through LDS
//                                 step by step (two barriers per step).
//   conv_mac_mfma_resident_kernel at most MM_RES_STEPS steps (the last one may be a quad step): the layer's A fragments
//                                 stay in LDS, a workgroup walks several output positions without a barrier, and the words
//                                 of the next step (possibly of the next position) are requested before the current
//                                 step's matrix work.  Workgroups that run side by side on one XCD take neighbouring
//                                 positions of the same 64-word block, so window overlaps are served by that XCD's L2.
//   conv_mac_mfma_strip_kernel    at most 2 steps and a narrow window: the four waves take four neighbouring output
//                                 positions (1 x 4 or 2 x 2) of ONE 16-word block, and the union of their windows (per
//                                 channel kh + (TY-1)*stride rows of kw + (TX-1)*stride pixels, 128 bytes each) is staged
//                                 once in LDS, zeros where the window leaves the image.  Every input line crosses the vector memory path once per four
//                                 positions instead of once per position and wave; the words come out of LDS with
//                                 offsets that never change, so the inner loop computes no addresses.
#pragma once

#define MM_WORDS 64    // words per workgroup
#define MM_MB 2        // 16-channel blocks per workgroup
#define MM_CH (16 * MM_MB)
#define MM_DIG 7       // base-256 digits per operand
#define MM_KMAX 16384  // taps (padded) that keep the int32 diagonals exact
#define MM_BIAS 0x0080808080808080ull
#define MM_FRAG (MM_MB * MM_DIG * 64)  // 16-byte A fragment chunks per step and channel group
#define MM_RES_STEPS 4                 // steps whose A fragments the resident kernel keeps in LDS
#define MM_STRIP_STEPS 2               // the same for the strip kernel
#define MM_STRIP_POS 4                 // output positions (one per wave) that share a staged strip
#define MM_STRIP_LINES 192             // 128-byte lines of a strip buffer (24 KB; two buffers)
#define MM_STRIP_ROUNDS (MM_STRIP_LINES / 32)  // a round: 256 threads x 16 bytes = 32 lines

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
#define MM_UNIFORM(v) (v)
#else
typedef int v4i __attribute__((ext_vector_type(4)));
#define MM_MFMA(a, b, c) __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0)
#define MM_PERM(hi, lo, sel) __builtin_amdgcn_perm(hi, lo, sel)
#define MM_UNIFORM(v) __builtin_amdgcn_readfirstlane(v)  // the same in every lane of the wave: keep it in a scalar register
#endif

// One tap packed in 32 bits: bits 0..21 (c*in_rows + u)*W + v = ciphertext index relative to the window origin,
// bits 22..26 kernel row u, bits 27..31 kernel column v; u = 31 marks a padding entry beyond the last tap.
// Table slot kb*64 + 16*g + t belongs to step kb, k-group g, byte t.  For windows that lie wholly inside the image no tap
// needs a bounds check; they use premultiplied offsets instead: a second 32-bit table holds delta * 2*level (limb rows), a
// 64-bit table the same in bytes (delta * 2*level * N * 8).  Entries beyond the last tap are 0 there: their weights are
// zero, any word will do.
typedef unsigned TapEnt;
#define MM_TAP_DELTA_MAX (1u << 22)
#define MM_TAP_KMAX 30  // largest kernel height / width

struct MacMfmaArgs {
    const u64d *in;       // [C][in_rows][W] ciphertexts
    u64d *out;            // [O][out_rows][Wo]
    const v4i *afrag;     // [level][Kb][Mg][MM_MB][MM_DIG][64 lanes] 16-byte A fragments
    const TapEnt *taps;   // [2][Kb*64]: packed entries, then premultiplied limb-row offsets
    const unsigned long long *off64;  // [Kb*64] premultiplied byte offsets
    const double *wsum;   // [level][Mg*MM_CH]  B * sum_tap w mod p, canonical
    const unsigned *tapoff;  // [Kb*64] strip kernel: byte offset of the tap's line in the strip, ((c*SR + u)*SC + v)*128
    const ModConst *modc;
    const WMul *pow24;    // 2^24 mod p per modulus
    int logN, level;
    int C, H, W, O, kh, kw, stride, pad, Wo;
    int in_row0, in_rows, out_row0, out_rows;
    int Kb, Mg;
    int quad;                            // the last step is a quad step
    unsigned positions;                  // out_rows * Wo
    int TY, TX;                          // strip kernel: the four waves' positions form a TY x TX block (1 x 4 or 2 x 2)
    int SR, SC, spr;                     // ... strip rows per channel kh + (TY-1)*stride, pixels per row kw + (TX-1)*stride, tiles per output row
    unsigned nrun, run;                  // resident kernel: workgroups that share a 64-word block; each takes `run` consecutive positions
    unsigned long long total_wgs, real_wgs;  // grid size (multiple of 8) and the number of real workgroups
};

// tap index of table slot (kb, g, t)
__host__ __device__ __forceinline__ int mm_slot_tap(int kb, int g, int t, int Kb, int quad) {
    return (quad && kb == Kb - 1) ? 64 * kb + t : 64 * kb + 16 * g + t;
}

// One thread per 16-byte A fragment chunk, per tap-table slot and per wsum entry.
__global__ __launch_bounds__(EW_THREADS) void mac_prepare_mfma_kernel(const long long *w, v4i *afrag, TapEnt *taps, unsigned long long *off64,
                                                                      unsigned *tapoff, int SR, int SC, double *wsum, const ModConst *modc, int level, int logN, int O, int C,
                                                                      int kh, int kw, int in_rows, int W, int Kb, int Mg, int quad) {
    const size_t idx = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    const int K = C * kh * kw;
    if (idx < (size_t)Kb * 64) {
        const int slot = (int)idx;
        const int k = mm_slot_tap(slot / 64, (slot % 64) / 16, slot % 16, Kb, quad);
        TapEnt e = 31u << 22;
        if (k < K) {
            const unsigned c = k / (kh * kw), u = (k / kw) % kh, v = k % kw;
            e = ((c * in_rows + u) * W + v) | (u << 22) | (v << 27);
        }
        taps[slot] = e;
        const unsigned rows = k < K ? (e & (MM_TAP_DELTA_MAX - 1)) * (unsigned)(2 * level) : 0u;
        taps[(size_t)Kb * 64 + slot] = rows;
        off64[slot] = ((unsigned long long)rows << logN) * 8ull;
        tapoff[slot] = k < K ? (unsigned)((((k / (kh * kw)) * SR + (k / kw) % kh) * SC + k % kw) * 128) : 0u;
    }
    if (idx < (size_t)level * Mg * MM_CH) {
        const int i = (int)(idx / ((size_t)Mg * MM_CH)), m = (int)(idx % ((size_t)Mg * MM_CH));
        const long long q = (long long)modc[i].p;
        long long s = 0;  // sum of the balanced weights mod q, in (-q, q)
        if (m < O)
            for (int k = 0; k < K; k++) s = (s + w[(size_t)m * K + k] % q) % q;
        if (s < 0) s += q;
        // B * s mod q by Horner over the 7 bytes of B (all 0x80): r < q < 2^51, so 256 r + 128 s < 2^60
        unsigned long long r = 0;
        for (int j = 0; j < MM_DIG; j++) r = (r * 256ull + 128ull * (unsigned long long)s) % (unsigned long long)q;
        wsum[idx] = (double)r;
    }
    const size_t total = (size_t)level * Kb * Mg * MM_FRAG;
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
    const int g = lane / 16;
    const bool qs = quad && kb == Kb - 1;
    const int dig = qs ? j - g : j;  // quad step: fragment i0 = j holds digit i0 - g in k-group g
    unsigned bytes[4] = {0, 0, 0, 0};
    for (int t = 0; t < 16; t++) {
        const int k = mm_slot_tap(kb, g, t, Kb, quad);
        long long bal = 0;
        if (m < O && k < K && dig >= 0) {
            bal = w[(size_t)m * K + k] % q;  // (-q, q)
            if (bal > q / 2) bal -= q;
            if (bal < -(q / 2)) bal += q;
        }
        const unsigned long long d7 = ((unsigned long long)bal + MM_BIAS) ^ MM_BIAS;
        bytes[t / 4] |= (unsigned)((d7 >> (8 * (dig < 0 ? 0 : dig))) & 0xff) << (8 * (t % 4));
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

// The 16 words of one step as B fragments: bf[d] = digit d (+ shift_bytes) of the 16 taps.  MASKED: bit t of mask says tap
// t is real; the others count as x = 0.  shift_bits = 8 * g in a quad step, 0 otherwise.
template <bool MASKED, bool QUAD>
__device__ __forceinline__ void mm_b_fragments(const u64d (&x)[16], unsigned mask, unsigned shift_bits, v4i (&bf)[8]) {
    unsigned lo[16], hi[16];
#pragma unroll
    for (int t = 0; t < 16; t++) {
        u64d dg = ((!MASKED || ((mask >> t) & 1u)) ? x[t] : 0ull) ^ MM_BIAS;
        if (QUAD) dg >>= shift_bits;
        lo[t] = (unsigned)dg;
        hi[t] = (unsigned)(dg >> 32);
    }
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
}

// The matrix work of one step from A fragments in LDS (`a`: [MM_MB][MM_DIG][64]) for the 16-channel blocks MB0 .. MB1 - 1.
// FIRST: the accumulators start here.
template <bool FIRST, bool QUAD, int MB0 = 0, int MB1 = MM_MB>
__device__ __forceinline__ void mm_step(const v4i *a, unsigned lane, const v4i (&bf)[8], v4i (&acc)[2 * MM_DIG - 1][MM_MB]) {
    const v4i zero = v4i{0, 0, 0, 0};
    if (!QUAD) {
#pragma unroll
        for (int j = 0; j < MM_DIG; j++) {
            v4i af[MM_MB];
#pragma unroll
            for (int mb = MB0; mb < MB1; mb++) af[mb] = a[(mb * MM_DIG + j) * 64 + lane];
#pragma unroll
            for (int d = 0; d < MM_DIG; d++)
#pragma unroll
                for (int mb = MB0; mb < MB1; mb++)  // diagonal d + j is first touched at j = 0, or at d = 6
                    acc[d + j][mb] = MM_MFMA(af[mb], bf[d], (FIRST && (j == 0 || d == MM_DIG - 1)) ? zero : acc[d + j][mb]);
        }
    } else {
#pragma unroll
        for (int i0 = 0; i0 < MM_DIG; i0++) {
            v4i af[MM_MB];
#pragma unroll
            for (int mb = MB0; mb < MB1; mb++) af[mb] = a[(mb * MM_DIG + i0) * 64 + lane];
#pragma unroll
            for (int d = i0; d < i0 + MM_DIG; d++) {
                // fragment i0 serves diagonal d when i0 = min(6, d) - 4n >= max(0, d - 6)
                const int ihi = d < MM_DIG ? d : MM_DIG - 1, ilo = d < MM_DIG ? 0 : d - (MM_DIG - 1);
                if (i0 > ihi || i0 < ilo || ((ihi - i0) & 3) != 0) continue;
#pragma unroll
                for (int mb = MB0; mb < MB1; mb++)  // fragments come in ascending order: the diagonal's lowest one starts it
                    acc[d][mb] = MM_MFMA(af[mb], bf[d - i0], (FIRST && i0 - 4 < ilo) ? zero : acc[d][mb]);
            }
        }
    }
}

// value = sum_d 256^d D_d + wsum: three diagonals combine exactly in a double (< 2^48), the groups by Horner in 2^24.
// Lane (g, column) holds rows 4g + r of each 16-channel block; outp points at channel 4g of the group, mstride = words
// between output channels.  ALL: every channel of the group exists (no test per value: the eight chains stay one
// straight-line block that the scheduler can interleave).
template <bool ALL, int MB0 = 0, int MB1 = MM_MB>
__device__ __forceinline__ void mm_recombine_store_impl(const v4i (&acc)[2 * MM_DIG - 1][MM_MB], const ModConst mc, const WMul P24,
                                                        const double (&ws)[MM_MB][4], u64d *outp, size_t mstride, int m0, int O) {
#pragma unroll
    for (int mb = MB0; mb < MB1; mb++)
#pragma unroll
        for (int r = 0; r < 4; r++) {
            double grp[5];
#pragma unroll
            for (int q = 0; q < 4; q++)
                grp[q] = fma(65536.0, (double)acc[3 * q + 2][mb][r], fma(256.0, (double)acc[3 * q + 1][mb][r], (double)acc[3 * q][mb][r]));
            grp[4] = (double)acc[12][mb][r];
            double v = grp[4];
#pragma unroll
            for (int q = 3; q >= 0; q--) v = mulmod_w(v, P24.w, P24.wp, mc.p) + grp[q];
            const u64d val = d2u(canon(v + ws[mb][r], mc.p, mc.pinv));
            if (ALL || m0 + mb * 16 + r < O) outp[(size_t)(mb * 16 + r) * mstride] = val;
        }
}
// mg: the channel group (the same for the whole workgroup)
__device__ __forceinline__ void mm_recombine_store(const v4i (&acc)[2 * MM_DIG - 1][MM_MB], const ModConst mc, const WMul P24,
                                                   const double (&ws)[MM_MB][4], u64d *outp, size_t mstride, unsigned mg, unsigned g, int O) {
    const int m0 = (int)(mg * MM_CH + 4 * g);
    if ((int)((mg + 1) * MM_CH) <= O)
        mm_recombine_store_impl<true>(acc, mc, P24, ws, outp, mstride, m0, O);
    else
        mm_recombine_store_impl<false>(acc, mc, P24, ws, outp, mstride, m0, O);
}

// Request the 16 words of one k-step (taps kb*64 + 16g + t of this lane's word) from their tap entries, and this
// thread's share of the step's A fragments.  INTERIOR: the window lies inside the image, the entries are limb-row
// offsets and every load is valid.  Otherwise a tap on padding reads limb row 0 of the strip instead (always valid) and
// counts as zero when the digits are formed: bit t of the returned mask says tap t is real.
#define MM_ACHUNKS ((MM_FRAG + 255) / 256)
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
        ap[e] = asrc[idx < MM_FRAG ? idx : 0];
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
    __shared__ v4i a_lds[MM_FRAG];
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
    const unsigned tid = threadIdx.x, lane = tid & 63, wave = MM_UNIFORM(tid >> 6);
    const unsigned i = lc % (unsigned)A.level;
    const int oyl = (int)(pos / (unsigned)A.Wo), ox = (int)(pos % (unsigned)A.Wo);
    const int iy0 = (A.out_row0 + oyl) * A.stride - A.pad, ix0 = ox * A.stride - A.pad;
    const int origin = (iy0 - A.in_row0) * A.W + ix0;
    const size_t ctw = (size_t)2 * A.level * N;
    const unsigned n = wb * MM_WORDS + wave * 16 + (lane & 15);
    const unsigned g = lane >> 4;
    const u64d *inw = A.in + (size_t)lc * N + n;
    const size_t astep = (size_t)A.Mg * MM_FRAG;
    const v4i *asrc = A.afrag + ((size_t)i * A.Kb * A.Mg + mg) * MM_FRAG;

    v4i acc[2 * MM_DIG - 1][MM_MB];

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
            if (idx < MM_FRAG) a_lds[idx] = ap[e];
        }
        __syncthreads();
        v4i bf[8];
        mm_b_fragments<!INTERIOR, false>(x, mask, 0u, bf);
        // the next step's operands are requested before this step's matrix work so that their latency hides behind it
        if (kb + 1 < A.Kb) {
            mask = mm_issue_loads<INTERIOR>(A, ent, iy0, ix0, origin, inw, asrc + (size_t)(kb + 1) * astep, tid, x, ap);
            if (kb + 2 < A.Kb) {
#pragma unroll
                for (int t = 0; t < 16; t++) ent[t] = tp[(kb + 2) * 64 + t];
            }
        }
        SCHED_FENCE();
        if (kb == 0)
            mm_step<true, false>(a_lds, lane, bf, acc);
        else
            mm_step<false, false>(a_lds, lane, bf, acc);
    }

    double ws[MM_MB][4];
#pragma unroll
    for (int mb = 0; mb < MM_MB; mb++)
#pragma unroll
        for (int r = 0; r < 4; r++) ws[mb][r] = A.wsum[((size_t)i * A.Mg + mg) * MM_CH + mb * 16 + 4 * g + r];
    const int m0 = (int)(mg * MM_CH + 4 * g);
    const size_t mstride = (size_t)A.out_rows * A.Wo * ctw;
    u64d *outp = A.out + (size_t)m0 * mstride + ((size_t)oyl * A.Wo + ox) * ctw + (size_t)lc * N + n;
    mm_recombine_store(acc, A.modc[i], A.pow24[i], ws, outp, mstride, mg, g, A.O);
}

// ---------------------------------------------------------------- layers of few taps: A fragments resident in LDS
// grid: 1-D, rounded up to a multiple of 8 and spread over the XCDs as above; v = ((limb * (N/64) + word block) * nrun + c),
// workgroup c of a block takes positions c*run ... c*run + run - 1: the workgroups in flight on an XCD sweep the image
// of one or two blocks front to back, so the rows a window shares with the windows below it are still in that XCD's L2.
struct MacPos {
    int oyl, ox, iy0, ix0, origin;
    bool interior;
};
__device__ __forceinline__ MacPos mm_position(const MacMfmaArgs &A, unsigned pos) {
    MacPos P;
    P.oyl = (int)(pos / (unsigned)A.Wo);
    P.ox = (int)(pos % (unsigned)A.Wo);
    P.iy0 = (A.out_row0 + P.oyl) * A.stride - A.pad;
    P.ix0 = P.ox * A.stride - A.pad;
    P.origin = (P.iy0 - A.in_row0) * A.W + P.ix0;
    P.interior = P.iy0 >= 0 && P.iy0 + A.kh <= A.H && P.ix0 >= 0 && P.ix0 + A.kw <= A.W;
    return P;
}

// the 16 words of step kb at position P; returns the mask of real taps (all ones inside the image)
__device__ __forceinline__ unsigned mm_resident_loads(const MacMfmaArgs &A, const MacPos &P, const unsigned long long *off_lds, const TapEnt *ent_lds,
                                                      int kb, unsigned g, const u64d *inw, u64d (&x)[16]) {
    const unsigned twoL = 2u * (unsigned)A.level;
    if (P.interior) {
        // inw + origin * 2*level * N words; origin is not negative for a window inside the image
        const char *base = (const char *)(inw + ((size_t)((unsigned)P.origin * twoL) << A.logN));
#pragma unroll
        for (int t = 0; t < 16; t++) x[t] = *(const u64d *)(base + off_lds[kb * 64 + 16 * g + t]);
        return 0xffffu;
    }
    unsigned mask = 0;
#pragma unroll
    for (int t = 0; t < 16; t++) {
        const unsigned e = ent_lds[kb * 64 + 16 * g + t];
        const int iy = P.iy0 + (int)((e >> 22) & 31u), ix = P.ix0 + (int)(e >> 27);
        const bool ok = (unsigned)iy < (unsigned)A.H && (unsigned)ix < (unsigned)A.W;
        const unsigned row = ok ? __umul24((unsigned)(P.origin + (int)(e & (MM_TAP_DELTA_MAX - 1))), twoL) : 0u;
        mask |= ok ? 1u << t : 0u;
        x[t] = inw[(size_t)row << A.logN];
    }
    return mask;
}

template <int KB, bool QUAD>
__global__ __launch_bounds__(256, 2) void conv_mac_mfma_resident_kernel(MacMfmaArgs A) {
    __shared__ v4i a_lds[KB * MM_FRAG];
    __shared__ unsigned long long off_lds[KB * 64];
    __shared__ TapEnt ent_lds[KB * 64];
    __shared__ double ws_lds[MM_CH];
    const unsigned N = 1u << A.logN;
    const size_t per_xcd = A.total_wgs / 8;
    size_t v = (size_t)(blockIdx.x % 8u) * per_xcd + blockIdx.x / 8u;
    if (v >= A.real_wgs) return;  // uniform for the workgroup
    const unsigned c = (unsigned)(v % A.nrun); v /= A.nrun;
    const unsigned wb = (unsigned)(v % (N / MM_WORDS)); v /= (N / MM_WORDS);
    const unsigned lc = (unsigned)v;
    const unsigned tid = threadIdx.x, lane = tid & 63, wave = MM_UNIFORM(tid >> 6), g = lane >> 4;
    const unsigned i = lc % (unsigned)A.level;
    const size_t ctw = (size_t)2 * A.level * N;
    const unsigned n = wb * MM_WORDS + wave * 16 + (lane & 15);
    const u64d *inw = A.in + (size_t)lc * N + n;
    const size_t mstride = (size_t)A.out_rows * A.Wo * ctw;
    const unsigned shift_bits = 8u * g;

    for (unsigned s = tid; s < (unsigned)KB * 64; s += 256) {
        off_lds[s] = A.off64[s];
        ent_lds[s] = A.taps[s];
    }
    for (unsigned mg = 0; mg < (unsigned)A.Mg; mg++) {
        __syncthreads();  // readers of the previous channel group's fragments are done
#pragma unroll
        for (int kb = 0; kb < KB; kb++) {
            const v4i *asrc = A.afrag + (((size_t)i * KB + kb) * A.Mg + mg) * MM_FRAG;
            for (unsigned e = tid; e < MM_FRAG; e += 256) a_lds[kb * MM_FRAG + e] = asrc[e];
        }
        if (tid < MM_CH) ws_lds[tid] = A.wsum[((size_t)i * A.Mg + mg) * MM_CH + tid];
        __syncthreads();
        const int m0 = (int)(mg * MM_CH + 4 * g);
        u64d *outm = A.out + (size_t)m0 * mstride + (size_t)lc * N + n;

        // every wave on its own from here: no barrier until the next channel group
        u64d x[16];
        unsigned pos = c * A.run;
        const unsigned pos_end = pos + A.run < A.positions ? pos + A.run : A.positions;
        MacPos P = mm_position(A, pos);
        unsigned mask = mm_resident_loads(A, P, off_lds, ent_lds, 0, g, inw, x);
        bool masked = !P.interior;
        while (pos < pos_end) {
            v4i acc[2 * MM_DIG - 1][MM_MB];
            const MacPos Pcur = P;
#pragma unroll
            for (int kb = 0; kb < KB; kb++) {
                const bool quad = QUAD && kb == KB - 1;  // folds: kb is an unrolled constant
                v4i bf[8];
                if (quad) {
                    if (masked) mm_b_fragments<true, true>(x, mask, shift_bits, bf); else mm_b_fragments<false, true>(x, mask, shift_bits, bf);
                } else {
                    if (masked) mm_b_fragments<true, false>(x, mask, 0u, bf); else mm_b_fragments<false, false>(x, mask, 0u, bf);
                }
                // the next step's words (of the next position after the last step) are requested before the matrix work
                if (kb + 1 < KB) {
                    mask = mm_resident_loads(A, Pcur, off_lds, ent_lds, kb + 1, g, inw, x);
                } else if (pos + 1 < pos_end) {
                    P = mm_position(A, pos + 1);
                    mask = mm_resident_loads(A, P, off_lds, ent_lds, 0, g, inw, x);
                    masked = !P.interior;
                }
                SCHED_FENCE();
                const v4i *a = a_lds + kb * MM_FRAG;
                if (kb == 0) {
                    if (quad) mm_step<true, true>(a, lane, bf, acc); else mm_step<true, false>(a, lane, bf, acc);
                } else {
                    if (quad) mm_step<false, true>(a, lane, bf, acc); else mm_step<false, false>(a, lane, bf, acc);
                }
            }
            double ws[MM_MB][4];
#pragma unroll
            for (int mb = 0; mb < MM_MB; mb++)
#pragma unroll
                for (int r = 0; r < 4; r++) ws[mb][r] = ws_lds[mb * 16 + 4 * g + r];
            mm_recombine_store(acc, A.modc[i], A.pow24[i], ws, outm + ((size_t)Pcur.oyl * A.Wo + Pcur.ox) * ctw, mstride, mg, g, A.O);
            pos++;
        }
    }
}

// ---------------------------------------------------------------- narrow layers: four positions share a staged strip
// grid: 1-D, rounded up to a multiple of 8 and spread over the XCDs as above;
// v = ((limb * (N/16) + 16-word block) * nrun + c); workgroup c of a block takes tiles c*run ... c*run + run - 1.  Tile tau
// covers output rows TY*(tau / spr) + wy and columns TX*(tau % spr) + wx, wave w = wy*TX + wx; a wave whose position lies
// beyond the requested rows or the row's end computes on whatever the strip holds and stores nothing.  The strip of the
// next tile is requested before the current tile's work and written to the other buffer after it: one barrier per tile.
// Strip line (c*SR + r)*SC + col holds the block's 16 words of pixel (iy0 + r, ix0 + col) of channel c, zeros outside
// the image.
template <int KB, bool QUAD, int TY>
__global__ __launch_bounds__(256, 2) void conv_mac_mfma_strip_kernel(MacMfmaArgs A) {
    constexpr int TX = MM_STRIP_POS / TY;
    __shared__ v4i a_lds[KB * MM_FRAG];
    __shared__ v4i strip[2][MM_STRIP_LINES * 8];
    __shared__ double ws_lds[MM_CH];
    __shared__ unsigned toff_lds[KB * 64];
    const unsigned N = 1u << A.logN;
    const size_t per_xcd = A.total_wgs / 8;
    size_t v = (size_t)(blockIdx.x % 8u) * per_xcd + blockIdx.x / 8u;
    if (v >= A.real_wgs) return;  // uniform for the workgroup
    const unsigned c = (unsigned)(v % A.nrun); v /= A.nrun;
    const unsigned wb = (unsigned)(v % (N / 16)); v /= (N / 16);
    const unsigned lc = (unsigned)v;
    const unsigned tid = threadIdx.x, lane = tid & 63, wave = MM_UNIFORM(tid >> 6), g = lane >> 4;
    const unsigned wy = wave / (unsigned)TX, wx = wave % (unsigned)TX;
    const unsigned i = lc % (unsigned)A.level;
    const size_t ctw = (size_t)2 * A.level * N;
    const u64d *inw = A.in + (size_t)lc * N + wb * 16;  // the block's first word in ciphertext 0
    const size_t mstride = (size_t)A.out_rows * A.Wo * ctw;
    const unsigned shift_bits = 8u * g;
    const unsigned tiles = (unsigned)((A.out_rows + TY - 1) / TY) * (unsigned)A.spr;
    const unsigned tau0 = c * A.run, tau1 = tau0 + A.run < tiles ? tau0 + A.run : tiles;
    const unsigned lines = (unsigned)(A.C * A.SR * A.SC);

    // staging: round r, this thread moves 16 bytes (part = tid % 8) of line r*32 + tid/8
    unsigned relc[MM_STRIP_ROUNDS];   // ciphertexts from the tile's origin pixel to this thread's line
    unsigned rcol[MM_STRIP_ROUNDS];   // strip row | strip column << 8 | line exists << 31
#pragma unroll
    for (int r = 0; r < MM_STRIP_ROUNDS; r++) {
        const unsigned line = (unsigned)r * 32u + tid / 8u;
        const unsigned row = line / (unsigned)A.SC, col = line % (unsigned)A.SC;
        const unsigned cc = row / (unsigned)A.SR, sr = row % (unsigned)A.SR;
        relc[r] = (cc * (unsigned)A.in_rows + sr) * (unsigned)A.W + col;
        rcol[r] = sr | (col << 8) | (line < lines ? 0x80000000u : 0u);
    }
    // this lane's words in a strip buffer: tap offset (LDS table) + its position's corner + its word
    const unsigned corner = ((wy * (unsigned)A.SC + wx) * (unsigned)A.stride) * 128u + (lane & 15u) * 8u;
    for (unsigned s = tid; s < (unsigned)KB * 64; s += 256) toff_lds[s] = A.tapoff[s];
    const u64d *inp = inw + (tid % 8u) * 2u;

    // the 16-byte pieces of tile tau's strip, zeros outside the image (and outside the rows the caller handed over)
    auto fetch = [&](unsigned tau, v4i (&sreg)[MM_STRIP_ROUNDS]) {
        const int ty = (int)(tau / (unsigned)A.spr), tx = (int)(tau % (unsigned)A.spr);
        const int iy0 = (A.out_row0 + ty * TY) * A.stride - A.pad, ix0 = tx * TX * A.stride - A.pad;
        const int origin = (iy0 - A.in_row0) * A.W + ix0;  // in ciphertexts; never negative for a pixel inside the strip
#pragma unroll
        for (int r = 0; r < MM_STRIP_ROUNDS; r++) {
            const int iy = iy0 + (int)(rcol[r] & 0xffu), ix = ix0 + (int)((rcol[r] >> 8) & 0xffffu);
            const bool ok = (rcol[r] >> 31) && (unsigned)iy < (unsigned)A.H && (unsigned)ix < (unsigned)A.W &&
                            (unsigned)(iy - A.in_row0) < (unsigned)A.in_rows;
            sreg[r] = ok ? *(const v4i *)(inp + (size_t)(unsigned)(origin + (int)relc[r]) * ctw) : v4i{0, 0, 0, 0};
        }
    };
    auto stash = [&](int buf, const v4i (&sreg)[MM_STRIP_ROUNDS]) {
#pragma unroll
        for (int r = 0; r < MM_STRIP_ROUNDS; r++) strip[buf][r * 256 + tid] = sreg[r];  // line r*32 + tid/8, part tid%8
    };

    for (unsigned mg = 0; mg < (unsigned)A.Mg; mg++) {
        __syncthreads();  // readers of the previous channel group's fragments and strips are done
#pragma unroll
        for (int kb = 0; kb < KB; kb++) {
            const v4i *asrc = A.afrag + (((size_t)i * KB + kb) * A.Mg + mg) * MM_FRAG;
            for (unsigned e = tid; e < MM_FRAG; e += 256) a_lds[kb * MM_FRAG + e] = asrc[e];
        }
        if (tid < MM_CH) ws_lds[tid] = A.wsum[((size_t)i * A.Mg + mg) * MM_CH + tid];
        {
            v4i sreg[MM_STRIP_ROUNDS];
            fetch(tau0, sreg);
            stash(0, sreg);
        }
        __syncthreads();
        const int m0 = (int)(mg * MM_CH + 4 * g);
        u64d *outm = A.out + (size_t)m0 * mstride + (size_t)lc * N + wb * 16 + (lane & 15u);

        for (unsigned tau = tau0; tau < tau1; tau++) {
            const int buf = (int)((tau - tau0) & 1u);
            const char *sb = (const char *)strip[buf];
            v4i acc[2 * MM_DIG - 1][MM_MB];
#pragma unroll
            for (int kb = 0; kb < KB; kb++) {
                const bool quad = QUAD && kb == KB - 1;  // folds: kb is an unrolled constant
                u64d x[16];
#pragma unroll
                for (int t = 0; t < 16; t++) x[t] = *(const u64d *)(sb + (toff_lds[kb * 64 + 16 * g + t] + corner));
                v4i bf[8];
                if (quad) mm_b_fragments<false, true>(x, 0xffffu, shift_bits, bf); else mm_b_fragments<false, false>(x, 0xffffu, 0u, bf);
                const v4i *a = a_lds + kb * MM_FRAG;
                if (kb == 0) {
                    if (quad) mm_step<true, true>(a, lane, bf, acc); else mm_step<true, false>(a, lane, bf, acc);
                } else {
                    if (quad) mm_step<false, true>(a, lane, bf, acc); else mm_step<false, false>(a, lane, bf, acc);
                }
            }
            // the next tile's strip is requested once the matrix work is issued: its registers are live only through the
            // recombination, whose latency covers the loads
            v4i sreg[MM_STRIP_ROUNDS];
            if (tau + 1 < tau1) fetch(tau + 1, sreg);
            const int oyl = (int)(tau / (unsigned)A.spr) * TY + (int)wy, ox = (int)(tau % (unsigned)A.spr) * TX + (int)wx;
            const bool real = oyl < A.out_rows && ox < A.Wo;
            double ws[MM_MB][4];
#pragma unroll
            for (int mb = 0; mb < MM_MB; mb++)
#pragma unroll
                for (int r = 0; r < 4; r++) ws[mb][r] = ws_lds[mb * 16 + 4 * g + r];
            if (real)  // uniform for the wave: one without a position stores nothing
                mm_recombine_store(acc, A.modc[i], A.pow24[i], ws, outm + ((size_t)oyl * A.Wo + ox) * ctw, mstride, mg, g, A.O);
            if (tau + 1 < tau1) stash(buf ^ 1, sreg);
            __syncthreads();
        }
    }
}

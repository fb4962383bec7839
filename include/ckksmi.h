/*
 * ckksmi.h -- C ABI of the MI355X-native RNS-CKKS ciphertext-arithmetic library.
 *
 * What it is for: the cloud side of encrypted CNN inference as the paper poses it
 * (abstract, section 1): the client encodes and encrypts, the server evaluates
 * convolution / polynomial-activation / fully-connected layers on ciphertexts,
 * the client decrypts.  The scheme is CKKS (paper section 2.1), used as a leveled
 * scheme without bootstrapping (section 2.1, first paragraph), in its RNS form.
 *
 * Conventions
 *   - Plain C, every function returns int: 0 = CKKSMI_OK, negative = error code
 *     below.  Nothing throws across the boundary.  Arguments are validated on the
 *     host before anything is enqueued; a failed call enqueues nothing.
 *   - Ring R = Z[X]/(X^N+1), N = 2^logN.  Moduli: ciphertext primes q_0..q_{n_q-1}
 *     then special primes p_0..p_{k-1}; "modulus index" t runs over that list.
 *     Every prime is < 2^51 and = 1 mod 2N.
 *   - word  = one residue, uint64_t, canonical representative in [0, modulus).
 *     limb  = N words.  A polynomial at `level` l is [l][N] (limb i mod q_i).
 *     A ciphertext is [2][l][N]; a degree-2 ciphertext (tensor output) [3][l][N];
 *     a batch is a dense array of those, batch index outermost.
 *   - Unless stated otherwise polynomials are in EVALUATION form: word j of limb i
 *     is the polynomial evaluated at psi_i^(2*brev(j)+1) mod q_i, brev = logN-bit
 *     reversal, psi_i the primitive 2N-th root reported by ckksmi_get_moduli.
 *   - Decryption convention of the paper (section 2.1): m ~ c0 + c1*s.
 *   - "host" pointers are ordinary memory; "device" pointers are HIP device
 *     memory on the context's GPU.  The library never allocates ciphertext or
 *     workspace memory: the caller passes device buffers and a hipStream_t (as
 *     void*; NULL = the default stream).  Device calls enqueue on that stream and
 *     return without synchronising (one exception: ckksmi_encode_device reads an overflow word back and therefore
 *     waits for its stream).  The context owns only its constant tables.
 *     Device buffers (ciphertexts, keys, workspace) must be 16-byte aligned: the
 *     kernels move two words per lane and memory instruction; a misaligned
 *     pointer is rejected with CKKSMI_EINVAL.
 *   - Scale is caller-side metadata; level and batch are explicit arguments.
 *   - A context created with device = -1 is host-only: the host functions work,
 *     every device function returns CKKSMI_EDEVICE.  There is no CPU fallback for
 *     the device functions.
 */
#ifndef CKKSMI_H
#define CKKSMI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CKKSMI_OK 0
#define CKKSMI_EINVAL (-1)       /* null pointer, bad shape or parameter */
#define CKKSMI_ELEVEL (-2)       /* level out of range for the operation */
#define CKKSMI_ENOKEY (-3)       /* no Galois key registered for that rotation */
#define CKKSMI_EWORKSPACE (-4)   /* workspace too small for even one item */
#define CKKSMI_EDEVICE (-5)      /* HIP error (see ckksmi_last_device_error) or host-only context */
#define CKKSMI_EUNSUPPORTED (-6) /* valid request this build does not implement */

typedef struct ckksmi_ctx ckksmi_ctx;

typedef struct {
    int logN;         /* 2 .. 17 */
    int n_q;          /* number of ciphertext primes (fresh level), 1 .. 62 */
    int q_bits;       /* 2^(q_bits-1) < q_i < 2^q_bits, q_bits <= 51 */
    int n_special;    /* k, 0 .. 4; 0 disables key switching */
    int special_bits; /* <= 51 */
    int alpha;        /* ciphertext primes per key-switch digit, 1 .. 4 and <= max(k,1) */
    const uint64_t *moduli_override; /* optional: n_q + k primes to use instead of the search rule */
    const uint64_t *psi_override;    /* optional with moduli_override: their 2N-th roots */
    int device;       /* HIP device ordinal, or -1 for a host-only context */
} ckksmi_params;

/* operations for ckksmi_workspace_bytes */
#define CKKSMI_OP_RELIN 1
#define CKKSMI_OP_RESCALE 2
#define CKKSMI_OP_HMUL_RELIN_RESCALE 3
#define CKKSMI_OP_ROTATE 4
#define CKKSMI_OP_CONV2D_MAC 5 /* `batch` = number of weights O*C*kh*kw (or O*F) */
#define CKKSMI_OP_MUL_SCALAR_RESCALE 6

/* ------------------------------------------------------------------ context */
/* Primes: the n_q largest q_bits-bit primes = 1 mod 2N in descending order, then
 * the k largest special_bits-bit ones (skipping any already taken); psi_t = x^((p-1)/2N)
 * for the first x = 2,3,.. whose power has order exactly 2N. */
int ckksmi_ctx_create(const ckksmi_params *params, ckksmi_ctx **out);
void ckksmi_ctx_destroy(ckksmi_ctx *ctx);
/* moduli, psi: host arrays of n_q + k words (either may be NULL) */
int ckksmi_get_moduli(const ckksmi_ctx *ctx, uint64_t *moduli, uint64_t *psi);
const char *ckksmi_strerror(int code);
/* last hipError_t seen by this context (0 = none) */
int ckksmi_last_device_error(const ckksmi_ctx *ctx);

/* ------------------------------------------------------------------ host side
 * All pointers are host pointers.  Randomness is an input: the samplers below
 * draw it from a seed, keygen/encrypt consume explicit polynomials, so that the
 * same draws can be given to any other implementation.  Paper section 2.1. */

/* i.i.d. uniform {-1,0,1} */
int ckksmi_sample_ternary(const ckksmi_ctx *ctx, uint64_t seed, int64_t *out /*[N]*/);
/* round(N(0, 3.2^2)) redrawn while |e| > 19 */
int ckksmi_sample_error(const ckksmi_ctx *ctx, uint64_t seed, int64_t *out /*[N]*/);
/* limb x uniform on [0, modulus[index[x]]) */
int ckksmi_sample_uniform(const ckksmi_ctx *ctx, uint64_t seed, const int *index, int n_limbs, uint64_t *out /*[n_limbs][N]*/);

/* m = round(scale * phi^-1(z)), z_k = re[k] + i*im[k] (im may be NULL) for the
 * N/2 slots, slot k evaluated at zeta^(5^k), zeta = exp(i*pi/N); written as a
 * plaintext at `level` in evaluation form. */
int ckksmi_encode(const ckksmi_ctx *ctx, const double *re, const double *im, double scale, int level, uint64_t *pt /*[level][N]*/);
/* inverse of the above on a decrypted polynomial (evaluation form): CRT to the
 * centred representative, then z_k = m(zeta^(5^k)) / scale. */
int ckksmi_decode(const ckksmi_ctx *ctx, const uint64_t *pt /*[level][N]*/, int level, double scale, double *re /*[N/2]*/, double *im /*[N/2] or NULL*/);

/* pk = (b = -a*s + e, a) over q_0..q_{n_q-1}; a in evaluation form. */
int ckksmi_keygen_public(const ckksmi_ctx *ctx, const int64_t *s /*[N]*/, const uint64_t *a /*[n_q][N]*/, const int64_t *e /*[N]*/, uint64_t *pk /*[2][n_q][N]*/);
/* Switching keys, layout [beta][2][n_q+k][N], beta = ceil(n_q/alpha):
 *   key[j][1][t] = a[j][t]
 *   key[j][0][t] = -a[j][t]*s + e[j] + [t = q_i, i in digit j]*(P mod q_i)*s'
 * digit j = {j*alpha .. min(n_q,(j+1)*alpha)-1}, P = product of special primes.
 * relin: s' = s^2.  galois: s' = s(X^g), g = 5^rot mod 2N (left rotation by rot slots). */
int ckksmi_keygen_relin(const ckksmi_ctx *ctx, const int64_t *s, const uint64_t *a /*[beta][n_q+k][N]*/, const int64_t *e /*[beta][N]*/, uint64_t *evk);
int ckksmi_keygen_galois(const ckksmi_ctx *ctx, const int64_t *s, int rot, const uint64_t *a, const int64_t *e, uint64_t *gk);
/* ct = (r*b + e0 + m, r*a + e1) on the first `level` limbs */
int ckksmi_encrypt(const ckksmi_ctx *ctx, const uint64_t *pk, const uint64_t *pt /*[level][N]*/, const int64_t *r, const int64_t *e0, const int64_t *e1, int level, uint64_t *ct /*[2][level][N]*/);
/* pt = c0 + c1*s (+ c2*s^2 when n_comp = 3), evaluation form */
int ckksmi_decrypt(const ckksmi_ctx *ctx, const int64_t *s, const uint64_t *ct, int level, int n_comp, uint64_t *pt /*[level][N]*/);

/* ------------------------------------------------------------------ device side
 * All data pointers are device pointers unless marked host.  `batch` = number of
 * ciphertexts.  In-place use (out == input) is allowed where noted. */

/* Remember the device address of the Galois key for left rotation by `rot` slots
 * (the key memory stays the caller's and must outlive its use). */
int ckksmi_galois_key_register(ckksmi_ctx *ctx, int rot, const uint64_t *gk_dev);

/* Forward / inverse negacyclic transform of n_limbs*batch limbs laid out
 * [batch][n_limbs][N]; limb x uses modulus index index[x] (host array).  In place.
 * forward: coefficient (natural) order -> evaluation order; inverse includes 1/N. */
int ckksmi_ntt(ckksmi_ctx *ctx, uint64_t *limbs, const int *index, int n_limbs, int batch, void *stream);
int ckksmi_intt(ckksmi_ctx *ctx, uint64_t *limbs, const int *index, int n_limbs, int batch, void *stream);

/* limb-wise ciphertext operations (paper section 2.1: addition of ciphertexts);
 * out may alias an input */
int ckksmi_add(ckksmi_ctx *ctx, const uint64_t *a, const uint64_t *b, uint64_t *out, int level, int batch, void *stream);
int ckksmi_sub(ckksmi_ctx *ctx, const uint64_t *a, const uint64_t *b, uint64_t *out, int level, int batch, void *stream);
/* both components times a plaintext [level][N]; pt_stride = words between the
 * plaintexts of consecutive items, 0 = one plaintext for the whole batch */
int ckksmi_mul_plain(ckksmi_ctx *ctx, const uint64_t *a, const uint64_t *pt, size_t pt_stride, uint64_t *out, int level, int batch, void *stream);
/* Sums of plaintext x ciphertext products, the inner sums of a matrix-vector product in the rotation-packed
 * (single-image) layout, where section 2.1's plaintext multiplications and additions come in hundreds per layer:
 *     out[g] = sum over the ciphertexts s with term[g][s] >= 0 of  pts[term[g][s]] (*) cts[s]
 * (slot-wise, both components, mod every q_i: the same words as ckksmi_mul_plain and ckksmi_add term by term).
 * cts: device [n_ct][2][level][N]; pts: device [n_pts][level][N], evaluation form; term: device int32
 * [n_groups][n_ct], the plaintext that multiplies ciphertext s in sum g, negative = none; out: device
 * [n_groups][2][level][N], must not overlap cts (CKKSMI_EINVAL).  The table lives on the device (a plan uploads it
 * once) and is not read by the host: an entry >= n_pts is treated as "none" by the kernel, it gives a wrong sum but
 * no access outside the buffers.  A sum without terms gives zeros. */
int ckksmi_plain_mac(ckksmi_ctx *ctx, const uint64_t *cts, int n_ct, const uint64_t *pts, int n_pts, const int32_t *term, int n_groups,
                     uint64_t *out, int level, void *stream);
/* every word times the signed constant c (reduced mod each q_i) */
int ckksmi_mul_scalar(ckksmi_ctx *ctx, const uint64_t *a, int64_t c, uint64_t *out, int level, int batch, void *stream);
/* add the constant polynomial c to component 0 (every slot += c/scale) */
int ckksmi_add_const(ckksmi_ctx *ctx, const uint64_t *a, int64_t c, uint64_t *out, int level, int batch, void *stream);
/* keep the first level_out limbs of each component; out must not alias a */
int ckksmi_mod_drop(ckksmi_ctx *ctx, const uint64_t *a, int level_in, int level_out, uint64_t *out, int batch, void *stream);

/* ct x ct tensor: d = (a0*b0, a0*b1 + a1*b0, a1*b1), [3][level][N] per item */
int ckksmi_hmul(ckksmi_ctx *ctx, const uint64_t *a, const uint64_t *b, uint64_t *d, int level, int batch, void *stream);
/* out = (d0 + ks0, d1 + ks1), ks = KeySwitch(d2) with evk (hybrid: ModUp per
 * digit, inner product with the key, ModDown = divide by P with rounding) */
int ckksmi_relin(ckksmi_ctx *ctx, const uint64_t *d, const uint64_t *evk, uint64_t *out, int level, int batch, void *ws, size_t ws_bytes, void *stream);
/* divide by q_{level-1} with rounding to nearest: level -> level-1.  out may alias a
 * only when batch == 1 */
int ckksmi_rescale(ckksmi_ctx *ctx, const uint64_t *a, uint64_t *out, int level, int batch, void *ws, size_t ws_bytes, void *stream);
/* ckksmi_rescale for callers that cannot allocate or hold a workspace (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same kernels and the same bits, with the intermediates (the dropped limb in
 * coefficient form and the converted limbs, (2 + 2*(level-1)) * N words per ciphertext) in a static device array of
 * CKKSMI_STATIC_SCRATCH_BYTES that every GPU the library runs on holds until the process ends.  The call allocates nothing
 * (no device or host memory, no events: it records no profiling data) and enqueues on `stream` like every device call.
 * a, out as ckksmi_rescale.  A batch whose intermediates exceed the array is swept in chunks; CKKSMI_EWORKSPACE if one
 * ciphertext's intermediates alone exceed it (e.g. N = 2^16 above level 64, N = 2^17 above level 32);
 * CKKSMI_EUNSUPPORTED on a device ordinal of 64 or more.  All calls on one GPU share the one array, whatever their context
 * or stream: calls that overlap in time on the same GPU race on it (calls on one stream are ordered and safe). */
#define CKKSMI_STATIC_SCRATCH_BYTES (64u << 20)
int ckksmi_rescale_static(ckksmi_ctx *ctx, const uint64_t *a, uint64_t *out, int level, int batch, void *stream);
/* Rescale(c * Drop(a -> level)) + addend, bit-identical to ckksmi_mod_drop, ckksmi_mul_scalar, ckksmi_rescale and
 * ckksmi_add in a row (the scalar steps of the polynomial activation schedules, section 2.2), without writing the
 * intermediate ciphertexts: the input is read at its own level level_in >= level (only its first `level` limbs are used),
 * the scalar rides in the constants of the dropped limb's inverse transform and in the last pass, which also adds the
 * addend.  a: [batch][2][level_in][N]; addend: NULL or [batch][2][level-1][N] (may be `out` itself);
 * out: [batch][2][level-1][N], must not alias a; workspace CKKSMI_OP_MUL_SCALAR_RESCALE (for `level`). */
int ckksmi_mul_scalar_rescale(ckksmi_ctx *ctx, const uint64_t *a, int64_t c, const uint64_t *addend, uint64_t *out, int level_in, int level, int batch, void *ws, size_t ws_bytes, void *stream);
/* the strict sequence hmul -> relin -> rescale, bit-identical to the three calls */
int ckksmi_hmul_relin_rescale(ckksmi_ctx *ctx, const uint64_t *a, const uint64_t *b, const uint64_t *evk, uint64_t *out /*[2][level-1][N]*/, int level, int batch, void *ws, size_t ws_bytes, void *stream);
/* Lazy relinearisation (a fewer-transform variant for sums of products; the paper fixes no order): item i holds `terms`
 * pairs, a, b: device [batch][terms][2][level][N]; the three-component tensors of the pairs are added limb-wise and
 * the sum is relinearised and rescaled ONCE, out_i = Rescale(Relin(sum_t Tensor(a_it, b_it))): one key switch instead of
 * `terms`.  Not the bits of adding separately relinearised products; terms = 1 is ckksmi_hmul_relin_rescale.
 * Workspace and errors as ckksmi_hmul_relin_rescale; CKKSMI_EINVAL for terms < 1. */
int ckksmi_hmul_sum_relin_rescale(ckksmi_ctx *ctx, const uint64_t *a, const uint64_t *b, int terms, const uint64_t *evk, uint64_t *out /*[batch][2][level-1][N]*/, int level, int batch, void *ws, size_t ws_bytes, void *stream);
/* The same product with ONE division instead of ModDown followed by rescale (a fewer-transform variant of the
 * multiplication of section 2.1; the paper fixes no order): the key-switch accumulators stay over the extended basis,
 * P*(d0, d1) joins them there, and both components are divided by P*q_{level-1} at once,
 *     out_c = DivRound_B(acc_c + P*d_c),  B = {q_{level-1}, p_0 .. p_{k-1}},
 * in the exact form of DivRound: the overshoot of the basis conversion, v = floor(sum_m y_m * (1/b_m)) evaluated in
 * double precision in the order of B (products and sums each rounded to nearest), is removed, so every coefficient is
 * floor((x + h)/(P*q_{level-1})) itself.  The result encrypts the same product at the same scale and level as
 * ckksmi_hmul_relin_rescale but differs from it by up to one unit per coefficient: the two are NOT bit-identical.
 * Arguments, layouts, workspace (CKKSMI_OP_HMUL_RELIN_RESCALE) and errors as ckksmi_hmul_relin_rescale; additionally
 * CKKSMI_EUNSUPPORTED when the context has more than 3 special primes. */
int ckksmi_hmul_relin_rescale_merged(ckksmi_ctx *ctx, const uint64_t *a, const uint64_t *b, const uint64_t *evk, uint64_t *out /*[2][level-1][N]*/, int level, int batch, void *ws, size_t ws_bytes, void *stream);
/* left rotation of item i by rot[i] slots (host array; each needs a registered
 * key): automorphism X -> X^g first, then key switch of the second component.
 * out must not overlap a (out == a is refused): several kernels of the call read the input. */
int ckksmi_rotate(ckksmi_ctx *ctx, const uint64_t *a, const int *rot /*host [batch]*/, uint64_t *out, int level, int batch, void *ws, size_t ws_bytes, void *stream);

/* Encoding and encryption on the device (section 2.1), for feeding many fresh ciphertexts without the host in the way.
 * ckksmi_encode_device: re, im: device doubles [batch][N/2] (im may be NULL: real slots); pt: device [batch][level][N],
 * evaluation form, m = round(scale * phi^-1(z)) computed with a double-precision complex inverse transform: coefficients
 * may differ from ckksmi_encode (long double) by a unit in the last place.  ws: device, batch*N*16 bytes.  Synchronises
 * the stream before returning (a coefficient of 2^62 or more is reported as CKKSMI_EINVAL).
 * ckksmi_encrypt_device: ct = (r*b + e0 + m, r*a + e1) exactly as ckksmi_encrypt; pk: device [2][n_q][N]; pt: device
 * [batch][level][N]; r, e0, e1: device int64 [batch][N] (the caller draws them: ternary r, small errors; magnitudes
 * below 2^51); ct: device [batch][2][level][N], must not overlap pt; ws: device, 3*level*N*8 bytes per item (a smaller
 * one makes several sweeps). */
/* Small polynomials drawn on the device (the randomness of encryption and key generation, section 2.1; the paper names
 * no distribution: ternary and rounded Gaussian are the usual ones).  Counter-based (Philox4x32-10, one block per
 * coefficient: counter (t, kind, polynomial index), key = seed), so polynomial p = first_index + row is the same
 * whenever and wherever it is drawn.  kind CKKSMI_SAMPLE_TERNARY: uniform on {-1, 0, 1}; CKKSMI_SAMPLE_GAUSSIAN:
 * round(N(0, sigma^2)) by comparison of 64 random bits with the cumulative thresholds floor(2^64 * erf((k + 1/2)/(sigma sqrt 2))),
 * k < 40, 0 < sigma < 64.  out: device int64 [rows][N], 8-byte aligned. */
#define CKKSMI_SAMPLE_TERNARY 0
#define CKKSMI_SAMPLE_GAUSSIAN 1
int ckksmi_sample_device(ckksmi_ctx *ctx, int kind, double sigma, uint64_t seed, uint64_t first_index, int rows, int64_t *out, void *stream);
int ckksmi_encode_device(ckksmi_ctx *ctx, const double *re, const double *im, double scale, int level, int batch, uint64_t *pt, void *ws, size_t ws_bytes, void *stream);
int ckksmi_encrypt_device(ckksmi_ctx *ctx, const uint64_t *pk, const uint64_t *pt, const int64_t *r, const int64_t *e0, const int64_t *e1, int level, int batch, uint64_t *ct, void *ws, size_t ws_bytes, void *stream);

/* n_rot rotations of EVERY item with one shared ModUp ("hoisting"; a fewer-transform variant of the rotation above, the
 * paper fixes no algorithm): the second component is decomposed and lifted to the extended basis once per item,
 * dt_j = NTT(ModUp_j(INTT(c1))), and rotation r applies its automorphism to the lifted digits before the inner product
 * with its key: acc_c = sum_j sigma_r(dt_j) * gk_r[j][c], ks = DivRound_P(acc), out = (sigma_r(c0) + ks0, ks1).
 * Decrypts like ckksmi_rotate's result but is NOT bit-identical to it (sigma(ModUp(d)) and ModUp(sigma(d)) are
 * different lifts of the same polynomial).  rot: host array of n_rot offsets (1 <= n_rot <= 64), each with a
 * registered key, CKKSMI_ENOKEY otherwise; out: device [batch][n_rot][2][level][N], must not alias a;
 * ws: device workspace of ckksmi_rotate_hoisted_workspace_bytes(level, batch, n_rot) bytes (a smaller one makes
 * several sweeps; CKKSMI_EWORKSPACE if not even one item fits). */
int ckksmi_rotate_hoisted(ckksmi_ctx *ctx, const uint64_t *a, const int *rot /*host [n_rot]*/, int n_rot, uint64_t *out, int level, int batch, void *ws, size_t ws_bytes, void *stream);
int ckksmi_rotate_hoisted_workspace_bytes(const ckksmi_ctx *ctx, int level, int batch, int n_rot, size_t *bytes);

/* Convolution / fully-connected layers of the paper's network (Table 1) over
 * per-pixel ciphertexts (slot s = image s), integer plaintext weights (device,
 * int64): out[o,y,x] = sum_{c,u,v} w[o,c,u,v] * in[c, y*stride+u-pad, x*stride+v-pad],
 * taps outside the image skipped; out at the same level (rescale separately).
 * in: [C][H][W] ciphertexts, out: [O][Ho][Wo], Ho = (H+2*pad-kh)/stride+1. */
int ckksmi_conv2d_mac(ckksmi_ctx *ctx, const uint64_t *in, const int64_t *w, int C, int H, int W, int O, int kh, int kw, int stride, int pad, uint64_t *out, int level, void *ws, size_t ws_bytes, void *stream);
/* Workspace for ckksmi_conv2d_mac / _rows / ckksmi_fc_mac (FC: C = F, kh = kw = 1) of this layer shape.  With at
 * least this much the multiply-accumulate runs on the matrix cores where the shape allows (ring degree >= 64, at
 * least 8 output channels, at most 16321 taps); with only ckksmi_workspace_bytes(CKKSMI_OP_CONV2D_MAC, ...) it runs
 * on the vector ALU.  Both produce the same words. */
int ckksmi_conv2d_workspace_bytes(const ckksmi_ctx *ctx, int C, int O, int kh, int kw, int level, size_t *bytes);
/* The same convolution restricted to output rows out_row0 .. out_row0+out_rows-1, for layers whose activations do
 * not fit in device memory at once: `in` holds only image rows in_row0 .. in_row0+in_rows-1 as [C][in_rows][W]
 * ciphertexts and `out` receives [O][out_rows][Wo].  H is still the height of the whole image (it decides where
 * the zero padding starts).  CKKSMI_EINVAL if a tap of the requested rows falls on an image row outside the strip. */
int ckksmi_conv2d_mac_rows(ckksmi_ctx *ctx, const uint64_t *in, const int64_t *w, int C, int H, int W, int O, int kh, int kw, int stride, int pad, int in_row0, int in_rows, int out_row0, int out_rows, uint64_t *out, int level, void *ws, size_t ws_bytes, void *stream);
/* in: [F] ciphertexts, w: [O][F], out: [O] ciphertexts */
int ckksmi_fc_mac(ckksmi_ctx *ctx, const uint64_t *in, const int64_t *w, int F, int O, uint64_t *out, int level, void *ws, size_t ws_bytes, void *stream);
/* Pooling layers of the paper's network (Table 1: zero padding and 2x2 average pooling) as a sum of ciphertexts over
 * windows of the image padded with `pad` zero rows / columns on every side (0 <= pad < k):
 * out[c,y,x] = sum_{u,v<k} in[c, k*y+u-pad, k*x+v-pad], positions outside the image contribute nothing; the 1/k^2 of
 * the average is left to the caller, who folds it into the next layer's plaintext weights.  in: [C][H][W]
 * ciphertexts, out: [C][(H+2*pad)/k][(W+2*pad)/k] at the same level; rows and columns beyond the last full window are
 * ignored; 1 <= k <= 16. */
int ckksmi_sum_pool2d(ckksmi_ctx *ctx, const uint64_t *in, int C, int H, int W, int k, int pad, uint64_t *out, int level, void *stream);

/* bytes of workspace that lets `op` process the whole batch in one sweep; with
 * less (but at least one item's worth, else CKKSMI_EWORKSPACE) the call splits
 * the batch into several sweeps. */
int ckksmi_workspace_bytes(const ckksmi_ctx *ctx, int op, int level, int batch, size_t *bytes);

#ifdef __cplusplus
}
#endif
#endif

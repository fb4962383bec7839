/*
 * ckksmi_profile.h -- measurement and tuning hooks of the ckksmi library.
 *
 * Not part of the method: these calls describe this build's kernels (per-kernel
 * timing for roofline reports) and one launch-shape knob used by benchmarks and
 * tests.  Same conventions as ckksmi.h (plain C, int return codes).
 */
#ifndef CKKSMI_PROFILE_H
#define CKKSMI_PROFILE_H

#include "ckksmi.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-kernel timing for roofline reports: while enabled, every kernel launch is
 * bracketed by two HIP events recorded on the launch stream.  ckksmi_profile_enable
 * also discards what was recorded so far.  ckksmi_profile_read waits for the recorded
 * events of one kernel class and returns their summed duration, the number of
 * launches and the summed units of work (limbs for the transforms and limb-wise
 * kernels).  Not thread-safe; meant for benchmarks. */
#define CKKSMI_K_NTT_FWD_COL 0 /* forward transform, strided first pass */
#define CKKSMI_K_NTT_FWD_ROW 1 /* forward transform, contiguous pass */
#define CKKSMI_K_NTT_INV_ROW 2
#define CKKSMI_K_NTT_INV_COL 3
#define CKKSMI_K_TENSOR 4
#define CKKSMI_K_MODUP 5
#define CKKSMI_K_INNER 6
#define CKKSMI_K_DIVCONV 7
#define CKKSMI_K_DIVFINAL 8
#define CKKSMI_K_AUTOMORPH 9
#define CKKSMI_K_MACPREP 10
#define CKKSMI_K_MAC 11
#define CKKSMI_K_ELEMWISE 12
#define CKKSMI_K_CONV_COLS_MODUP 13 /* ModUp fused into the strided pass of the forward transform */
#define CKKSMI_K_CONV_COLS_DIV 14   /* DivRound conversion fused likewise */
#define CKKSMI_K_ROWS_INNER 15      /* contiguous pass fused with the inner product */
#define CKKSMI_K_ROWS_FINAL 16      /* contiguous pass fused with DivRound's last step */
#define CKKSMI_K_CONV_COLS_RESCALE 17 /* the same with a single dropped prime (rescale) */
#define CKKSMI_K_MAC_MFMA 18      /* conv / FC multiply-accumulate on the matrix cores */
#define CKKSMI_K_MACPREP_MFMA 19  /* its weight digits and tap table */
#define CKKSMI_K_NTT_LDS 20       /* whole limb transform inside one workgroup's LDS */
#define CKKSMI_K_TENSOR_ROWS 21   /* tensor product fused with the inverse contiguous pass of its third component */
#define CKKSMI_K_AXPY_LIMB 22     /* one limb of every row += constant * another limb (merged division: P*d on the dropped q) */
#define CKKSMI_K_CONV_COLS_MERGED 23 /* the conversion kernel in the exact form of DivRound, sources {q_last, special primes} */
#define CKKSMI_K_INNER_HOISTED 24 /* inner product of hoisted rotations (gathers the lifted digits through each automorphism) */
#define CKKSMI_K_AUTOMORPH_BCAST 25 /* first component of every item through every rotation's automorphism */
#define CKKSMI_K_ENCODE 26          /* device-side encoding: scatter, complex inverse transform, rounding */
#define CKKSMI_K_ENCRYPT 27         /* device-side encryption: residues of the small polynomials, combination with the key */
#define CKKSMI_K_CONV_COLS_TAIL 28  /* ModDown followed by rescale as one conversion (the strict sequence's bits) */
#define CKKSMI_K_MAC_MFMA_RES 29    /* the same for layers of few taps: weight digits resident in LDS, several positions per workgroup */
#define CKKSMI_K_MAC_MFMA_STRIP 30  /* ... and a narrow window: four neighbouring positions share a strip of the image staged in LDS */
#define CKKSMI_K_COUNT 31
int ckksmi_profile_enable(ckksmi_ctx *ctx, int on);
int ckksmi_profile_read(ckksmi_ctx *ctx, int kernel_class, double *total_ms, long long *launches, double *units);
/* name of the kernel that class runs as in this context (the transforms have size-specific kernels) */
const char *ckksmi_kernel_class_name(const ckksmi_ctx *ctx, int kernel_class);


/* Launch-shape knobs (benchmarks and tests; the defaults suit a full GPU).
 * CKKSMI_TUNE_TARGET_WGS: number of workgroups a transform launch aims for before its workgroups start looping over
 * the items of the batch (default 8192; a small value makes even a small batch exercise the item loops).  The
 * matrix-core multiply-accumulate aims for half of it before a workgroup walks several output positions. */
#define CKKSMI_TUNE_TARGET_WGS 0
int ckksmi_tune(ckksmi_ctx *ctx, int knob, int value);

#ifdef __cplusplus
}
#endif
#endif

/*
 * qrm_diag.h - diagnostic entry points of libqrm, for benchmarks and tests only.
 *
 * Nothing here is part of the detection path (Section 4.3 of the paper); a production caller needs
 * include/qrm.h alone.  The calls exist so that measurements and tests can be made through the same
 * C ABI as everything else, without environment variables read inside the hot path.
 */
#ifndef QRM_DIAG_H
#define QRM_DIAG_H

#include "qrm.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Flags of qrm_diag_set_flags; none of them changes what a call computes. */
#define QRM_DIAG_NO_FUSED_PAIRS 1   /* run every convolution block as a launch of its own (A/B timing; the two
                                       schedules round differently, both within the tolerance) */
#define QRM_DIAG_POISON_WORKSPACE 2 /* fill every newly allocated workspace with 0xFF bytes (NaN as bf16 and as
                                       fp32): a kernel that reads workspace bytes no kernel wrote shows in the
                                       results; bits 8..15 of the flags, when not zero, give another fill byte */

#define QRM_DIAG_FUSE_ALWAYS 4      /* run the fused schedule on wide tiles (more than 64 columns) also when a launch
                                       has too few images to fill the compute units that way (tests of that path on
                                       small batches) */

/* Sets the context's diagnostic flags (0 = production behaviour).  Affects calls made afterwards. */
QRM_API qrm_status qrm_diag_set_flags(qrm_ctx *ctx, int32_t flags);

/*
 * The rate the matrix pipes sustain when nothing else runs - eight wavefronts per compute unit issuing the bf16
 * 32x32x16 matrix instruction back to back for a few milliseconds - on operands of the given kind: data = 0
 * zeros, 1 one constant, 2 random (one side small normal values like weights, the other half zeros and half
 * positive like activations after a ReLU).  The part's clock follows its power budget and the power of a matrix
 * instruction follows its data, so the third figure, not the published peak, is what a convolution on real
 * activations can approach.  *tflops receives 10^12 FLOP/s.
 * Allocates and frees a small device buffer; synchronises the device's default stream.
 */
QRM_API qrm_status qrm_diag_matrix_rate(qrm_ctx *ctx, int32_t data, double *tflops);

#ifdef __cplusplus
}
#endif
#endif /* QRM_DIAG_H */

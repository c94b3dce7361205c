/*
 * fastforward_diag.h - tuning and measurement hooks of the block-sparse FFN
 * library.  Nothing here belongs to the method's statement (fastforward.h has
 * that); these calls exist so that a benchmark can time the stages of the path
 * on the library's own stream, force one kernel variant, and calibrate
 * hardware byte counters against a kernel of known traffic.
 */
#ifndef FASTFORWARD_DIAG_H
#define FASTFORWARD_DIAG_H

#include "fastforward.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Further names ff_set_option() takes.  All of them only choose between
 * kernels that compute the same sums (fp32 rounding order may differ):
 *   "gemm1_variant", "gemm2_variant"  -1 = choose by shape (default), else one
 *       tile shape of the gate/up or the down GEMM; an unknown number is an
 *       error.
 *   "gemm1_split"  -1 = decide by shape, 0 = never, 1 = always: whether the
 *       list positions beyond the last full tile of the gate/up GEMM (the
 *       compensator's units, typically) run as a second launch of small tiles
 *       (-1 never splits under a forced gemm1_variant).
 *   "gemm1_heavy_tiles"  -1 / 0 / 1 likewise: whether, in a split launch, the
 *       positions of a few much longer lists (first and last block dense)
 *       beyond the common length run as a launch of their own with small tiles
 *       instead of as tiles of the main launch.
 *   "gemm2_split"  -1 / 0 / 1 likewise: whether the last output-column tiles of
 *       the down GEMM run as a second launch of half-width tiles, which saves a
 *       mostly empty last round of workgroups.
 *   "gemm2_row_mode"  -1 = decide by shape, 1 = the down GEMM reads the ids of
 *       its gathered rows from a table of 16-bit ids in LDS, 2 = by scalar
 *       loads of the list, 3 = from a small LDS ring the list streams through
 *       (only the eight-wavefront tile has it).  A mode the chosen tile lacks,
 *       or that does not fit, makes the compute call fail with FF_ERR_DEVICE.
 *   "gemm2_ksplit"  -1 = decide by shape, 0 = never, n > 0 = at most n short
 *       pieces: whether the down GEMM cuts the few lists that are much longer
 *       than the rest (first and last block dense) along the list into a tile
 *       like everybody else's plus short tiles, and adds their fp32 partial
 *       sums in piece order in one more launch. */

/* Per-stage GPU timing with HIP events on the context's stream.
 * ff_profile_enable(ctx, n, mask) makes every later compute call bracket each
 * kernel stage whose bit is set in stage_mask (1 << FF_STAGE_*) with a pair of
 * events, for at most max_records stage launches (further ones go unrecorded);
 * max_records = 0 switches profiling off and frees the events.  This is the one
 * call besides ff_create that allocates.  ff_profile_read synchronises the
 * stream, adds up the recorded milliseconds and launch counts per stage into
 * the two host arrays of FF_N_STAGES entries, and clears the records. */
enum {
  FF_STAGE_POOL = 0,   /* Eq. 12: logits + pooling                  */
  FF_STAGE_MLP = 1,    /* Eq. 13: predictor MLP -> scores           */
  FF_STAGE_TOPK = 2,   /* Eq. 14: top-K select                      */
  FF_STAGE_GEMM1 = 3,  /* gathered gate/up GEMM + SiLU*up epilogue  */
  FF_STAGE_GEMM2 = 4,  /* gathered down GEMM + compensation         */
  FF_STAGE_GLUE = 5,   /* RMSNorm, residual add                     */
  FF_N_STAGES = 6
};
ff_status ff_profile_enable(ff_ctx *ctx, int32_t max_records, uint32_t stage_mask);
ff_status ff_profile_read(ff_ctx *ctx, double *ms_sum, int32_t *launches);

/* Device-to-device copy of `bytes` (a multiple of 16) with a plain kernel on the
 * context's stream; buffers must not overlap.  It is the kernel of known
 * traffic against which the HBM byte counters of a profile are calibrated. */
ff_status ff_copy(ff_ctx *ctx, void *dst, const void *src, size_t bytes);

/* Enqueues a register-only loop of bf16 matrix instructions (v_mfma_f32_32x32x16_bf16,
 * eight independent accumulators, two wavefronts per SIMD on every compute unit)
 * that runs `iters` rounds, and stores in *flops the floating-point operations one
 * such launch performs.  Timed by the caller (events on the context's stream), it
 * gives the rate the matrix pipes really sustain on this machine, to print beside
 * the published peak: with zero_operands != 0 on all-zero operands, else on
 * pseudo-random bf16 values (the clock the chip holds depends on the data). */
ff_status ff_mfma_peak(ff_ctx *ctx, int32_t iters, int32_t zero_operands, double *flops);

#ifdef __cplusplus
}
#endif
#endif /* FASTFORWARD_DIAG_H */

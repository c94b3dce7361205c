/*
 * fastforward.h - C ABI of the MI355X (gfx950) block-sparse FFN prefill library.
 *
 * The library runs, on one GPU, the inference-time path of block-wise
 * predictive FFN sparsity (Sec. 3.1-3.3 of the paper): for every block of
 * N_block prompt tokens a small predictor scores the d_ffn neurons (Eq. 12-13),
 * the K best are kept (Eq. 14), a gated FFN runs over the gathered weight rows
 * only (Eq. 15-18) and a low-rank compensation term is added (Eq. 20-21).  A
 * dense gated FFN (Eq. 10) is exported as the reference call, and a layer-stack
 * helper chains layers with RMSNorm and a residual add.
 *
 * Conventions that hold for every call
 * ------------------------------------
 *  - Pointers marked "dev" are device pointers on the context's GPU, owned by
 *    the caller, 16-byte aligned, and must stay valid until the context's
 *    stream has passed the call.  Pointers marked "host" are ordinary host
 *    memory, read before the call returns.
 *  - Matrices are row-major.  bf16 means the upper 16 bits of an IEEE float32.
 *  - Every hidden unit (FFN neuron or compensator unit) owns one contiguous row
 *    of d_model values in each of its matrices:
 *        w_gate, w_up, w_down : bf16 [d_ffn][d_model]   (W_down of Eq. 10 is
 *                               stored transposed: row j is what neuron j adds)
 *        wc1, wc2             : bf16 [r_comp][d_model]  (W_comp1 of Eq. 20 is
 *                               stored transposed)
 *    Predictor weights are stored as the paper writes them:
 *        w1 : bf16 [d_model][r_pred],  w2 : bf16 [r_pred][d_ffn]
 *  - Compute calls only enqueue work on the context's stream; they neither
 *    allocate, free nor synchronise (the one exception is stated at
 *    k_per_block below).  All scratch lives in the workspace the caller gives.
 *  - Every call returns FF_OK or an error code; after an error
 *    ff_last_error() holds a one-line description.  Argument errors are found
 *    on the host before anything is launched.  Nothing throws across the ABI.
 *  - A context is not thread-safe; use one per host thread and stream.
 *  - Selected-neuron lists are int32, ascending, one row of k_stride entries
 *    per block; entries past the block's K are -1.
 *  - The prompt is cut into blocks of `block` tokens (Sec. 3.1); if n_tokens
 *    is not a multiple the last block is short.  n_blocks = ceil(n_tokens /
 *    block).
 *  - k_per_block is a host array of n_blocks entries, each in [1, d_ffn].
 *    When all entries are equal the value travels as a kernel argument and the
 *    call enqueues kernels only (it may be captured in a HIP graph).  Unequal
 *    entries are staged through a small ring of pinned buffers owned by the
 *    context: the call waits on the host only if all ring slots are still in
 *    flight, and it returns FF_ERR_INVALID_ARG while its stream is capturing
 *    (a replay would read whatever the slot holds by then).  A call whose
 *    entries equal those staged last (ff_predict and ff_sparse_ffn of one
 *    step, the same budgets step after step) reuses that copy.
 */
#ifndef FASTFORWARD_H
#define FASTFORWARD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ff_ctx ff_ctx; /* opaque */

typedef enum {
  FF_OK = 0,
  FF_ERR_INVALID_ARG = 1, /* null pointer, bad enum value, non-positive size */
  FF_ERR_SHAPE = 2,       /* sizes the kernels cannot take (see ff_shape)    */
  FF_ERR_ALIGNMENT = 3,   /* a device pointer is not 16-byte aligned          */
  FF_ERR_INDEX = 4,       /* index list not ascending / out of range (only in
                             validate mode, see ff_set_option)                */
  FF_ERR_WORKSPACE = 5,   /* workspace missing or too small                   */
  FF_ERR_DEVICE = 6,      /* a HIP call failed                                */
  FF_ERR_UNIMPLEMENTED = 7
} ff_status;

/* Sizes of one layer's problem.
 * Limits: d_model a multiple of 128, d_ffn a multiple of 8, r_pred in
 * [1, 1024], r_comp a multiple of 8 in [0, 4096] (0 = no compensator),
 * block >= 1 (at most 4096 with softmax pooling), n_tokens >= 1, at most
 * 16384 blocks, n_tokens + block below 2^31.  Anything else returns
 * FF_ERR_SHAPE. */
typedef struct {
  int32_t d_model;
  int32_t d_ffn;
  int32_t n_tokens;
  int32_t block;
  int32_t r_pred;
  int32_t r_comp;
} ff_shape;

/* Expert-neuron predictor (Sec. 3.2, Eq. 12-13). */
typedef struct {
  const void *q_pred; /* dev bf16 [d_model], or NULL = mean pooling (Eq. 12 at q = 0) */
  const void *w1;     /* dev bf16 [d_model][r_pred] */
  const void *w2;     /* dev bf16 [r_pred][d_ffn]   */
} ff_predictor;

/* Gated FFN weights (Eq. 10 / Eq. 15-17), neuron-major. */
typedef struct {
  const void *w_gate; /* dev bf16 [d_ffn][d_model] */
  const void *w_up;   /* dev bf16 [d_ffn][d_model] */
  const void *w_down; /* dev bf16 [d_ffn][d_model] */
} ff_ffn_weights;

enum { FF_ACT_SILU = 0, FF_ACT_RELU = 1, FF_ACT_IDENTITY = 2 };
enum { FF_OUT_BF16 = 0, FF_OUT_F32 = 1 };

/* Error-compensation network (Sec. 3.3, Eq. 20), unit-major. */
typedef struct {
  const void *wc1; /* dev bf16 [r_comp][d_model] */
  const void *wc2; /* dev bf16 [r_comp][d_model] */
  int32_t act;     /* FF_ACT_*; the paper writes the FFN's own sigma: SiLU */
} ff_compensator;

/* ---- context ----------------------------------------------------------- */

/* Creates a context bound to GPU `device` and to `hip_stream` (a hipStream_t,
 * NULL = the default stream).  Allocates only the small pinned staging ring. */
ff_status ff_create(ff_ctx **out, int device, void *hip_stream);
ff_status ff_destroy(ff_ctx *ctx);
/* Rebinds the context to another stream of the same device. */
ff_status ff_set_stream(ff_ctx *ctx, void *hip_stream);
/* Name of a status; `status` is an ff_status value, any other number gives
 * "unknown status". */
const char *ff_status_str(int status);
const char *ff_last_error(const ff_ctx *ctx);

/* Bytes of device scratch the compute calls need for this shape when at most
 * k_max neurons are kept per block (activations H of Eq. 18, the predictor's
 * partial sums and scores of Eq. 12-13, for calls of at most 8
 * tokens the partial sums of the down projection, for blocks shorter than
 * 128 tokens the merged lists of neighbouring blocks, and at most 48 MiB of
 * fp32 partial sums for the rows of a few blocks whose lists are much longer
 * than the others', Sec. 3.4). */
ff_status ff_workspace_bytes(const ff_shape *shape, int32_t k_max, size_t *bytes);
/* Hands the context a caller-owned device buffer (256-byte aligned) to use as
 * scratch until it is replaced or the context is destroyed. */
ff_status ff_set_workspace(ff_ctx *ctx, void *dev_ptr, size_t bytes);

/* Options: "validate" (0/1, default 0): ff_sparse_ffn first checks on the GPU
 * that every index row is ascending, in range and -1 padded, synchronises,
 * and returns FF_ERR_INDEX instead of launching if not (while the stream is
 * capturing a HIP graph the call returns FF_ERR_INVALID_ARG).  "small_path" (0/1,
 * default 1): calls with at most 8 tokens in total (the generation-time
 * regime) use gather-GEMV kernels, which read every selected weight row once
 * at HBM speed, instead of the MFMA tiles; 0 forces the tiles.
 * "merge_blocks" (-1 = when it is expected to pay, the default; 0 = never;
 * 1 = whenever the shape allows): blocks of 16, 32 or 64 tokens leave most of
 * a 128-token tile idle; ff_sparse_ffn may instead run the union of the lists
 * of the 128 / block neighbouring blocks over all their tokens and write the
 * activations of (block, neuron) pairs that were not selected as zero - the
 * same sums, faster when the lists are long; a call of at most 8 tokens with
 * several lists reads their union once for all tokens the same way.  Names that only serve tuning
 * and measurement are listed in fastforward_diag.h. */
ff_status ff_set_option(ff_ctx *ctx, const char *name, int32_t value);

/* Neurons kept at a sparsity level: K = clamp(floor((1 - s) d_ffn + 1/2), 1,
 * d_ffn).  Pure host arithmetic. */
ff_status ff_k_from_sparsity(int32_t d_ffn, double sparsity, int32_t *k);

/* Layer-wise budget allocation (Sec. 3.4, Alg. 1): importance scores of
 * n_layers layers and a mean budget in (0, 1] -> keep fractions b_i <= 1.
 * Host arrays, pure host arithmetic. */
ff_status ff_layer_budgets(const double *importance, int32_t n_layers,
                           double budget, double *keep_fraction);

/* ---- compute ----------------------------------------------------------- */

/* predict: block hidden states -> selected neuron indices (Eq. 12-14).
 *   x            dev bf16 [n_tokens][d_model]
 *   k_per_block  host int32 [n_blocks]
 *   k_stride     row pitch of `indices`, >= max k
 *   indices      dev int32 [n_blocks][k_stride], out: ascending, tail = -1
 *   scores_opt   dev f64 [n_blocks][d_ffn] out, or NULL
 * Scores are computed in float64 without intermediate rounding; the K highest
 * are kept and equal scores go to the lower index (-0 and +0 are equal).
 * Scores are expected to be finite; if one is not, exactly K in-range indices
 * are still written, with NaN ranked by its bit pattern. */
ff_status ff_predict(ff_ctx *ctx, const ff_shape *shape, const void *x,
                     const ff_predictor *pred, const int32_t *k_per_block,
                     int32_t k_stride, int32_t *indices, double *scores_opt);

/* For callers that cannot allocate device memory or own a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The same computation and arguments as ff_predict, but its scratch
 * (pooling logits, the first predictor layer's partial sums, scores) lives in a fixed
 * 32 MiB array inside the library (FF_STATIC_SCRATCH_BYTES; every GPU the
 * library is loaded on holds one until the process ends) instead of the
 * workspace, which need not be set.  The call allocates and frees nothing.
 * A shape whose predictor scratch exceeds the array returns FF_ERR_WORKSPACE
 * (about 8 (n_blocks (d_ffn + ceil(d_model / 512) r_pred) + n_tokens) bytes
 * are needed: the Llama-3.1-8B layer with 64 blocks takes 7.6 MiB, the
 * Qwen2.5-7B layer with 128 blocks 19.5 MiB).  All calls on one GPU share that
 * GPU's array: calls that overlap in time on one GPU, from any context or
 * stream, race.  Nothing is kept in the array between calls. */
#define FF_STATIC_SCRATCH_BYTES (32u << 20)
ff_status ff_predict_static(ff_ctx *ctx, const ff_shape *shape, const void *x,
                            const ff_predictor *pred, const int32_t *k_per_block,
                            int32_t k_stride, int32_t *indices, double *scores_opt);

/* sparse_ffn: Y = W^down (SiLU(W^gate X) * (W^up X)) over each block's selected
 * neurons (Eq. 15-18), plus the compensation term if `comp` is not NULL
 * (Eq. 20-21).  Any valid ascending index list may be given, not only
 * predict's.  bf16 operands, fp32 accumulation; the activations H and the
 * compensator's hidden units are rounded to bf16 once.
 *   indices      dev int32 [n_blocks][k_stride]
 *   y            dev [n_tokens][d_model], bf16 or f32 by out_dtype */
ff_status ff_sparse_ffn(ff_ctx *ctx, const ff_shape *shape, const void *x,
                        const ff_ffn_weights *w, const ff_compensator *comp,
                        const int32_t *indices, const int32_t *k_per_block,
                        int32_t k_stride, void *y, int32_t out_dtype);

/* dense_ffn: Eq. 10 with all d_ffn neurons, no predictor, no compensator.
 * shape->block, r_pred, r_comp are ignored.  A workspace of
 * ff_workspace_bytes(shape, d_ffn) is enough (H is d_ffn wide here). */
ff_status ff_dense_ffn(ff_ctx *ctx, const ff_shape *shape, const void *x,
                       const ff_ffn_weights *w, void *y, int32_t out_dtype);

/* ffn_stack: n_layers pre-norm residual layers around the sparse FFN path:
 *   x_l = bf16(RMSNorm(h, eps)) (gain 1);  idx = predict(x_l);
 *   y = bf16(sparse_ffn(x_l, idx) (+ compensation));  h = bf16(h + y)
 *   (the add happens in the down GEMM's epilogue; y is never stored).
 *   h                   dev bf16 [n_tokens][d_model], updated in place
 *   pred, w, comp       host arrays of n_layers structs (comp may be NULL)
 *   k_per_layer_block   host int32 [n_layers][n_blocks]
 *   indices_opt         dev int32 [n_layers][n_blocks][k_stride] out, or NULL
 *   x_dump_opt          dev bf16 [n_layers][n_tokens][d_model] out, or NULL:
 *                       each layer's normalised input, for layer-wise checks */
ff_status ff_ffn_stack(ff_ctx *ctx, const ff_shape *shape, int32_t n_layers,
                       void *h, const ff_predictor *pred,
                       const ff_ffn_weights *w, const ff_compensator *comp,
                       const int32_t *k_per_layer_block, int32_t k_stride,
                       float rms_eps, int32_t *indices_opt, void *x_dump_opt);

/* Stack glue, exported for tests: x = bf16(RMSNorm(h)), h = bf16(h + y). */
ff_status ff_rmsnorm(ff_ctx *ctx, int32_t n_tokens, int32_t d_model,
                     const void *h, float eps, void *x);
ff_status ff_residual_add(ff_ctx *ctx, int32_t n_tokens, int32_t d_model,
                          void *h, const void *y);

#ifdef __cplusplus
}
#endif
#endif /* FASTFORWARD_H */

// Internal declarations shared by the library's own translation units
// (kernel parameter blocks and host-side launchers).  Not part of the ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fastforward.h"
#include "fastforward_diag.h"

typedef uint16_t bf16_t;  // raw bf16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
  return __uint_as_float(((uint32_t)v) << 16);
}
// round-to-nearest-even, NaN stays NaN: the hardware's packed conversion (v_cvt_pk_bf16_f32), one instruction
// for two values
typedef __attribute__((ext_vector_type(2))) float ff_f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 ff_bf16x2_t;
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const ff_f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, ff_bf16x2_t));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  return (bf16_t)(pack_bf16x2(f, 0.0f) & 0xffffu);
}

// Per-block neuron count: either one value for all blocks or a device array.
constexpr int kMaxHeavy = 8;
struct KSpec {
  const int32_t *per_block;  // device, [n_blocks], or nullptr
  int32_t uniform;           // used when per_block == nullptr
  int32_t k_max;             // host-known maximum over blocks
  // Scheduling hints for lists of unequal length (host-known; never needed for correctness):
  // k_base = the most common K; heavy[0 .. n_heavy) = the blocks with K > k_base when there
  // are at most kMaxHeavy of them (the "first and last block dense" pattern), else n_heavy = 0
  // and k_base = k_max.
  int32_t k_base = 0;
  int32_t n_heavy = 0;
  int32_t heavy[kMaxHeavy] = {0, 0, 0, 0, 0, 0, 0, 0};
};

// Stage timing hooks: begin/end bracket a stage's launches with events when the
// stage is being profiled (prof may be nullptr).
struct Profiler {
  hipEvent_t *ev = nullptr;  // 2 * cap events
  int32_t *stage = nullptr;  // stage of each record
  int cap = 0, n = 0;
  uint32_t mask = 0;
  int open = -1;
};
inline void prof_begin(Profiler *pr, int stage, hipStream_t s) {
  if (!pr || !((pr->mask >> stage) & 1u) || pr->n >= pr->cap) return;
  pr->open = pr->n;
  pr->stage[pr->n] = stage;
  (void)hipEventRecord(pr->ev[2 * pr->n], s);
}
inline void prof_end(Profiler *pr, hipStream_t s) {
  if (!pr || pr->open < 0) return;
  (void)hipEventRecord(pr->ev[2 * pr->open + 1], s);
  pr->n = pr->open + 1;
  pr->open = -1;
}

// ---- predictor path (Eq. 12-14) -------------------------------------------
struct PredictParams {
  const bf16_t *x;       // [T][d_model]
  const bf16_t *q_pred;  // [d_model] or nullptr
  const bf16_t *w1;      // [d_model][r]
  const bf16_t *w2;      // [r][d_ffn]
  int32_t T, d_model, d_ffn, block, r, n_blocks;
  double *z;        // [T] pooling logits (softmax pooling only)
  double *hpart;    // [n_blocks][ceil(d_model / 512)][r]: the first layer's sums over slices of 512 channels
  double *scores;   // [n_blocks][d_ffn]
  KSpec k;
  int32_t k_stride;
  int32_t *indices;  // [n_blocks][k_stride]
};
hipError_t ff_launch_predict(const PredictParams &p, int lds_limit, hipStream_t s, Profiler *prof);

// ---- gathered GEMMs (Eq. 15-18, 20-21; Eq. 10 with idx == nullptr) ---------
struct Gemm1Params {
  const bf16_t *x;     // [T][d_model]
  const bf16_t *wg;    // [d_ffn][d_model]
  const bf16_t *wu;    // [d_ffn][d_model]
  const bf16_t *wc1;   // [rc][d_model] or nullptr
  const int32_t *idx;  // [n_blocks][k_stride], or nullptr: list position p is row p (dense) or nullptr (= all neurons in order)
  bf16_t *h;           // [T][hs]
  int32_t T, d_model, d_ffn, block, n_blocks, rc, comp_act, k_stride, hs;
  // Merged lists of short blocks: position p of block b belongs to the rows of its sub-block s
  // (sub tokens each) iff bit s of mask[b * k_stride + p] is set; elsewhere H is written as 0, so that
  // the down projection adds nothing for it.  nullptr = every position belongs to every row.
  const uint8_t *mask = nullptr;
  int32_t sub_shift = 0;   // log2 of the sub-block's token count
  // set by the launcher: full_only = this launch skips a block's last, part-filled N tile;
  // rem_bn != 0 = this launch covers exactly those parts: positions from the last multiple of
  // rem_bn below the block's list length
  int32_t full_only, rem_bn;
  int32_t rem_cap = 0x7fffffff;   // with rem_bn: the launch starts no later than this position (where the main launch stopped)
  int32_t skip_heavy = 0;         // this launch leaves out the blocks of k.heavy
  KSpec k;
};
struct Gemm2Params {
  const bf16_t *h;     // [T][hs]
  const bf16_t *wd;    // [d_ffn][d_model]
  const bf16_t *wc2;   // [rc][d_model] or nullptr
  const int32_t *idx;
  void *y;             // [T][d_model] bf16 or f32
  bf16_t *res;         // or nullptr.  Residual mode: res[t][:] = bf16(res[t][:] + bf16(Y[t][:])) in place, y unused
  int32_t T, d_model, d_ffn, block, n_blocks, rc, k_stride, hs, out_f32;
  int32_t col0 = 0;    // first output column of this launch (set by ff_launch_gemm2)
  // Lists much longer than the common length, cut along k (see ff_launch_gemm2).  The caller gives
  // room for fp32 partial sums (or nullptr: never cut); the launcher sets the rest: n_pieces per heavy
  // block (0 = not cut), the first piece = positions [0, cut0), the others piece_len positions each.
  float *part = nullptr;        // [n_heavy][n_pieces][block][d_model]
  size_t part_bytes = 0;
  int32_t n_pieces = 0, cut0 = 0, piece_len = 0;
  KSpec k;
};
// variant < 0: choose by shape.  Returns hipErrorInvalidValue for an unknown variant.
// split (gemm1): whether the positions beyond the last full N tile go to a second launch with
// small tiles: -1 = the launcher decides (never with a forced variant), 0 = never, 1 = whenever
// there are such positions.
// heavy_tiles: where the positions of a few much longer lists beyond the common length go when the launch is
// split: -1 = the launcher decides, 0 = tiles of the main launch, 1 = a launch of their own with 128 x 64 tiles.
hipError_t ff_launch_gemm1(const Gemm1Params &p, int variant, int split, int heavy_tiles, hipStream_t s);
// split (gemm2): whether the last output-column tiles of every block go to a second launch with
// half-width tiles when that saves a mostly empty last round of workgroups: -1 = the launcher decides
// (never with a forced variant or lists of unequal length), 0 = never, 1 = whenever there are two
// column tiles or more.
// ksplit: whether lists much longer than the common length ("first and last block dense") are cut along k
// into a tile like everybody else's plus short tiles that start at once on CUs of their own, all writing
// fp32 partial sums to p.part that one more launch adds in piece order: -1 = whenever there are such lists
// and p.part has room for at least two short pieces, 0 = never, n > 0 = into at most n short pieces.
// row_mode: where the kernel takes a gathered row's id from: -1 = the launcher decides, 1 = a table of
// 16-bit ids in LDS, 2 = scalar loads of the list, 3 = the list streamed through a small LDS ring (only
// the eight-wavefront tile has it).  A forced mode the tile does not have, or that does not fit, is an error.
hipError_t ff_launch_gemm2(const Gemm2Params &p, int variant, int split, int row_mode, int ksplit, hipStream_t s);
size_t ff_gemm2_part_bytes(int n_tokens, int block, int d_model);   // room that lets two heavy blocks be cut as finely as the launcher would
hipError_t ff_gemm_init(int lds_limit);  // raises the kernels' dynamic-LDS limits; once per process
int ff_gemm1_num_variants();
int ff_gemm2_num_variants();

// ---- few-token path (at most kGemvMaxTokens tokens in the whole call) ---------
constexpr int kGemvMaxTokens = 8;
constexpr int kGemvChunks = 256;   // most pieces the list is cut into for the down projection
struct GemvParams {
  const bf16_t *x, *wg, *wu, *wd, *wc1, *wc2;
  const int32_t *idx;  // [n_blocks][k_stride], or nullptr: list position p is row p (dense)
  bf16_t *h;           // [T][hs]
  float *part;         // [n_chunks][T][d_model]
  void *y;             // [T][d_model] bf16 or f32
  bf16_t *res;         // or nullptr: residual mode as in Gemm2Params
  int32_t T, d_model, d_ffn, block, n_blocks, rc, comp_act, k_stride, hs, out_f32;
  int32_t n_chunks, pos_per_wg;   // chosen by ff_launch_gemv
  // merged lists (as in Gemm1Params): position p belongs to token t iff bit (t - block start) / sub_block of
  // mask[b * k_stride + p] is set; nullptr = every position belongs to every token
  const uint8_t *mask = nullptr;
  int32_t sub_block = 1;
  KSpec k;
};
size_t ff_gemv_part_bytes(int n_tokens, int d_model);
bool ff_gemv_eligible(int n_tokens, int block, int d_model, int lds_limit);
hipError_t ff_launch_gemv(const GemvParams &p, int lds_limit, hipStream_t s, Profiler *prof);

// ---- glue -----------------------------------------------------------------
hipError_t ff_launch_rmsnorm(const bf16_t *h, bf16_t *x, int T, int d_model, float eps, hipStream_t s);
hipError_t ff_launch_residual(bf16_t *h, const bf16_t *y, size_t n, hipStream_t s);
hipError_t ff_launch_copy(void *dst, const void *src, size_t bytes, hipStream_t s);
// register-only MFMA loop over the whole chip; *flops = what one launch computes
hipError_t ff_launch_mfma_peak(int iters, int zero_operands, float *sink, double *flops, hipStream_t s);
// flag[0] is set to 1 + first bad block if some index row is not ascending, in
// range and -1 padded.  The caller zeroes flag[0] first.
// the lists of every g neighbouring blocks merged into one ascending list (u_idx, u_k) with a membership
// byte per entry (u_mask); d_ffn bytes of LDS
hipError_t ff_launch_merge_lists(const int32_t *idx, int k_stride, KSpec ks, int n_blocks, int g, int d_ffn,
                                 int32_t *u_idx, uint8_t *u_mask, int u_stride, int32_t *u_k, int lds_limit,
                                 hipStream_t s);
hipError_t ff_launch_validate(const int32_t *idx, int n_blocks, int k_stride, KSpec k,
                              int d_ffn, int32_t *flag, hipStream_t s);

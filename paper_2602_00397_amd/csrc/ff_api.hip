// C ABI of the library: argument checks, workspace carve-up, kernel sequencing.
// Every step of the path runs in the kernels of this library; nothing falls back
// to the host.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <cmath>
#include <new>

#include "ff_internal.h"

#include <vector>

// Scratch of ff_predict_static: a fixed array in device memory that every GPU the library runs on
// holds from the moment the code object is loaded until the process ends.  Host code never uses
// the array's name as an address: ff_create asks the runtime where the current device keeps its
// copy and the kernels get that pointer as an argument.
static __device__ __align__(256) unsigned char scratch[FF_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};   // address of `scratch` on each device, filled at ff_create

constexpr int kRing = 8;          // pinned staging slots for per-block K arrays
constexpr int kRingCap = 16384;   // int32 entries per slot = most blocks per call

struct Slot {
  int32_t *host = nullptr;
  int32_t *dev = nullptr;
  hipEvent_t ev = nullptr;
  bool used = false;
};

}  // namespace

struct ff_ctx {
  int device = 0;
  hipStream_t stream = nullptr;
  void *ws = nullptr;
  size_t ws_bytes = 0;
  void *static_scratch = nullptr;  // this device's copy of `scratch`
  int lds_limit = 65536;
  int validate = 0;
  int gemm1_variant = -1, gemm2_variant = -1, gemm1_split = -1, gemm2_split = -1, gemm2_row_mode = -1, gemm2_ksplit = -1, gemm1_heavy_tiles = -1;
  int small_path = 1;              // few-token calls take the GEMV kernels
  int merge_blocks = -1;           // lists of short blocks merged per 128 tokens: -1 = when it pays, 0 = never, 1 = whenever possible
  std::vector<int32_t> k_sorted;   // host scratch for the K statistics of a call
  Slot ring[kRing];
  int ring_next = 0;
  int staged_slot = -1, staged_n = 0;   // the slot staged last and its length: the same values again need no new copy
  int32_t *flag_dev = nullptr;
  int32_t *flag_host = nullptr;
  Profiler prof;
  char err[320] = {0};
};

namespace {

ff_status fail(ff_ctx *ctx, ff_status st, const char *fmt, ...) {
  if (ctx) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    va_end(ap);
  }
  return st;
}

#define FF_HIP(ctx, call)                                                                   \
  do {                                                                                      \
    hipError_t e_ = (call);                                                                 \
    if (e_ != hipSuccess) return fail(ctx, FF_ERR_DEVICE, "%s: %s", #call, hipGetErrorString(e_)); \
  } while (0)

inline size_t up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct Layout {
  int hs = 0;  // row pitch of H in elements
  size_t h = 0, z = 0, hpart = 0, scores = 0, sx = 0, sidx = 0, gemv_part = 0, total = 0;
  int sidx_stride = 0;
  // merged lists of short blocks (merge_g blocks per 128 tokens; 0 = none)
  int merge_g = 0, mu_stride = 0, mu_kmax = 0;
  size_t mu_idx = 0, mu_mask = 0, mu_k = 0;
  // fp32 partial sums of the down GEMM where a few lists much longer than the rest are cut along k
  size_t g2part = 0, g2part_bytes = 0;
};

constexpr int kMergeTokens = 128;   // short blocks are merged up to the token tile of the 128-token kernels

// Blocks shorter than the 128-token tile leave most of it idle and fetch every weight row for few
// tokens.  When the lists are long (little sparsity) the union of g = 128 / block neighbouring lists
// is hardly longer than one of them, and running the union over all 128 tokens, with the activations
// of the pairs (sub-block, neuron) nobody selected written as zero, computes the same sums faster.
// A call of at most 8 tokens (the GEMV kernels) merges all its lists into one for the same reason.
// Returns g, or 0 where merging does not apply to this shape at all.
int merge_factor(const ff_shape &s, int lds_limit) {
  if ((size_t)s.d_ffn + 1024 > (size_t)lds_limit) return 0;   // a membership byte per neuron in LDS
  if (s.n_tokens <= s.block) return 0;
  if (s.n_tokens <= kGemvMaxTokens) {
    // the few-token kernels read every listed row once per list: all the call's lists (at most 8) become one
    return ff_gemv_eligible(s.n_tokens, s.n_tokens, s.d_model, lds_limit) ? (s.n_tokens + s.block - 1) / s.block : 0;
  }
  if (s.block >= kMergeTokens || s.block < 16 || (s.block & (s.block - 1)) != 0) return 0;
  return kMergeTokens / s.block;
}
// whether it pays: expected length of the union of g independent lists of keep fraction f (real lists
// overlap more), against the measured rate of the short-block tiles relative to the 128-token ones
// (Llama-3.1-8B shape: 64-token blocks gain up to 50% sparsity and break even up to 75%; 32-token blocks
// gain everywhere)
bool merge_pays(int g, double f, bool few_tokens) {
  double none = 1.0;
  for (int i = 0; i < g; ++i) none *= 1.0 - f;
  // few tokens: bytes read, one pass over the union against one pass over each of the g lists
  if (few_tokens) return (1.0 - none) / (g * f) < 0.9;
  const double rel_eff = g == 2 ? 0.55 : (g == 4 ? 0.32 : 0.18);
  return (1.0 - none) / f * rel_eff < 0.92;
}

// the merge factor a call with these per-block K should use (0 = run the blocks' own tiles)
int merge_choice(const ff_ctx *ctx, const ff_shape &s, const int32_t *k_per_block, int n_blocks);

// pred_only: just what ff_predict's kernels use (pooling logits, the first layer's partial sums, scores);
// merge_g > 1: with room for the lists of every merge_g blocks merged into one
Layout make_layout(const ff_shape &s, int k_max, bool pred_only = false, int merge_g = 0) {
  Layout L;
  const size_t nB = ((size_t)s.n_tokens + s.block - 1) / s.block;
  const size_t T = s.n_tokens;
  L.merge_g = merge_g > 1 ? merge_g : 0;
  L.mu_kmax = L.merge_g ? (int)std::min<long>((long)s.d_ffn, (long)L.merge_g * k_max) : 0;
  L.mu_stride = (int)up((size_t)L.mu_kmax, 64);
  L.hs = (int)up((size_t)std::max(k_max, L.mu_kmax) + s.r_comp, 64);
  L.sidx_stride = (int)up((size_t)k_max, 64);
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += up(bytes, 256); return at; };
  L.h = take(pred_only ? 0 : T * L.hs * 2);
  L.z = take(T * 8);
  L.hpart = take(nB * (((size_t)s.d_model + 511) / 512) * (size_t)s.r_pred * 8);
  L.scores = take(nB * (size_t)s.d_ffn * 8);
  L.sx = take(pred_only ? 0 : T * s.d_model * 2);
  L.sidx = take(pred_only ? 0 : nB * (size_t)L.sidx_stride * 4);
  L.gemv_part = take(pred_only ? 0 : ff_gemv_part_bytes(s.n_tokens, s.d_model));
  if (L.merge_g) {
    const size_t nG = (nB + L.merge_g - 1) / L.merge_g;
    L.mu_idx = take(nG * L.mu_stride * 4);
    L.mu_mask = take(nG * L.mu_stride);
    L.mu_k = take(nG * 4);
  }
  L.g2part_bytes = pred_only ? 0 : ff_gemm2_part_bytes(s.n_tokens, s.block, s.d_model);
  L.g2part = take(L.g2part_bytes);
  L.total = o;
  return L;
}

ff_status check_shape(ff_ctx *ctx, const ff_shape *s, bool need_pred) {
  if (!s) return fail(ctx, FF_ERR_INVALID_ARG, "shape is NULL");
  if (s->d_model <= 0 || s->d_ffn <= 0 || s->n_tokens <= 0 || s->block <= 0)
    return fail(ctx, FF_ERR_INVALID_ARG, "sizes must be positive");
  if (s->d_model % 128) return fail(ctx, FF_ERR_SHAPE, "d_model (%d) must be a multiple of 128", s->d_model);
  if (s->d_ffn % 8) return fail(ctx, FF_ERR_SHAPE, "d_ffn (%d) must be a multiple of 8", s->d_ffn);
  if (need_pred && (s->r_pred < 1 || s->r_pred > 1024))
    return fail(ctx, FF_ERR_SHAPE, "r_pred (%d) must be in [1, 1024]", s->r_pred);
  if (s->r_comp < 0 || s->r_comp > 4096 || s->r_comp % 8)
    return fail(ctx, FF_ERR_SHAPE, "r_comp (%d) must be a multiple of 8 in [0, 4096]", s->r_comp);
  if ((long)s->n_tokens + s->block > 0x7fffffffL) return fail(ctx, FF_ERR_SHAPE, "n_tokens + block must stay below 2^31");
  const long nB = ((long)s->n_tokens + s->block - 1) / s->block;
  if (nB > kRingCap) return fail(ctx, FF_ERR_SHAPE, "more than %d blocks", kRingCap);
  return FF_OK;
}

// validates k_per_block, finds max / uniformity
ff_status scan_k(ff_ctx *ctx, const int32_t *k, int n, int d_ffn, int k_stride, int *k_max, bool *uniform) {
  if (!k) return fail(ctx, FF_ERR_INVALID_ARG, "k_per_block is NULL");
  int mx = 0;
  bool uni = true;
  for (int i = 0; i < n; ++i) {
    if (k[i] < 1 || k[i] > d_ffn) return fail(ctx, FF_ERR_INVALID_ARG, "k_per_block[%d] = %d not in [1, %d]", i, k[i], d_ffn);
    mx = std::max(mx, k[i]);
    uni = uni && k[i] == k[0];
  }
  if (k_stride < mx) return fail(ctx, FF_ERR_INVALID_ARG, "k_stride (%d) < largest k (%d)", k_stride, mx);
  *k_max = mx;
  *uniform = uni;
  return FF_OK;
}

// host K array -> KSpec (staged through the pinned ring when not uniform)
ff_status stage_k(ff_ctx *ctx, const int32_t *k, int n, int k_max, bool uniform, KSpec *out) {
  *out = KSpec();
  out->k_max = k_max;
  out->uniform = k[0];
  out->per_block = nullptr;
  out->k_base = k_max;
  if (uniform) return FF_OK;
  {  // scheduling hints: the most common K, and the few blocks above it
    std::vector<int32_t> &sorted = ctx->k_sorted;   // capacity reserved at ff_create: no allocation here
    sorted.assign(k, k + n);
    std::sort(sorted.begin(), sorted.end());
    int best = sorted[0], best_n = 0;
    for (int i = 0; i < n;) {
      int j = i;
      while (j < n && sorted[j] == sorted[i]) ++j;
      if (j - i > best_n) { best_n = j - i; best = sorted[i]; }
      i = j;
    }
    int above = 0;
    for (int i = 0; i < n; ++i) above += k[i] > best;
    if (above >= 1 && above <= kMaxHeavy) {
      out->k_base = best;
      for (int i = 0; i < n; ++i)
        if (k[i] > best) out->heavy[out->n_heavy++] = i;
    }
  }
  // The copy below reads a pinned slot that later calls overwrite: a captured graph would replay
  // it with whatever the slot holds by then.
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  FF_HIP(ctx, hipStreamIsCapturing(ctx->stream, &cap));
  if (cap != hipStreamCaptureStatusNone)
    return fail(ctx, FF_ERR_INVALID_ARG, "k_per_block with unequal entries cannot be captured in a HIP graph (its values are copied at call time)");
  // The same values as the copy enqueued last on this stream (ff_predict and ff_sparse_ffn of one step, or the
  // next step with the same budgets): that slot is the newest, so nothing has overwritten it.
  if (ctx->staged_slot >= 0 && ctx->staged_n == n &&
      memcmp(ctx->ring[ctx->staged_slot].host, k, (size_t)n * sizeof(int32_t)) == 0) {
    out->per_block = ctx->ring[ctx->staged_slot].dev;
    return FF_OK;
  }
  const int slot = ctx->ring_next;
  Slot &sl = ctx->ring[slot];
  ctx->staged_slot = -1;
  ctx->ring_next = (ctx->ring_next + 1) % kRing;
  if (sl.used) FF_HIP(ctx, hipEventSynchronize(sl.ev));
  memcpy(sl.host, k, (size_t)n * sizeof(int32_t));
  FF_HIP(ctx, hipMemcpyAsync(sl.dev, sl.host, (size_t)n * sizeof(int32_t), hipMemcpyHostToDevice, ctx->stream));
  FF_HIP(ctx, hipEventRecord(sl.ev, ctx->stream));
  sl.used = true;
  ctx->staged_slot = slot;
  ctx->staged_n = n;
  out->per_block = sl.dev;
  return FF_OK;
}

ff_status need_ws(ff_ctx *ctx, const Layout &L) {
  if (!ctx->ws) return fail(ctx, FF_ERR_WORKSPACE, "no workspace set (ff_set_workspace)");
  if (ctx->ws_bytes < L.total)
    return fail(ctx, FF_ERR_WORKSPACE, "workspace has %zu bytes, this call needs %zu", ctx->ws_bytes, L.total);
  return FF_OK;
}

inline uint8_t *wsp(ff_ctx *ctx, size_t off) { return static_cast<uint8_t *>(ctx->ws) + off; }

// predict with K already on the device
ff_status run_predict(ff_ctx *ctx, const ff_shape &s, const Layout &L, const void *x, const ff_predictor &pr,
                      const KSpec &ks, int k_stride, int32_t *indices, double *scores_opt, void *scratch_base = nullptr) {
  uint8_t *base = static_cast<uint8_t *>(scratch_base ? scratch_base : ctx->ws);
  PredictParams p;
  p.x = static_cast<const bf16_t *>(x);
  p.q_pred = static_cast<const bf16_t *>(pr.q_pred);
  p.w1 = static_cast<const bf16_t *>(pr.w1);
  p.w2 = static_cast<const bf16_t *>(pr.w2);
  p.T = s.n_tokens; p.d_model = s.d_model; p.d_ffn = s.d_ffn; p.block = s.block; p.r = s.r_pred;
  p.n_blocks = (s.n_tokens + s.block - 1) / s.block;
  p.z = reinterpret_cast<double *>(base + L.z);
  p.hpart = reinterpret_cast<double *>(base + L.hpart);
  p.scores = scores_opt ? scores_opt : reinterpret_cast<double *>(base + L.scores);
  p.k = ks;
  p.k_stride = k_stride;
  p.indices = indices;
  FF_HIP(ctx, ff_launch_predict(p, ctx->lds_limit, ctx->stream, &ctx->prof));
  return FF_OK;
}

ff_status run_ffn(ff_ctx *ctx, const ff_shape &s, const Layout &L, const void *x, const ff_ffn_weights &w,
                  const ff_compensator *comp, const int32_t *indices, const KSpec &ks, int k_stride,
                  void *y, int out_dtype, int block, int g1v, int g2v, bf16_t *residual = nullptr, bool merge = true) {
  const int g1split = ctx->gemm1_split;
  const int rc = comp ? s.r_comp : 0;
  if (ctx->small_path && g1v < 0 && g2v < 0 && ff_gemv_eligible(s.n_tokens, block, s.d_model, ctx->lds_limit)) {
    GemvParams v;
    v.x = static_cast<const bf16_t *>(x);
    v.wg = static_cast<const bf16_t *>(w.w_gate);
    v.wu = static_cast<const bf16_t *>(w.w_up);
    v.wd = static_cast<const bf16_t *>(w.w_down);
    v.wc1 = comp ? static_cast<const bf16_t *>(comp->wc1) : nullptr;
    v.wc2 = comp ? static_cast<const bf16_t *>(comp->wc2) : nullptr;
    v.idx = indices;
    v.h = reinterpret_cast<bf16_t *>(wsp(ctx, L.h));
    v.part = reinterpret_cast<float *>(wsp(ctx, L.gemv_part));
    v.y = y;
    v.res = residual;
    v.T = s.n_tokens; v.d_model = s.d_model; v.d_ffn = s.d_ffn; v.block = block;
    v.n_blocks = (s.n_tokens + block - 1) / block;
    v.rc = rc; v.comp_act = comp ? comp->act : FF_ACT_SILU; v.k_stride = k_stride; v.hs = L.hs;
    v.out_f32 = out_dtype == FF_OUT_F32;
    v.k = ks;
    if (merge && L.merge_g > 1 && indices != nullptr) {
      // all lists of the call merged into one, read once for all tokens; H is zero where a token did not
      // select the neuron
      int32_t *u_idx = reinterpret_cast<int32_t *>(wsp(ctx, L.mu_idx));
      uint8_t *u_mask = wsp(ctx, L.mu_mask);
      int32_t *u_k = reinterpret_cast<int32_t *>(wsp(ctx, L.mu_k));
      prof_begin(&ctx->prof, FF_STAGE_GEMM1, ctx->stream);
      FF_HIP(ctx, ff_launch_merge_lists(indices, k_stride, ks, v.n_blocks, L.merge_g, s.d_ffn, u_idx, u_mask,
                                        L.mu_stride, u_k, ctx->lds_limit, ctx->stream));
      prof_end(&ctx->prof, ctx->stream);
      v.idx = u_idx;
      v.k_stride = L.mu_stride;
      v.mask = u_mask;
      v.sub_block = block;
      v.block = s.n_tokens;
      v.n_blocks = 1;
      v.k = KSpec();
      v.k.per_block = u_k;
      v.k.uniform = L.mu_kmax;
      v.k.k_max = L.mu_kmax;
      v.k.k_base = L.mu_kmax;
    }
    FF_HIP(ctx, ff_launch_gemv(v, ctx->lds_limit, ctx->stream, &ctx->prof));
    return FF_OK;
  }
  Gemm1Params a;
  a.x = static_cast<const bf16_t *>(x);
  a.wg = static_cast<const bf16_t *>(w.w_gate);
  a.wu = static_cast<const bf16_t *>(w.w_up);
  a.wc1 = comp ? static_cast<const bf16_t *>(comp->wc1) : nullptr;
  a.idx = indices;
  a.h = reinterpret_cast<bf16_t *>(wsp(ctx, L.h));
  a.T = s.n_tokens; a.d_model = s.d_model; a.d_ffn = s.d_ffn; a.block = block;
  a.n_blocks = (s.n_tokens + block - 1) / block;
  a.rc = rc; a.comp_act = comp ? comp->act : FF_ACT_SILU; a.k_stride = k_stride; a.hs = L.hs;
  a.k = ks;
  prof_begin(&ctx->prof, FF_STAGE_GEMM1, ctx->stream);
  if (merge && L.merge_g > 1 && indices != nullptr) {
    // the lists of every merge_g neighbouring blocks become one list over 128 tokens; both GEMMs then
    // run on those (their lengths are known on the device only: an upper bound sizes the launches)
    int32_t *u_idx = reinterpret_cast<int32_t *>(wsp(ctx, L.mu_idx));
    uint8_t *u_mask = wsp(ctx, L.mu_mask);
    int32_t *u_k = reinterpret_cast<int32_t *>(wsp(ctx, L.mu_k));
    FF_HIP(ctx, ff_launch_merge_lists(indices, k_stride, ks, a.n_blocks, L.merge_g, s.d_ffn, u_idx, u_mask,
                                      L.mu_stride, u_k, ctx->lds_limit, ctx->stream));
    a.idx = u_idx;
    a.k_stride = L.mu_stride;
    a.mask = u_mask;
    a.sub_shift = 0;
    while ((1 << a.sub_shift) < block) ++a.sub_shift;
    a.block = kMergeTokens;
    a.n_blocks = (s.n_tokens + kMergeTokens - 1) / kMergeTokens;
    a.k = KSpec();
    a.k.per_block = u_k;
    a.k.uniform = L.mu_kmax;
    a.k.k_max = L.mu_kmax;
    a.k.k_base = L.mu_kmax;
  }
  FF_HIP(ctx, ff_launch_gemm1(a, g1v, g1split, ctx->gemm1_heavy_tiles, ctx->stream));
  prof_end(&ctx->prof, ctx->stream);
  Gemm2Params g;
  g.h = a.h;
  g.wd = static_cast<const bf16_t *>(w.w_down);
  g.wc2 = comp ? static_cast<const bf16_t *>(comp->wc2) : nullptr;
  g.idx = a.idx;
  g.y = y;
  g.res = residual;
  g.T = s.n_tokens; g.d_model = s.d_model; g.d_ffn = s.d_ffn; g.block = a.block; g.n_blocks = a.n_blocks;
  g.rc = rc; g.k_stride = a.k_stride; g.hs = L.hs; g.out_f32 = out_dtype == FF_OUT_F32;
  g.k = a.k;
  if (L.g2part_bytes > 0 && g.block == s.block) {
    g.part = reinterpret_cast<float *>(wsp(ctx, L.g2part));
    g.part_bytes = L.g2part_bytes;
  }
  prof_begin(&ctx->prof, FF_STAGE_GEMM2, ctx->stream);
  FF_HIP(ctx, ff_launch_gemm2(g, g2v, ctx->gemm2_split, ctx->gemm2_row_mode, ctx->gemm2_ksplit, ctx->stream));
  prof_end(&ctx->prof, ctx->stream);
  return FF_OK;
}

int merge_choice(const ff_ctx *ctx, const ff_shape &s, const int32_t *k_per_block, int n_blocks) {
  const int mg = merge_factor(s, ctx->lds_limit);
  if (mg <= 1 || ctx->merge_blocks == 0 || ctx->gemm1_variant >= 0 || ctx->gemm2_variant >= 0) return 0;
  if (ctx->merge_blocks > 0) return mg;
  double k_sum = 0.0;
  for (int i = 0; i < n_blocks; ++i) k_sum += k_per_block[i];
  const bool few = s.n_tokens <= kGemvMaxTokens;
  if (few && !ctx->small_path) return 0;
  return merge_pays(mg, k_sum / n_blocks / s.d_ffn, few) ? mg : 0;
}

ff_status check_weights(ff_ctx *ctx, const ff_ffn_weights *w) {
  if (!w || !w->w_gate || !w->w_up || !w->w_down) return fail(ctx, FF_ERR_INVALID_ARG, "FFN weight pointer is NULL");
  if (!aligned16(w->w_gate) || !aligned16(w->w_up) || !aligned16(w->w_down))
    return fail(ctx, FF_ERR_ALIGNMENT, "FFN weights must be 16-byte aligned");
  return FF_OK;
}
ff_status check_pred(ff_ctx *ctx, const ff_shape &s, const ff_predictor *p) {
  if (!p || !p->w1 || !p->w2) return fail(ctx, FF_ERR_INVALID_ARG, "predictor weight pointer is NULL");
  if (!aligned16(p->w1) || !aligned16(p->w2) || !aligned16(p->q_pred))
    return fail(ctx, FF_ERR_ALIGNMENT, "predictor weights must be 16-byte aligned");
  if (p->q_pred && s.block > 4096) return fail(ctx, FF_ERR_SHAPE, "softmax pooling takes blocks of at most 4096 tokens");
  return FF_OK;
}
ff_status check_comp(ff_ctx *ctx, const ff_shape &s, const ff_compensator *c) {
  if (!c) return FF_OK;
  if (s.r_comp <= 0) return fail(ctx, FF_ERR_INVALID_ARG, "compensator given but r_comp = %d", s.r_comp);
  if (!c->wc1 || !c->wc2) return fail(ctx, FF_ERR_INVALID_ARG, "compensator weight pointer is NULL");
  if (!aligned16(c->wc1) || !aligned16(c->wc2)) return fail(ctx, FF_ERR_ALIGNMENT, "compensator weights must be 16-byte aligned");
  if (c->act < FF_ACT_SILU || c->act > FF_ACT_IDENTITY) return fail(ctx, FF_ERR_INVALID_ARG, "unknown compensator activation %d", c->act);
  return FF_OK;
}

}  // namespace

static void prof_free(ff_ctx *ctx);

extern "C" {

const char *ff_status_str(int status) {
  switch (status) {
    case FF_OK: return "ok";
    case FF_ERR_INVALID_ARG: return "invalid argument";
    case FF_ERR_SHAPE: return "unsupported shape";
    case FF_ERR_ALIGNMENT: return "misaligned pointer";
    case FF_ERR_INDEX: return "bad index list";
    case FF_ERR_WORKSPACE: return "workspace missing or too small";
    case FF_ERR_DEVICE: return "device error";
    case FF_ERR_UNIMPLEMENTED: return "not implemented";
  }
  return "unknown status";
}

const char *ff_last_error(const ff_ctx *ctx) { return ctx ? ctx->err : "context is NULL"; }

ff_status ff_create(ff_ctx **out, int device, void *hip_stream) {
  if (!out) return FF_ERR_INVALID_ARG;
  *out = nullptr;
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev) return FF_ERR_DEVICE;
  ff_ctx *ctx = new (std::nothrow) ff_ctx();
  if (!ctx) return FF_ERR_DEVICE;
  ctx->device = device;
  ctx->stream = static_cast<hipStream_t>(hip_stream);
  ff_status st = FF_OK;
  do {
    if (hipSetDevice(device) != hipSuccess) { st = FF_ERR_DEVICE; break; }
    int lds = 0;
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, device) != hipSuccess) { st = FF_ERR_DEVICE; break; }
    ctx->lds_limit = lds;
    if (device < kMaxDevices) {
      // once per device, with that device current: each GPU holds its own copy of the array
      if (g_scratch_ptr[device] == nullptr) {
        void *sp = nullptr;
        if (hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)) != hipSuccess || sp == nullptr) { st = FF_ERR_DEVICE; break; }
        g_scratch_ptr[device] = sp;
      }
      ctx->static_scratch = g_scratch_ptr[device];
    }
    try {
      ctx->k_sorted.reserve(kRingCap);
    } catch (...) {   // nothing may be thrown across the C boundary
      st = FF_ERR_DEVICE;
      break;
    }
    if (ff_gemm_init(lds) != hipSuccess) { st = FF_ERR_DEVICE; break; }
    for (int i = 0; i < kRing && st == FF_OK; ++i) {
      if (hipHostMalloc(reinterpret_cast<void **>(&ctx->ring[i].host), kRingCap * sizeof(int32_t), hipHostMallocDefault) != hipSuccess ||
          hipMalloc(reinterpret_cast<void **>(&ctx->ring[i].dev), kRingCap * sizeof(int32_t)) != hipSuccess ||
          hipEventCreateWithFlags(&ctx->ring[i].ev, hipEventDisableTiming) != hipSuccess)
        st = FF_ERR_DEVICE;
    }
    if (st != FF_OK) break;
    if (hipMalloc(reinterpret_cast<void **>(&ctx->flag_dev), 256) != hipSuccess ||
        hipHostMalloc(reinterpret_cast<void **>(&ctx->flag_host), 256, hipHostMallocDefault) != hipSuccess)
      st = FF_ERR_DEVICE;
  } while (0);
  if (st != FF_OK) {
    ff_destroy(ctx);
    return st;
  }
  *out = ctx;
  return FF_OK;
}

ff_status ff_destroy(ff_ctx *ctx) {
  if (!ctx) return FF_OK;
  (void)hipSetDevice(ctx->device);
  (void)hipStreamSynchronize(ctx->stream);
  for (int i = 0; i < kRing; ++i) {
    if (ctx->ring[i].host) (void)hipHostFree(ctx->ring[i].host);
    if (ctx->ring[i].dev) (void)hipFree(ctx->ring[i].dev);
    if (ctx->ring[i].ev) (void)hipEventDestroy(ctx->ring[i].ev);
  }
  if (ctx->flag_dev) (void)hipFree(ctx->flag_dev);
  if (ctx->flag_host) (void)hipHostFree(ctx->flag_host);
  prof_free(ctx);
  delete ctx;
  return FF_OK;
}

ff_status ff_set_stream(ff_ctx *ctx, void *hip_stream) {
  if (!ctx) return FF_ERR_INVALID_ARG;
  FF_HIP(ctx, hipStreamSynchronize(ctx->stream));  // staged K arrays are ordered on the old stream
  ctx->stream = static_cast<hipStream_t>(hip_stream);
  return FF_OK;
}

ff_status ff_workspace_bytes(const ff_shape *shape, int32_t k_max, size_t *bytes) {
  if (!bytes) return FF_ERR_INVALID_ARG;
  ff_status st = check_shape(nullptr, shape, false);
  if (st != FF_OK) return st;
  if (k_max < 1 || k_max > shape->d_ffn) return FF_ERR_INVALID_ARG;
  // (with room for the merged lists of short blocks, whether or not a call will use them)
  *bytes = std::max(make_layout(*shape, k_max).total,
                    make_layout(*shape, k_max, false, merge_factor(*shape, 160 * 1024)).total);
  return FF_OK;
}

ff_status ff_set_workspace(ff_ctx *ctx, void *dev_ptr, size_t bytes) {
  if (!ctx) return FF_ERR_INVALID_ARG;
  if (dev_ptr && (reinterpret_cast<uintptr_t>(dev_ptr) & 255u)) return fail(ctx, FF_ERR_ALIGNMENT, "workspace must be 256-byte aligned");
  ctx->ws = dev_ptr;
  ctx->ws_bytes = dev_ptr ? bytes : 0;
  return FF_OK;
}

ff_status ff_set_option(ff_ctx *ctx, const char *name, int32_t value) {
  if (!ctx || !name) return FF_ERR_INVALID_ARG;
  if (!strcmp(name, "validate")) { ctx->validate = value != 0; return FF_OK; }
  if (!strcmp(name, "gemm1_variant")) {
    if (value >= ff_gemm1_num_variants()) return fail(ctx, FF_ERR_INVALID_ARG, "gemm1_variant %d does not exist", value);
    ctx->gemm1_variant = value;
    return FF_OK;
  }
  if (!strcmp(name, "gemm1_split")) { ctx->gemm1_split = value < 0 ? -1 : (value != 0); return FF_OK; }
  if (!strcmp(name, "gemm1_heavy_tiles")) { ctx->gemm1_heavy_tiles = value < 0 ? -1 : (value != 0); return FF_OK; }
  if (!strcmp(name, "gemm2_split")) { ctx->gemm2_split = value < 0 ? -1 : (value != 0); return FF_OK; }
  if (!strcmp(name, "small_path")) { ctx->small_path = value != 0; return FF_OK; }
  if (!strcmp(name, "merge_blocks")) { ctx->merge_blocks = value < 0 ? -1 : (value != 0); return FF_OK; }
  if (!strcmp(name, "gemm2_row_mode")) {
    if (value == 0 || value > 3) return fail(ctx, FF_ERR_INVALID_ARG, "gemm2_row_mode %d does not exist", value);
    ctx->gemm2_row_mode = value < 0 ? -1 : value;
    return FF_OK;
  }
  if (!strcmp(name, "gemm2_ksplit")) { ctx->gemm2_ksplit = value < 0 ? -1 : value; return FF_OK; }
  if (!strcmp(name, "gemm2_variant")) {
    if (value >= ff_gemm2_num_variants()) return fail(ctx, FF_ERR_INVALID_ARG, "gemm2_variant %d does not exist", value);
    ctx->gemm2_variant = value;
    return FF_OK;
  }
  return fail(ctx, FF_ERR_INVALID_ARG, "unknown option '%s'", name);
}

static void prof_free(ff_ctx *ctx) {
  Profiler &pr = ctx->prof;
  for (int i = 0; i < 2 * pr.cap; ++i)
    if (pr.ev && pr.ev[i]) (void)hipEventDestroy(pr.ev[i]);
  delete[] pr.ev;
  delete[] pr.stage;
  pr = Profiler();
}

ff_status ff_profile_enable(ff_ctx *ctx, int32_t max_records, uint32_t stage_mask) {
  if (!ctx || max_records < 0 || max_records > (1 << 20)) return FF_ERR_INVALID_ARG;
  FF_HIP(ctx, hipSetDevice(ctx->device));
  FF_HIP(ctx, hipStreamSynchronize(ctx->stream));
  prof_free(ctx);
  if (max_records == 0) return FF_OK;
  Profiler &pr = ctx->prof;
  pr.ev = new (std::nothrow) hipEvent_t[2 * (size_t)max_records]();
  pr.stage = new (std::nothrow) int32_t[max_records]();
  if (!pr.ev || !pr.stage) { prof_free(ctx); return fail(ctx, FF_ERR_DEVICE, "out of host memory"); }
  pr.cap = max_records;
  pr.mask = stage_mask;
  for (int i = 0; i < 2 * max_records; ++i)
    if (hipEventCreate(&pr.ev[i]) != hipSuccess) { prof_free(ctx); return fail(ctx, FF_ERR_DEVICE, "hipEventCreate failed"); }
  return FF_OK;
}

ff_status ff_profile_read(ff_ctx *ctx, double *ms_sum, int32_t *launches) {
  if (!ctx || !ms_sum || !launches) return FF_ERR_INVALID_ARG;
  for (int i = 0; i < FF_N_STAGES; ++i) { ms_sum[i] = 0.0; launches[i] = 0; }
  FF_HIP(ctx, hipStreamSynchronize(ctx->stream));
  Profiler &pr = ctx->prof;
  for (int i = 0; i < pr.n; ++i) {
    float ms = 0.f;
    FF_HIP(ctx, hipEventElapsedTime(&ms, pr.ev[2 * i], pr.ev[2 * i + 1]));
    ms_sum[pr.stage[i]] += ms;
    launches[pr.stage[i]] += 1;
  }
  pr.n = 0;
  pr.open = -1;
  return FF_OK;
}

ff_status ff_k_from_sparsity(int32_t d_ffn, double sparsity, int32_t *k) {
  if (!k || d_ffn < 1 || !(sparsity >= 0.0 && sparsity <= 1.0)) return FF_ERR_INVALID_ARG;
  const double v = std::floor((1.0 - sparsity) * (double)d_ffn + 0.5);
  *k = (int32_t)std::min<double>(std::max<double>(v, 1.0), (double)d_ffn);
  return FF_OK;
}

ff_status ff_layer_budgets(const double *importance, int32_t n_layers, double budget, double *keep_fraction) {
  if (!importance || !keep_fraction || n_layers < 1 || !(budget > 0.0 && budget <= 1.0)) return FF_ERR_INVALID_ARG;
  double s_total = 0.0;
  for (int i = 0; i < n_layers; ++i) {
    if (!(importance[i] > 0.0)) return FF_ERR_INVALID_ARG;
    s_total += importance[i];
  }
  double left = budget * (double)n_layers;  // budget not yet handed out
  for (int i = 0; i < n_layers; ++i) {
    const double b = std::min(1.0, importance[i] / s_total * left);
    keep_fraction[i] = b;
    left -= b;
    s_total -= importance[i];
  }
  return FF_OK;
}

ff_status ff_predict(ff_ctx *ctx, const ff_shape *shape, const void *x, const ff_predictor *pred,
                     const int32_t *k_per_block, int32_t k_stride, int32_t *indices, double *scores_opt) {
  if (!ctx) return FF_ERR_INVALID_ARG;
  ff_status st = check_shape(ctx, shape, true);
  if (st != FF_OK) return st;
  if (!x || !indices) return fail(ctx, FF_ERR_INVALID_ARG, "x or indices is NULL");
  if (!aligned16(x) || !aligned16(indices) || !aligned16(scores_opt)) return fail(ctx, FF_ERR_ALIGNMENT, "x / indices / scores must be 16-byte aligned");
  if ((st = check_pred(ctx, *shape, pred)) != FF_OK) return st;
  const int nB = (shape->n_tokens + shape->block - 1) / shape->block;
  int k_max;
  bool uniform;
  if ((st = scan_k(ctx, k_per_block, nB, shape->d_ffn, k_stride, &k_max, &uniform)) != FF_OK) return st;
  const Layout L = make_layout(*shape, k_max);
  if ((st = need_ws(ctx, L)) != FF_OK) return st;
  FF_HIP(ctx, hipSetDevice(ctx->device));
  KSpec ks;
  if ((st = stage_k(ctx, k_per_block, nB, k_max, uniform, &ks)) != FF_OK) return st;
  return run_predict(ctx, *shape, L, x, *pred, ks, k_stride, indices, scores_opt);
}

ff_status ff_predict_static(ff_ctx *ctx, const ff_shape *shape, const void *x, const ff_predictor *pred,
                            const int32_t *k_per_block, int32_t k_stride, int32_t *indices, double *scores_opt) {
  if (!ctx) return FF_ERR_INVALID_ARG;
  ff_status st = check_shape(ctx, shape, true);
  if (st != FF_OK) return st;
  if (!x || !indices) return fail(ctx, FF_ERR_INVALID_ARG, "x or indices is NULL");
  if (!aligned16(x) || !aligned16(indices) || !aligned16(scores_opt)) return fail(ctx, FF_ERR_ALIGNMENT, "x / indices / scores must be 16-byte aligned");
  if ((st = check_pred(ctx, *shape, pred)) != FF_OK) return st;
  const int nB = (shape->n_tokens + shape->block - 1) / shape->block;
  int k_max;
  bool uniform;
  if ((st = scan_k(ctx, k_per_block, nB, shape->d_ffn, k_stride, &k_max, &uniform)) != FF_OK) return st;
  const Layout L = make_layout(*shape, k_max, true);
  if (L.total > (size_t)FF_STATIC_SCRATCH_BYTES)
    return fail(ctx, FF_ERR_WORKSPACE, "this shape needs %zu bytes of predictor scratch, the built-in array has %u "
                                       "(use ff_predict with a workspace)", L.total, (unsigned)FF_STATIC_SCRATCH_BYTES);
  if (!ctx->static_scratch) return fail(ctx, FF_ERR_DEVICE, "no built-in scratch on device %d", ctx->device);
  FF_HIP(ctx, hipSetDevice(ctx->device));
  KSpec ks;
  if ((st = stage_k(ctx, k_per_block, nB, k_max, uniform, &ks)) != FF_OK) return st;
  // every byte of scratch the kernels read they have written earlier in this same call: nothing to clear
  return run_predict(ctx, *shape, L, x, *pred, ks, k_stride, indices, scores_opt, ctx->static_scratch);
}

ff_status ff_sparse_ffn(ff_ctx *ctx, const ff_shape *shape, const void *x, const ff_ffn_weights *w,
                        const ff_compensator *comp, const int32_t *indices, const int32_t *k_per_block,
                        int32_t k_stride, void *y, int32_t out_dtype) {
  if (!ctx) return FF_ERR_INVALID_ARG;
  ff_status st = check_shape(ctx, shape, false);
  if (st != FF_OK) return st;
  if (!x || !indices || !y) return fail(ctx, FF_ERR_INVALID_ARG, "x, indices or y is NULL");
  if (!aligned16(x) || !aligned16(indices) || !aligned16(y)) return fail(ctx, FF_ERR_ALIGNMENT, "x / indices / y must be 16-byte aligned");
  if (out_dtype != FF_OUT_BF16 && out_dtype != FF_OUT_F32) return fail(ctx, FF_ERR_INVALID_ARG, "unknown out_dtype %d", out_dtype);
  if ((st = check_weights(ctx, w)) != FF_OK) return st;
  if ((st = check_comp(ctx, *shape, comp)) != FF_OK) return st;
  const int nB = (shape->n_tokens + shape->block - 1) / shape->block;
  int k_max;
  bool uniform;
  if ((st = scan_k(ctx, k_per_block, nB, shape->d_ffn, k_stride, &k_max, &uniform)) != FF_OK) return st;
  ff_shape s = *shape;
  if (!comp) s.r_comp = 0;
  Layout L = make_layout(s, k_max);
  if ((st = need_ws(ctx, L)) != FF_OK) return st;
  // short blocks with long lists: merge the lists of neighbouring blocks when that is expected to pay
  // and the workspace has room for the merged lists (ff_workspace_bytes asks for it)
  const int mg = merge_choice(ctx, s, k_per_block, nB);
  if (mg > 1) {
    const Layout Lm = make_layout(s, k_max, false, mg);
    if (ctx->ws_bytes >= Lm.total) L = Lm;
  }
  FF_HIP(ctx, hipSetDevice(ctx->device));
  KSpec ks;
  if ((st = stage_k(ctx, k_per_block, nB, k_max, uniform, &ks)) != FF_OK) return st;
  if (ctx->validate) {
    // the check reads its result back and waits for it: not something a graph can hold
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    FF_HIP(ctx, hipStreamIsCapturing(ctx->stream, &cap));
    if (cap != hipStreamCaptureStatusNone)
      return fail(ctx, FF_ERR_INVALID_ARG, "the validate option synchronises the stream and cannot be captured in a HIP graph");
    FF_HIP(ctx, hipMemsetAsync(ctx->flag_dev, 0, sizeof(int32_t), ctx->stream));
    FF_HIP(ctx, ff_launch_validate(indices, nB, k_stride, ks, shape->d_ffn, ctx->flag_dev, ctx->stream));
    FF_HIP(ctx, hipMemcpyAsync(ctx->flag_host, ctx->flag_dev, sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream));
    FF_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->flag_host[0] != 0)
      return fail(ctx, FF_ERR_INDEX, "index row of block %d is not ascending, in range and -1 padded", ctx->flag_host[0] - 1);
  }
  // Every block keeps every neuron: a valid list of d_ffn entries can only be 0 .. d_ffn-1, so the
  // blocks no longer differ and the tokens are tiled as in the dense call (the compensator still rides along).
  if (uniform && k_max == s.d_ffn && !(ctx->small_path && ff_gemv_eligible(s.n_tokens, s.block, s.d_model, ctx->lds_limit)) &&
      ctx->gemm1_variant < 0 && ctx->gemm2_variant < 0) {
    L.merge_g = 0;
    return run_ffn(ctx, s, L, x, *w, comp, nullptr, ks, 0, y, out_dtype, std::max(s.block, 256), -1, -1);
  }
  return run_ffn(ctx, s, L, x, *w, comp, indices, ks, k_stride, y, out_dtype, shape->block,
                 ctx->gemm1_variant, ctx->gemm2_variant);
}

ff_status ff_dense_ffn(ff_ctx *ctx, const ff_shape *shape, const void *x, const ff_ffn_weights *w, void *y,
                       int32_t out_dtype) {
  if (!ctx) return FF_ERR_INVALID_ARG;
  if (!shape) return fail(ctx, FF_ERR_INVALID_ARG, "shape is NULL");
  ff_shape s = *shape;
  s.r_comp = 0;
  s.r_pred = 1;
  s.block = 256;  // no selection: tokens are only grouped into M tiles
  ff_status st = check_shape(ctx, &s, false);
  if (st != FF_OK) return st;
  if (!x || !y) return fail(ctx, FF_ERR_INVALID_ARG, "x or y is NULL");
  if (!aligned16(x) || !aligned16(y)) return fail(ctx, FF_ERR_ALIGNMENT, "x / y must be 16-byte aligned");
  if (out_dtype != FF_OUT_BF16 && out_dtype != FF_OUT_F32) return fail(ctx, FF_ERR_INVALID_ARG, "unknown out_dtype %d", out_dtype);
  if ((st = check_weights(ctx, w)) != FF_OK) return st;
  const Layout L = make_layout(s, s.d_ffn);
  // only H is used by this call
  if (!ctx->ws) return fail(ctx, FF_ERR_WORKSPACE, "no workspace set (ff_set_workspace)");
  // (the few-token kernels also keep their partial sums there)
  const bool few = ctx->small_path && ff_gemv_eligible(s.n_tokens, s.block, s.d_model, ctx->lds_limit);
  const size_t need = few ? L.gemv_part + ff_gemv_part_bytes(s.n_tokens, s.d_model) : (size_t)s.n_tokens * L.hs * 2;
  if (ctx->ws_bytes < need) return fail(ctx, FF_ERR_WORKSPACE, "workspace has %zu bytes, dense_ffn needs %zu", ctx->ws_bytes, need);
  FF_HIP(ctx, hipSetDevice(ctx->device));
  KSpec ks;
  ks.per_block = nullptr;
  ks.uniform = s.d_ffn;
  ks.k_max = s.d_ffn;
  ks.k_base = s.d_ffn;
  return run_ffn(ctx, s, L, x, *w, nullptr, nullptr, ks, 0, y, out_dtype, s.block, ctx->gemm1_variant,
                 ctx->gemm2_variant);
}

ff_status ff_rmsnorm(ff_ctx *ctx, int32_t n_tokens, int32_t d_model, const void *h, float eps, void *x) {
  if (!ctx) return FF_ERR_INVALID_ARG;
  if (!h || !x || n_tokens < 1 || d_model < 1) return fail(ctx, FF_ERR_INVALID_ARG, "bad argument");
  if (d_model % 8) return fail(ctx, FF_ERR_SHAPE, "d_model must be a multiple of 8");
  if (!aligned16(h) || !aligned16(x)) return fail(ctx, FF_ERR_ALIGNMENT, "h / x must be 16-byte aligned");
  FF_HIP(ctx, hipSetDevice(ctx->device));
  FF_HIP(ctx, ff_launch_rmsnorm(static_cast<const bf16_t *>(h), static_cast<bf16_t *>(x), n_tokens, d_model, eps, ctx->stream));
  return FF_OK;
}

ff_status ff_residual_add(ff_ctx *ctx, int32_t n_tokens, int32_t d_model, void *h, const void *y) {
  if (!ctx) return FF_ERR_INVALID_ARG;
  if (!h || !y || n_tokens < 1 || d_model < 1) return fail(ctx, FF_ERR_INVALID_ARG, "bad argument");
  if (d_model % 8) return fail(ctx, FF_ERR_SHAPE, "d_model must be a multiple of 8");
  if (!aligned16(h) || !aligned16(y)) return fail(ctx, FF_ERR_ALIGNMENT, "h / y must be 16-byte aligned");
  FF_HIP(ctx, hipSetDevice(ctx->device));
  FF_HIP(ctx, ff_launch_residual(static_cast<bf16_t *>(h), static_cast<const bf16_t *>(y), (size_t)n_tokens * d_model, ctx->stream));
  return FF_OK;
}

ff_status ff_copy(ff_ctx *ctx, void *dst, const void *src, size_t bytes) {
  if (!ctx) return FF_ERR_INVALID_ARG;
  if (!dst || !src || bytes == 0 || bytes % 16 || bytes / 16 / 256 > 0x7fffffffu) return fail(ctx, FF_ERR_INVALID_ARG, "bad argument");
  if (!aligned16(dst) || !aligned16(src)) return fail(ctx, FF_ERR_ALIGNMENT, "dst / src must be 16-byte aligned");
  FF_HIP(ctx, hipSetDevice(ctx->device));
  FF_HIP(ctx, ff_launch_copy(dst, src, bytes, ctx->stream));
  return FF_OK;
}

ff_status ff_mfma_peak(ff_ctx *ctx, int32_t iters, int32_t zero_operands, double *flops) {
  if (!ctx) return FF_ERR_INVALID_ARG;
  if (!flops || iters < 1 || iters > (1 << 24)) return fail(ctx, FF_ERR_INVALID_ARG, "bad argument");
  FF_HIP(ctx, hipSetDevice(ctx->device));
  FF_HIP(ctx, ff_launch_mfma_peak(iters, zero_operands != 0, reinterpret_cast<float *>(ctx->flag_dev) + 8, flops, ctx->stream));
  return FF_OK;
}

ff_status ff_ffn_stack(ff_ctx *ctx, const ff_shape *shape, int32_t n_layers, void *h, const ff_predictor *pred,
                       const ff_ffn_weights *w, const ff_compensator *comp, const int32_t *k_per_layer_block,
                       int32_t k_stride, float rms_eps, int32_t *indices_opt, void *x_dump_opt) {
  if (!ctx) return FF_ERR_INVALID_ARG;
  ff_status st = check_shape(ctx, shape, true);
  if (st != FF_OK) return st;
  if (!h || !pred || !w || !k_per_layer_block || n_layers < 1) return fail(ctx, FF_ERR_INVALID_ARG, "bad argument");
  if (!aligned16(h) || !aligned16(indices_opt) || !aligned16(x_dump_opt)) return fail(ctx, FF_ERR_ALIGNMENT, "h / indices / x_dump must be 16-byte aligned");
  const int nB = (shape->n_tokens + shape->block - 1) / shape->block;
  int k_max_all = 0;
  for (int l = 0; l < n_layers; ++l) {
    int km;
    bool uni;
    if ((st = scan_k(ctx, k_per_layer_block + (size_t)l * nB, nB, shape->d_ffn, indices_opt ? k_stride : shape->d_ffn, &km, &uni)) != FF_OK) return st;
    k_max_all = std::max(k_max_all, km);
    if ((st = check_weights(ctx, &w[l])) != FF_OK) return st;
    if ((st = check_pred(ctx, *shape, &pred[l])) != FF_OK) return st;
    if (comp && (st = check_comp(ctx, *shape, &comp[l])) != FF_OK) return st;
  }
  ff_shape s = *shape;
  if (!comp) s.r_comp = 0;
  Layout L = make_layout(s, k_max_all);
  if ((st = need_ws(ctx, L)) != FF_OK) return st;
  // short blocks: one layout with room for merged lists serves every layer; each layer decides for itself
  bool any_merge = false;
  for (int l = 0; l < n_layers; ++l) any_merge = any_merge || merge_choice(ctx, s, k_per_layer_block + (size_t)l * nB, nB) > 1;
  if (any_merge) {
    const Layout Lm = make_layout(s, k_max_all, false, merge_factor(s, ctx->lds_limit));
    if (ctx->ws_bytes >= Lm.total) L = Lm;
  }
  FF_HIP(ctx, hipSetDevice(ctx->device));
  const size_t act_elems = (size_t)s.n_tokens * s.d_model;
  for (int l = 0; l < n_layers; ++l) {
    const int32_t *kl = k_per_layer_block + (size_t)l * nB;
    int km;
    bool uni;
    (void)scan_k(ctx, kl, nB, s.d_ffn, s.d_ffn, &km, &uni);
    KSpec ks;
    if ((st = stage_k(ctx, kl, nB, km, uni, &ks)) != FF_OK) return st;
    bf16_t *xbuf = x_dump_opt ? static_cast<bf16_t *>(x_dump_opt) + (size_t)l * act_elems
                              : reinterpret_cast<bf16_t *>(wsp(ctx, L.sx));
    int32_t *idx = indices_opt ? indices_opt + (size_t)l * nB * k_stride : reinterpret_cast<int32_t *>(wsp(ctx, L.sidx));
    const int stride = indices_opt ? k_stride : L.sidx_stride;
    prof_begin(&ctx->prof, FF_STAGE_GLUE, ctx->stream);
    FF_HIP(ctx, ff_launch_rmsnorm(static_cast<const bf16_t *>(h), xbuf, s.n_tokens, s.d_model, rms_eps, ctx->stream));
    prof_end(&ctx->prof, ctx->stream);
    if ((st = run_predict(ctx, s, L, xbuf, pred[l], ks, stride, idx, nullptr)) != FF_OK) return st;
    // the residual add h <- bf16(h + bf16(y)) happens in the down GEMM's epilogue
    if ((st = run_ffn(ctx, s, L, xbuf, w[l], comp ? &comp[l] : nullptr, idx, ks, stride, nullptr, FF_OUT_BF16,
                      s.block, ctx->gemm1_variant, ctx->gemm2_variant, static_cast<bf16_t *>(h),
                      merge_choice(ctx, s, kl, nB) > 1)) != FF_OK) return st;
  }
  return FF_OK;
}

}  // extern "C"

/* Host-side checks of the C ABI, meant to be built with the host sanitizers
 * (-fsanitize=address,undefined on the host pass only) and run as a program of its own.
 *
 * Part 1 needs no GPU: the pure host helpers at their edges, every entry point with a NULL
 * context, ff_create on devices that do not exist.
 * Part 2 runs when device 0 exists: every argument error of every compute call.  The context is
 * given a workspace of 1 KiB only, and the pointers are made-up aligned addresses, so a call that
 * passed every argument check would still stop at "workspace too small" before anything is launched;
 * the calls that take no workspace are only ever given invalid arguments.
 * Part 3 (device 0 exists) makes real, valid calls on zero-filled device buffers of a tiny layer, enough
 * of them to wrap the pinned ring that stages unequal K, with stage timing and list validation on:
 * the host code between the checks and the launches runs under the sanitizers too.
 *
 * Exit code 0 = every call returned what it should; the sanitizers abort on their own findings.   */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "fastforward.h"
#include "fastforward_diag.h"

static int n_fail = 0, n_checks = 0;
#define EXPECT(call, want)                                                                     \
  do {                                                                                         \
    ff_status got_ = (call);                                                                   \
    ++n_checks;                                                                                \
    if (got_ != (want)) {                                                                      \
      ++n_fail;                                                                                \
      fprintf(stderr, "line %d: %s returned %d (%s), expected %d\n", __LINE__, #call, (int)got_, \
              ff_status_str(got_), (int)(want));                                               \
    }                                                                                          \
  } while (0)

#define FAKE(n) ((void *)(uintptr_t)(0x10000000u + 0x100000u * (n)))   /* aligned, never dereferenced */

static void part1_no_gpu(void) {
  int32_t k = 0;
  double keep[4];
  const double imp[4] = {1.0, 2.0, 3.0, 4.0}, bad[2] = {1.0, -1.0};
  size_t bytes = 0;
  ff_ctx *ctx = NULL;
  ff_shape ok = {4096, 14336, 8192, 128, 128, 64};
  ff_shape huge = {1 << 20, 1 << 30, 2147483647 - 131072, 131072, 1024, 4096};
  ff_shape s;
  ff_predictor pr = {NULL, FAKE(1), FAKE(2)};
  ff_ffn_weights w = {FAKE(3), FAKE(4), FAKE(5)};
  const int32_t kb[1] = {1};
  int i;

  for (i = -1; i < 10; ++i)
    if (!ff_status_str((ff_status)i)) ++n_fail;
  if (!ff_last_error(NULL)) ++n_fail;

  EXPECT(ff_k_from_sparsity(14336, 0.5, &k), FF_OK);
  if (k != 7168) ++n_fail;
  EXPECT(ff_k_from_sparsity(1, 1.0, &k), FF_OK);
  if (k != 1) ++n_fail;
  EXPECT(ff_k_from_sparsity(2147483647, 0.0, &k), FF_OK);
  if (k != 2147483647) ++n_fail;
  EXPECT(ff_k_from_sparsity(10, NAN, &k), FF_ERR_INVALID_ARG);
  EXPECT(ff_k_from_sparsity(10, -0.1, &k), FF_ERR_INVALID_ARG);
  EXPECT(ff_k_from_sparsity(0, 0.5, &k), FF_ERR_INVALID_ARG);
  EXPECT(ff_k_from_sparsity(10, 0.5, NULL), FF_ERR_INVALID_ARG);

  EXPECT(ff_layer_budgets(imp, 4, 0.5, keep), FF_OK);
  EXPECT(ff_layer_budgets(imp, 1, 1.0, keep), FF_OK);
  EXPECT(ff_layer_budgets(bad, 2, 0.5, keep), FF_ERR_INVALID_ARG);
  EXPECT(ff_layer_budgets(imp, 0, 0.5, keep), FF_ERR_INVALID_ARG);
  EXPECT(ff_layer_budgets(imp, 4, 0.0, keep), FF_ERR_INVALID_ARG);
  EXPECT(ff_layer_budgets(imp, 4, NAN, keep), FF_ERR_INVALID_ARG);
  EXPECT(ff_layer_budgets(NULL, 4, 0.5, keep), FF_ERR_INVALID_ARG);
  EXPECT(ff_layer_budgets(imp, 4, 0.5, NULL), FF_ERR_INVALID_ARG);

  EXPECT(ff_workspace_bytes(&ok, 7168, &bytes), FF_OK);
  if (bytes < (size_t)8192 * (7168 + 64) * 2) ++n_fail;
  EXPECT(ff_workspace_bytes(&ok, 7168, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_workspace_bytes(NULL, 7168, &bytes), FF_ERR_INVALID_ARG);
  EXPECT(ff_workspace_bytes(&ok, 0, &bytes), FF_ERR_INVALID_ARG);
  EXPECT(ff_workspace_bytes(&ok, 14337, &bytes), FF_ERR_INVALID_ARG);
  EXPECT(ff_workspace_bytes(&huge, 1 << 30, &bytes), FF_OK);   /* sizes are computed in size_t */
  s = huge; s.n_tokens = 2147483647;
  EXPECT(ff_workspace_bytes(&s, 1 << 30, &bytes), FF_ERR_SHAPE);
  s = ok; s.d_model = 100;
  EXPECT(ff_workspace_bytes(&s, 7168, &bytes), FF_ERR_SHAPE);
  s = ok; s.d_ffn = 14340;
  EXPECT(ff_workspace_bytes(&s, 7168, &bytes), FF_ERR_SHAPE);
  s = ok; s.r_comp = 5000;
  EXPECT(ff_workspace_bytes(&s, 7168, &bytes), FF_ERR_SHAPE);
  s = ok; s.block = 0;
  EXPECT(ff_workspace_bytes(&s, 7168, &bytes), FF_ERR_INVALID_ARG);
  s = ok; s.n_tokens = 40000; s.block = 2;
  EXPECT(ff_workspace_bytes(&s, 7168, &bytes), FF_ERR_SHAPE);   /* more blocks than a call takes */

  EXPECT(ff_create(NULL, 0, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_create(&ctx, -1, NULL), FF_ERR_DEVICE);
  EXPECT(ff_create(&ctx, 9999, NULL), FF_ERR_DEVICE);
  if (ctx != NULL) ++n_fail;
  EXPECT(ff_destroy(NULL), FF_OK);
  EXPECT(ff_set_stream(NULL, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_set_workspace(NULL, FAKE(6), 1024), FF_ERR_INVALID_ARG);
  EXPECT(ff_set_option(NULL, "validate", 1), FF_ERR_INVALID_ARG);
  EXPECT(ff_profile_enable(NULL, 4, 1), FF_ERR_INVALID_ARG);
  EXPECT(ff_profile_read(NULL, keep, &k), FF_ERR_INVALID_ARG);
  EXPECT(ff_predict(NULL, &ok, FAKE(7), &pr, kb, 1, (int32_t *)FAKE(8), NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_predict_static(NULL, &ok, FAKE(7), &pr, kb, 1, (int32_t *)FAKE(8), NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_sparse_ffn(NULL, &ok, FAKE(7), &w, NULL, (const int32_t *)FAKE(8), kb, 1, FAKE(9), FF_OUT_F32), FF_ERR_INVALID_ARG);
  EXPECT(ff_dense_ffn(NULL, &ok, FAKE(7), &w, FAKE(9), FF_OUT_F32), FF_ERR_INVALID_ARG);
  EXPECT(ff_ffn_stack(NULL, &ok, 1, FAKE(7), &pr, &w, NULL, kb, 1, 1e-6f, NULL, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_rmsnorm(NULL, 4, 128, FAKE(7), 1e-6f, FAKE(9)), FF_ERR_INVALID_ARG);
  EXPECT(ff_residual_add(NULL, 4, 128, FAKE(7), FAKE(9)), FF_ERR_INVALID_ARG);
  EXPECT(ff_copy(NULL, FAKE(7), FAKE(9), 1024), FF_ERR_INVALID_ARG);
}

static void part2_argument_errors(ff_ctx *ctx) {
  ff_shape ok = {256, 688, 256, 64, 32, 16};
  ff_shape s;
  ff_predictor pr = {NULL, FAKE(1), FAKE(2)}, prq = {FAKE(10), FAKE(1), FAKE(2)}, pr_bad;
  ff_ffn_weights w = {FAKE(3), FAKE(4), FAKE(5)}, w_bad;
  ff_compensator cp = {FAKE(11), FAKE(12), FF_ACT_SILU}, cp_bad;
  int32_t ks[4] = {344, 344, 344, 344}, ks_zero[4] = {344, 0, 344, 344}, ks_big[4] = {344, 689, 344, 344};
  int32_t ks_ragged[4] = {688, 100, 344, 7};
  void *x = FAKE(7), *y = FAKE(9);
  int32_t *idx = (int32_t *)FAKE(8);
  void *odd = (void *)((uintptr_t)FAKE(13) + 2);

  EXPECT(ff_set_option(ctx, NULL, 1), FF_ERR_INVALID_ARG);
  EXPECT(ff_set_option(ctx, "no_such_option", 1), FF_ERR_INVALID_ARG);
  EXPECT(ff_set_option(ctx, "gemm1_variant", 1000), FF_ERR_INVALID_ARG);
  EXPECT(ff_set_option(ctx, "gemm2_variant", 1000), FF_ERR_INVALID_ARG);
  EXPECT(ff_set_option(ctx, "gemm2_row_mode", 4), FF_ERR_INVALID_ARG);
  EXPECT(ff_set_option(ctx, "gemm2_row_mode", 0), FF_ERR_INVALID_ARG);
  {
    static const char *const names[] = {"validate", "small_path", "merge_blocks", "gemm1_split", "gemm2_split",
                                        "gemm1_heavy_tiles", "gemm2_ksplit"};
    size_t n;
    for (n = 0; n < sizeof(names) / sizeof(names[0]); ++n) {   /* every documented name is known; back to the default */
      EXPECT(ff_set_option(ctx, names[n], 1), FF_OK);
      EXPECT(ff_set_option(ctx, names[n], strcmp(names[n], "validate") && strcmp(names[n], "small_path") ? -1 : (n == 1)), FF_OK);
    }
  }
  EXPECT(ff_set_workspace(ctx, odd, 1024), FF_ERR_ALIGNMENT);
  EXPECT(ff_profile_enable(ctx, -1, 1), FF_ERR_INVALID_ARG);

  /* no workspace at all, then one of 1 KiB: valid arguments stop there, nothing is launched */
  EXPECT(ff_set_workspace(ctx, NULL, 0), FF_OK);
  EXPECT(ff_predict(ctx, &ok, x, &pr, ks, 344, idx, NULL), FF_ERR_WORKSPACE);
  EXPECT(ff_set_workspace(ctx, FAKE(6), 1024), FF_OK);
  EXPECT(ff_predict(ctx, &ok, x, &pr, ks, 344, idx, NULL), FF_ERR_WORKSPACE);
  EXPECT(ff_predict(ctx, &ok, x, &prq, ks_ragged, 688, idx, (double *)FAKE(14)), FF_ERR_WORKSPACE);
  EXPECT(ff_sparse_ffn(ctx, &ok, x, &w, &cp, idx, ks, 344, y, FF_OUT_BF16), FF_ERR_WORKSPACE);
  EXPECT(ff_sparse_ffn(ctx, &ok, x, &w, NULL, idx, ks_ragged, 688, y, FF_OUT_F32), FF_ERR_WORKSPACE);
  EXPECT(ff_dense_ffn(ctx, &ok, x, &w, y, FF_OUT_F32), FF_ERR_WORKSPACE);
  EXPECT(ff_ffn_stack(ctx, &ok, 1, x, &pr, &w, &cp, ks, 344, 1e-6f, NULL, NULL), FF_ERR_WORKSPACE);

  /* shapes */
  s = ok; s.d_model = 200;
  EXPECT(ff_predict(ctx, &s, x, &pr, ks, 344, idx, NULL), FF_ERR_SHAPE);
  EXPECT(ff_predict_static(ctx, &s, x, &pr, ks, 344, idx, NULL), FF_ERR_SHAPE);
  EXPECT(ff_sparse_ffn(ctx, &s, x, &w, &cp, idx, ks, 344, y, FF_OUT_BF16), FF_ERR_SHAPE);
  EXPECT(ff_dense_ffn(ctx, &s, x, &w, y, FF_OUT_BF16), FF_ERR_SHAPE);
  s = ok; s.d_ffn = 690;
  EXPECT(ff_sparse_ffn(ctx, &s, x, &w, &cp, idx, ks, 344, y, FF_OUT_BF16), FF_ERR_SHAPE);
  s = ok; s.r_pred = 0;
  EXPECT(ff_predict(ctx, &s, x, &pr, ks, 344, idx, NULL), FF_ERR_SHAPE);
  s = ok; s.r_pred = 2000;
  EXPECT(ff_predict_static(ctx, &s, x, &pr, ks, 344, idx, NULL), FF_ERR_SHAPE);
  s = ok; s.r_comp = 12;
  EXPECT(ff_sparse_ffn(ctx, &s, x, &w, &cp, idx, ks, 344, y, FF_OUT_BF16), FF_ERR_SHAPE);
  s = ok; s.n_tokens = 0;
  EXPECT(ff_sparse_ffn(ctx, &s, x, &w, &cp, idx, ks, 344, y, FF_OUT_BF16), FF_ERR_INVALID_ARG);
  s = ok; s.block = -4;
  EXPECT(ff_predict(ctx, &s, x, &pr, ks, 344, idx, NULL), FF_ERR_INVALID_ARG);
  s = ok; s.n_tokens = 20000; s.block = 1;
  EXPECT(ff_predict(ctx, &s, x, &pr, ks, 344, idx, NULL), FF_ERR_SHAPE);
  s = ok; s.block = 8192; s.n_tokens = 8192;
  EXPECT(ff_predict(ctx, &s, x, &prq, ks, 344, idx, NULL), FF_ERR_SHAPE);   /* softmax pooling: block too long */
  EXPECT(ff_predict(ctx, NULL, x, &pr, ks, 344, idx, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_dense_ffn(ctx, NULL, x, &w, y, FF_OUT_BF16), FF_ERR_INVALID_ARG);
  /* a predictor scratch beyond the built-in array (the one check ff_predict_static adds) */
  s.d_model = 4096; s.d_ffn = 14336; s.n_tokens = 512 * 128; s.block = 128; s.r_pred = 128; s.r_comp = 64;
  {
    int32_t *kmany = (int32_t *)malloc(512 * sizeof(int32_t));
    int i;
    for (i = 0; i < 512; ++i) kmany[i] = 7168;
    EXPECT(ff_predict_static(ctx, &s, x, &pr, kmany, 7168, idx, NULL), FF_ERR_WORKSPACE);
    free(kmany);
  }

  /* pointers */
  EXPECT(ff_predict(ctx, &ok, NULL, &pr, ks, 344, idx, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_predict(ctx, &ok, x, &pr, ks, 344, NULL, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_predict(ctx, &ok, x, NULL, ks, 344, idx, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_predict(ctx, &ok, x, &pr, NULL, 344, idx, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_predict(ctx, &ok, odd, &pr, ks, 344, idx, NULL), FF_ERR_ALIGNMENT);
  EXPECT(ff_predict(ctx, &ok, x, &pr, ks, 344, idx, (double *)odd), FF_ERR_ALIGNMENT);
  EXPECT(ff_predict_static(ctx, &ok, x, &pr, ks, 344, (int32_t *)odd, NULL), FF_ERR_ALIGNMENT);
  EXPECT(ff_predict_static(ctx, &ok, NULL, &pr, ks, 344, idx, NULL), FF_ERR_INVALID_ARG);
  pr_bad = pr; pr_bad.w2 = NULL;
  EXPECT(ff_predict(ctx, &ok, x, &pr_bad, ks, 344, idx, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_predict_static(ctx, &ok, x, &pr_bad, ks, 344, idx, NULL), FF_ERR_INVALID_ARG);
  pr_bad = pr; pr_bad.q_pred = odd;
  EXPECT(ff_predict(ctx, &ok, x, &pr_bad, ks, 344, idx, NULL), FF_ERR_ALIGNMENT);
  w_bad = w; w_bad.w_up = NULL;
  EXPECT(ff_sparse_ffn(ctx, &ok, x, &w_bad, &cp, idx, ks, 344, y, FF_OUT_BF16), FF_ERR_INVALID_ARG);
  EXPECT(ff_dense_ffn(ctx, &ok, x, &w_bad, y, FF_OUT_BF16), FF_ERR_INVALID_ARG);
  w_bad = w; w_bad.w_down = odd;
  EXPECT(ff_sparse_ffn(ctx, &ok, x, &w_bad, &cp, idx, ks, 344, y, FF_OUT_BF16), FF_ERR_ALIGNMENT);
  EXPECT(ff_sparse_ffn(ctx, &ok, x, NULL, &cp, idx, ks, 344, y, FF_OUT_BF16), FF_ERR_INVALID_ARG);
  EXPECT(ff_sparse_ffn(ctx, &ok, x, &w, &cp, NULL, ks, 344, y, FF_OUT_BF16), FF_ERR_INVALID_ARG);
  EXPECT(ff_sparse_ffn(ctx, &ok, x, &w, &cp, idx, ks, 344, NULL, FF_OUT_BF16), FF_ERR_INVALID_ARG);
  EXPECT(ff_sparse_ffn(ctx, &ok, x, &w, &cp, idx, ks, 344, odd, FF_OUT_BF16), FF_ERR_ALIGNMENT);
  cp_bad = cp; cp_bad.wc2 = NULL;
  EXPECT(ff_sparse_ffn(ctx, &ok, x, &w, &cp_bad, idx, ks, 344, y, FF_OUT_BF16), FF_ERR_INVALID_ARG);
  cp_bad = cp; cp_bad.wc1 = odd;
  EXPECT(ff_sparse_ffn(ctx, &ok, x, &w, &cp_bad, idx, ks, 344, y, FF_OUT_BF16), FF_ERR_ALIGNMENT);
  cp_bad = cp; cp_bad.act = 9;
  EXPECT(ff_sparse_ffn(ctx, &ok, x, &w, &cp_bad, idx, ks, 344, y, FF_OUT_BF16), FF_ERR_INVALID_ARG);
  s = ok; s.r_comp = 0;
  EXPECT(ff_sparse_ffn(ctx, &s, x, &w, &cp, idx, ks, 344, y, FF_OUT_BF16), FF_ERR_INVALID_ARG);   /* compensator without units */

  /* K, pitch, output type */
  EXPECT(ff_sparse_ffn(ctx, &ok, x, &w, &cp, idx, ks_zero, 344, y, FF_OUT_BF16), FF_ERR_INVALID_ARG);
  EXPECT(ff_sparse_ffn(ctx, &ok, x, &w, &cp, idx, ks_big, 689, y, FF_OUT_BF16), FF_ERR_INVALID_ARG);
  EXPECT(ff_sparse_ffn(ctx, &ok, x, &w, &cp, idx, ks, 343, y, FF_OUT_BF16), FF_ERR_INVALID_ARG);
  EXPECT(ff_sparse_ffn(ctx, &ok, x, &w, &cp, idx, ks, 344, y, 7), FF_ERR_INVALID_ARG);
  EXPECT(ff_dense_ffn(ctx, &ok, x, &w, y, -1), FF_ERR_INVALID_ARG);
  EXPECT(ff_predict(ctx, &ok, x, &pr, ks_zero, 344, idx, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_predict_static(ctx, &ok, x, &pr, ks_big, 689, idx, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_predict_static(ctx, &ok, x, &pr, ks, 100, idx, NULL), FF_ERR_INVALID_ARG);

  /* stack */
  EXPECT(ff_ffn_stack(ctx, &ok, 0, x, &pr, &w, &cp, ks, 344, 1e-6f, NULL, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_ffn_stack(ctx, &ok, 1, NULL, &pr, &w, &cp, ks, 344, 1e-6f, NULL, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_ffn_stack(ctx, &ok, 1, x, &pr, &w, &cp, NULL, 344, 1e-6f, NULL, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_ffn_stack(ctx, &ok, 1, odd, &pr, &w, &cp, ks, 344, 1e-6f, NULL, NULL), FF_ERR_ALIGNMENT);
  EXPECT(ff_ffn_stack(ctx, &ok, 1, x, &pr, &w, &cp, ks, 100, 1e-6f, idx, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_ffn_stack(ctx, &ok, 1, x, &pr, &w_bad, &cp, ks, 344, 1e-6f, NULL, NULL), FF_ERR_ALIGNMENT);

  /* calls without a workspace: invalid arguments only */
  EXPECT(ff_rmsnorm(ctx, 4, 128, NULL, 1e-6f, y), FF_ERR_INVALID_ARG);
  EXPECT(ff_rmsnorm(ctx, 0, 128, x, 1e-6f, y), FF_ERR_INVALID_ARG);
  EXPECT(ff_rmsnorm(ctx, 4, 100, x, 1e-6f, y), FF_ERR_SHAPE);
  EXPECT(ff_rmsnorm(ctx, 4, 128, odd, 1e-6f, y), FF_ERR_ALIGNMENT);
  EXPECT(ff_residual_add(ctx, 4, 128, x, NULL), FF_ERR_INVALID_ARG);
  EXPECT(ff_residual_add(ctx, 4, 100, x, y), FF_ERR_SHAPE);
  EXPECT(ff_residual_add(ctx, 4, 128, x, odd), FF_ERR_ALIGNMENT);
  EXPECT(ff_copy(ctx, x, y, 0), FF_ERR_INVALID_ARG);
  EXPECT(ff_copy(ctx, x, y, 100), FF_ERR_INVALID_ARG);
  EXPECT(ff_copy(ctx, NULL, y, 1024), FF_ERR_INVALID_ARG);
  EXPECT(ff_copy(ctx, odd, y, 1024), FF_ERR_ALIGNMENT);
  if (!strlen(ff_last_error(ctx))) ++n_fail;
  EXPECT(ff_set_workspace(ctx, NULL, 0), FF_OK);
}

static int part3_real_calls(ff_ctx *ctx) {
  /* a tiny layer, all inputs zero (every score ties: the lists are 0 .. K-1, the output is 0) */
  ff_shape sh = {256, 688, 230, 64, 32, 16};
  const size_t dm = 256, df = 688, T = 230;
  const int32_t nB = 4, ks_ragged[4] = {688, 100, 344, 7}, ks[4] = {344, 344, 344, 344};
  const int32_t kl[2 * 4] = {344, 344, 344, 344, 688, 100, 344, 7};
  void *x = NULL, *wg = NULL, *wu = NULL, *wd = NULL, *w1 = NULL, *w2 = NULL, *wc1 = NULL, *wc2 = NULL, *y = NULL, *ws = NULL, *h = NULL;
  int32_t *idx = NULL, host_idx[8];
  size_t need = 0;
  double ms[FF_N_STAGES];
  int32_t cnt[FF_N_STAGES];
  int i, rc = 0;
  ff_predictor pr;
  ff_ffn_weights w;
  ff_compensator cp;
  ff_predictor prs[2];
  ff_ffn_weights wsl[2];
  ff_compensator cps[2];

  if (ff_workspace_bytes(&sh, 688, &need) != FF_OK) return 1;
#define DEVBUF(p, n) do { if (hipMalloc((void **)&(p), (n)) != hipSuccess || hipMemset((p), 0, (n)) != hipSuccess) { rc = 1; goto done; } } while (0)
  DEVBUF(x, T * dm * 2); DEVBUF(h, T * dm * 2); DEVBUF(wg, df * dm * 2); DEVBUF(wu, df * dm * 2); DEVBUF(wd, df * dm * 2);
  DEVBUF(w1, dm * 32 * 2); DEVBUF(w2, 32 * df * 2); DEVBUF(wc1, 16 * dm * 2); DEVBUF(wc2, 16 * dm * 2);
  DEVBUF(y, T * dm * 4); DEVBUF(idx, (size_t)nB * 688 * 4); DEVBUF(ws, need);
  pr.q_pred = NULL; pr.w1 = w1; pr.w2 = w2;
  w.w_gate = wg; w.w_up = wu; w.w_down = wd;
  cp.wc1 = wc1; cp.wc2 = wc2; cp.act = FF_ACT_SILU;
  EXPECT(ff_set_workspace(ctx, ws, need), FF_OK);
  EXPECT(ff_set_option(ctx, "validate", 1), FF_OK);
  EXPECT(ff_profile_enable(ctx, 64, 0x3fu), FF_OK);
  for (i = 0; i < 12; ++i) {            /* more calls with new unequal K than the staging ring has slots */
    int32_t ks_step[4];
    memcpy(ks_step, ks_ragged, sizeof(ks_step));
    ks_step[1] += i;                     /* (equal values would reuse the copy staged last) */
    EXPECT(ff_predict(ctx, &sh, x, &pr, ks_step, 688, idx, NULL), FF_OK);
    EXPECT(ff_sparse_ffn(ctx, &sh, x, &w, &cp, idx, ks_step, 688, y, (i & 1) ? FF_OUT_F32 : FF_OUT_BF16), FF_OK);
  }
  {                                     /* the launchers' choices for a few much longer lists, each way */
    int32_t ks_long[4] = {688, 96, 96, 600};
    int v;
    EXPECT(ff_predict(ctx, &sh, x, &pr, ks_long, 688, idx, NULL), FF_OK);
    EXPECT(ff_set_option(ctx, "merge_blocks", 0), FF_OK);   /* the blocks' own lists, not merged ones */
    for (v = 0; v < 4; ++v) {
      EXPECT(ff_set_option(ctx, "gemm2_ksplit", v == 3 ? 16 : v), FF_OK);
      EXPECT(ff_set_option(ctx, "gemm1_heavy_tiles", v & 1), FF_OK);
      EXPECT(ff_set_option(ctx, "gemm1_split", v < 2), FF_OK);
      EXPECT(ff_sparse_ffn(ctx, &sh, x, &w, &cp, idx, ks_long, 688, y, FF_OUT_BF16), FF_OK);
    }
    EXPECT(ff_set_option(ctx, "gemm2_ksplit", -1), FF_OK);
    EXPECT(ff_set_option(ctx, "gemm1_heavy_tiles", -1), FF_OK);
    EXPECT(ff_set_option(ctx, "gemm1_split", -1), FF_OK);
    EXPECT(ff_set_option(ctx, "merge_blocks", -1), FF_OK);
  }
  EXPECT(ff_predict_static(ctx, &sh, x, &pr, ks, 688, idx, NULL), FF_OK);
  EXPECT(ff_sparse_ffn(ctx, &sh, x, &w, NULL, idx, ks, 688, y, FF_OUT_F32), FF_OK);
  EXPECT(ff_dense_ffn(ctx, &sh, x, &w, y, FF_OUT_F32), FF_OK);
  EXPECT(ff_profile_read(ctx, ms, cnt), FF_OK);
  if (cnt[FF_STAGE_GEMM1] < 1 || cnt[FF_STAGE_TOPK] < 1) ++n_fail;
  EXPECT(ff_profile_enable(ctx, 0, 0), FF_OK);
  EXPECT(ff_set_option(ctx, "validate", 0), FF_OK);
  prs[0] = prs[1] = pr; wsl[0] = wsl[1] = w; cps[0] = cps[1] = cp;
  EXPECT(ff_ffn_stack(ctx, &sh, 2, h, prs, wsl, cps, kl, 688, 1e-6f, NULL, NULL), FF_OK);
  EXPECT(ff_rmsnorm(ctx, (int32_t)T, (int32_t)dm, h, 1e-6f, x), FF_OK);
  EXPECT(ff_residual_add(ctx, (int32_t)T, (int32_t)dm, h, x), FF_OK);
  EXPECT(ff_copy(ctx, y, x, T * dm * 2), FF_OK);
  if (hipDeviceSynchronize() != hipSuccess) { rc = 1; goto done; }
  if (hipMemcpy(host_idx, idx, sizeof(host_idx), hipMemcpyDeviceToHost) != hipSuccess) { rc = 1; goto done; }
  for (i = 0; i < 8; ++i)
    if (host_idx[i] != i) ++n_fail;     /* all scores equal: the lowest indices win */
done:
  (void)ff_set_workspace(ctx, NULL, 0);
  (void)hipDeviceSynchronize();
  hipFree(x); hipFree(h); hipFree(wg); hipFree(wu); hipFree(wd); hipFree(w1); hipFree(w2); hipFree(wc1); hipFree(wc2);
  hipFree(y); hipFree(idx); hipFree(ws);
  return rc;
}

int main(void) {
  ff_ctx *ctx = NULL;
  ff_status st;
  part1_no_gpu();
  st = ff_create(&ctx, 0, NULL);
  if (st == FF_OK) {
    part2_argument_errors(ctx);
    if (part3_real_calls(ctx)) { fprintf(stderr, "device memory set-up failed\n"); ++n_fail; }
    EXPECT(ff_destroy(ctx), FF_OK);
    printf("host checks with a GPU: %d calls checked, %d wrong\n", n_checks, n_fail);
  } else {
    printf("host checks without a GPU (ff_create: %s): %d calls checked, %d wrong\n", ff_status_str(st), n_checks, n_fail);
  }
  return n_fail ? 1 : 0;
}

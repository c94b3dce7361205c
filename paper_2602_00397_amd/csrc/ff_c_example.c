/* A caller of the C ABI that knows nothing of Python or PyTorch: plain C, the HIP runtime for
 * device memory, and libfastforward.  It reads one layer's inputs from a file, runs ff_predict and
 * ff_sparse_ffn (Eq. 12-21), and writes the index lists and the output to another file.  Used by the
 * GPU tests to check the library outside a PyTorch process, and as an example of the boundary.
 *
 * input file : int32 d_model, d_ffn, n_tokens, block, r_pred, r_comp, k; then bf16 bit patterns of
 *              x [T][d_model], w_gate, w_up, w_down [d_ffn][d_model] each, w1 [d_model][r_pred],
 *              w2 [r_pred][d_ffn], wc1, wc2 [r_comp][d_model] each
 * output file: int32 indices [n_blocks][k], then float y [T][d_model]
 * usage      : ff_c_example <input> <output>                                                        */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "fastforward.h"

#define HIP_OK(call)                                                              \
  do {                                                                            \
    hipError_t e_ = (call);                                                       \
    if (e_ != hipSuccess) {                                                       \
      fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));                  \
      return 2;                                                                   \
    }                                                                             \
  } while (0)
#define FF_CHECK(call)                                                            \
  do {                                                                            \
    ff_status s_ = (call);                                                        \
    if (s_ != FF_OK) {                                                            \
      fprintf(stderr, "%s: %s (%s)\n", #call, ff_status_str(s_), ff_last_error(ctx)); \
      return 3;                                                                   \
    }                                                                             \
  } while (0)

/* reads n bf16 values from the file into a fresh device buffer */
static int upload(FILE *f, size_t n, void **dev) {
  uint16_t *host = (uint16_t *)malloc(n * 2);
  if (!host || fread(host, 2, n, f) != n) { free(host); return 1; }
  if (hipMalloc(dev, n * 2) != hipSuccess || hipMemcpy(*dev, host, n * 2, hipMemcpyHostToDevice) != hipSuccess) { free(host); return 1; }
  free(host);
  return 0;
}

int main(int argc, char **argv) {
  if (argc != 3) { fprintf(stderr, "usage: %s <input> <output>\n", argv[0]); return 1; }
  FILE *f = fopen(argv[1], "rb");
  int32_t hd[7];
  if (!f || fread(hd, 4, 7, f) != 7) { fprintf(stderr, "cannot read %s\n", argv[1]); return 1; }
  ff_shape shape = {hd[0], hd[1], hd[2], hd[3], hd[4], hd[5]};
  const int32_t k = hd[6];
  const size_t dm = (size_t)shape.d_model, df = (size_t)shape.d_ffn, T = (size_t)shape.n_tokens;
  const int32_t n_blocks = (shape.n_tokens + shape.block - 1) / shape.block;

  HIP_OK(hipSetDevice(0));
  void *x, *wg, *wu, *wd, *w1, *w2, *wc1, *wc2;
  if (upload(f, T * dm, &x) || upload(f, df * dm, &wg) || upload(f, df * dm, &wu) || upload(f, df * dm, &wd) ||
      upload(f, dm * shape.r_pred, &w1) || upload(f, (size_t)shape.r_pred * df, &w2) ||
      upload(f, (size_t)shape.r_comp * dm, &wc1) || upload(f, (size_t)shape.r_comp * dm, &wc2)) {
    fprintf(stderr, "short input file or out of device memory\n");
    return 1;
  }
  fclose(f);

  ff_ctx *ctx = NULL;
  FF_CHECK(ff_create(&ctx, 0, NULL));
  size_t ws_bytes = 0;
  FF_CHECK(ff_workspace_bytes(&shape, k, &ws_bytes));
  void *ws = NULL, *y = NULL;
  int32_t *idx = NULL;
  HIP_OK(hipMalloc(&ws, ws_bytes));
  HIP_OK(hipMalloc((void **)&idx, (size_t)n_blocks * k * 4));
  HIP_OK(hipMalloc(&y, T * dm * 4));
  FF_CHECK(ff_set_workspace(ctx, ws, ws_bytes));

  int32_t *ks = (int32_t *)malloc((size_t)n_blocks * 4);
  for (int32_t b = 0; b < n_blocks; ++b) ks[b] = k;
  ff_predictor pred = {NULL, w1, w2};
  ff_ffn_weights w = {wg, wu, wd};
  ff_compensator comp = {wc1, wc2, FF_ACT_SILU};
  FF_CHECK(ff_predict(ctx, &shape, x, &pred, ks, k, idx, NULL));
  FF_CHECK(ff_sparse_ffn(ctx, &shape, x, &w, &comp, idx, ks, k, y, FF_OUT_F32));
  HIP_OK(hipDeviceSynchronize());

  int32_t *idx_h = (int32_t *)malloc((size_t)n_blocks * k * 4);
  float *y_h = (float *)malloc(T * dm * 4);
  HIP_OK(hipMemcpy(idx_h, idx, (size_t)n_blocks * k * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(y_h, y, T * dm * 4, hipMemcpyDeviceToHost));
  FILE *o = fopen(argv[2], "wb");
  if (!o || fwrite(idx_h, 4, (size_t)n_blocks * k, o) != (size_t)n_blocks * k || fwrite(y_h, 4, T * dm, o) != T * dm) {
    fprintf(stderr, "cannot write %s\n", argv[2]);
    return 1;
  }
  fclose(o);
  FF_CHECK(ff_destroy(ctx));
  printf("ok: %d blocks of %d tokens, %d of %d neurons kept\n", n_blocks, shape.block, k, shape.d_ffn);
  return 0;
}

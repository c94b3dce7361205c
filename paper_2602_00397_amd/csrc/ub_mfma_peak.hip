// Stand-alone microbenchmark (not part of the library): the sustained rate of
// v_mfma_f32_32x32x16_bf16 with register operands only, on all-zero, random and small-valued
// bf16 data, at one and two wavefronts per SIMD.  It calibrates what "MFMA-bound" can mean on
// a given box: the clock under matrix load depends on the operand values.
//   hipcc --offload-arch=gfx950 -O3 -o ub_mfma_peak ub_mfma_peak.hip && ./ub_mfma_peak
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstdint>
#include <vector>
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("hip error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)

template <int NACC>
__global__ __launch_bounds__(512) void mfma_loop(const u32x4_t *in, float *out, int iters) {
  const int lane = threadIdx.x & 63;
  u32x4_t a[4], b[4];
  for (int i = 0; i < 4; ++i) { a[i] = in[(i * 64 + lane)]; b[i] = in[((4 + i) * 64 + lane)]; }
  f32x16_t acc[NACC];
  for (int i = 0; i < NACC; ++i) for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < NACC; ++i)
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a[i & 3]), __builtin_bit_cast(bf16x8_t, b[(i >> 2) & 3]), acc[i], 0, 0, 0);
  }
  float s = 0.f;
  for (int i = 0; i < NACC; ++i) for (int e = 0; e < 16; ++e) s += acc[i][e];
  if (s == 12345.678f) out[0] = s;
}

template <int NACC>
void run(const char *name, const u32x4_t *din, float *dout, int threads, int wgs, int iters) {
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  mfma_loop<NACC><<<wgs, threads>>>(din, dout, iters);
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0));
  for (int r = 0; r < 5; ++r) mfma_loop<NACC><<<wgs, threads>>>(din, dout, iters);
  CK(hipEventRecord(e1)); CK(hipDeviceSynchronize());
  float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ms /= 5;
  double flops = 2.0 * 32 * 32 * 16 * (double)NACC * iters * (threads / 64) * wgs;
  printf("%-40s threads %d wgs %d iters %d: %.3f ms  %.1f TFLOP/s\n", name, threads, wgs, iters, ms, flops / ms / 1e9);
  fflush(stdout);
}

int main() {
  std::vector<uint32_t> h(8 * 64 * 4);
  u32x4_t *din; float *dout;
  CK(hipMalloc(&din, h.size() * 4)); CK(hipMalloc(&dout, 64));
  for (int mode = 0; mode < 3; ++mode) {
    srand(1);
    for (auto &v : h) {
      if (mode == 0) v = 0;
      else if (mode == 1) {  // random bf16 in [-1,1): random mantissa/sign, exponent 126..119
        auto r = []() { uint32_t m = rand() & 0x7f, s = rand() & 1, e = 126 - (rand() % 6); return (s << 15) | (e << 7) | m; };
        v = r() | (r() << 16);
      } else {  // small weights-like values ~0.02
        auto r = []() { uint32_t m = rand() & 0x7f, s = rand() & 1, e = 121 - (rand() % 3); return (s << 15) | (e << 7) | m; };
        v = r() | (r() << 16);
      }
    }
    CK(hipMemcpy(din, h.data(), h.size() * 4, hipMemcpyHostToDevice));
    const char *mn[] = {"zeros", "random[-1,1)", "small"};
    printf("== data %s\n", mn[mode]);
    run<8>("8 acc, 1 wave/SIMD", din, dout, 256, 256 * 4, 20000);
    run<8>("8 acc, 2 waves/SIMD", din, dout, 512, 256 * 4, 10000);
    run<4>("4 acc, 2 waves/SIMD", din, dout, 512, 256 * 4, 20000);
  }
  return 0;
}

// Stand-alone microbenchmark (not part of the library): gather of whole 128-byte lines at random
// places of a region that fits L2 (2-3 MiB), the Infinity Cache (64 MiB) or neither (512 MiB),
// (0) with ordinary loads into VGPRs, (1) with global_load_lds_dwordx4 straight into LDS; U
// wave-loads per batch, two batches in flight.  It shows what the GEMMs' operand path can deliver.
//   hipcc --offload-arch=gfx950 -O3 -o ub_load_path ub_load_path.hip && ./ub_load_path
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
#include <cstdlib>
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("hip error %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)

__device__ __forceinline__ uint32_t hash32(uint32_t x) { x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16; return x; }

template <int MODE, int U>
__global__ __launch_bounds__(256) void ld(const uint8_t *__restrict__ buf, uint32_t n_lines, int iters, uint32_t *out) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t seed = (blockIdx.x * 4 + wave) * 0x9e3779b9u;
  u32x4 acc = {0, 0, 0, 0};
  const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) uint8_t *)smem + wave * (U * 2 * 1024);
  for (int it = 0; it < iters; ++it) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t line = hash32(seed + (it * U + u) * 8 + (lane >> 3)) % n_lines;
      const uint8_t *p = buf + (size_t)line * 128 + (lane & 7) * 16;
      if (MODE == 0) {
        v[u] = *reinterpret_cast<const u32x4 *>(p);
      } else {
        const uint32_t dst = lds_base + ((it & 1) * U + u) * 1024;
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(p), "s"(dst) : "memory");
      }
    }
    if (MODE == 0) {
#pragma unroll
      for (int u = 0; u < U; ++u) acc ^= v[u];
    } else {
      asm volatile("s_waitcnt vmcnt(%0)" : : "n"(U) : "memory");   // previous batch landed, this one in flight
    }
  }
  if (MODE == 1) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    acc = *reinterpret_cast<u32x4 *>(smem + threadIdx.x * 16);
  }
  if (acc.x == 0x12345678u) out[0] = acc.y ^ acc.z ^ acc.w;
}

template <int MODE, int U>
void run(const char *name, const uint8_t *buf, uint32_t n_lines, uint32_t *out, int wgs) {
  const int iters = 4096 / U;
  const size_t lds = 4 * U * 2 * 1024;
  CK(hipFuncSetAttribute(reinterpret_cast<const void *>(&ld<MODE, U>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
  ld<MODE, U><<<wgs, 256, lds>>>(buf, n_lines, iters, out);
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(a));
  for (int r = 0; r < 3; ++r) ld<MODE, U><<<wgs, 256, lds>>>(buf, n_lines, iters, out);
  CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
  float ms; CK(hipEventElapsedTime(&ms, a, b)); ms /= 3;
  const double bytes = (double)wgs * 4 * iters * U * 1024;
  printf("%-28s U=%2d wgs %4d region %6u KiB: %.3f ms  %.2f TB/s\n", name, U, wgs, n_lines / 8, ms, bytes / ms / 1e9);
  fflush(stdout);
}

int main() {
  uint8_t *buf; uint32_t *out;
  const size_t cap = 512u << 20;
  CK(hipMalloc(&buf, cap)); CK(hipMemset(buf, 1, cap)); CK(hipMalloc(&out, 64));
  for (uint32_t kib : {2048u, 3072u, 65536u, 524288u}) {
    const uint32_t n_lines = kib * 8;
    for (int wgs : {512, 1024}) {
      run<0, 4>("regs", buf, n_lines, out, wgs);
      run<0, 8>("regs", buf, n_lines, out, wgs);
      run<0, 16>("regs", buf, n_lines, out, wgs);
      run<1, 4>("global_load_lds", buf, n_lines, out, wgs);
      run<1, 8>("global_load_lds", buf, n_lines, out, wgs);
      run<1, 16>("global_load_lds", buf, n_lines, out, wgs);
    }
  }
  return 0;
}

// Layer-stack glue around the FFN path (pre-norm residual stack) and the index
// list validator.  All HBM-bound, one pass over the data each.
#include "ff_internal.h"

namespace {

// x_t = bf16(h_t / sqrt(mean(h_t^2) + eps)), gain 1; one wavefront per token,
// statistics in float64 with a fixed reduction order.
__global__ __launch_bounds__(256) void ff_rmsnorm_kernel(const bf16_t *__restrict__ h,
                                                         bf16_t *__restrict__ x, int T, int d_model,
                                                         float eps) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + wave;
  if (t >= T) return;
  const bf16_t *row = h + (size_t)t * d_model;
  double ss = 0.0;
  for (int c = lane * 8; c < d_model; c += 512) {
    const uint4 v = *reinterpret_cast<const uint4 *>(row + c);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const double a = (double)__uint_as_float(w[j] << 16), b = (double)__uint_as_float(w[j] & 0xffff0000u);
      ss = fma(a, a, ss);
      ss = fma(b, b, ss);
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  const double inv = 1.0 / sqrt(ss / (double)d_model + (double)eps);
  bf16_t *orow = x + (size_t)t * d_model;
  for (int c = lane * 8; c < d_model; c += 512) {
    const uint4 v = *reinterpret_cast<const uint4 *>(row + c);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const double a = (double)__uint_as_float(w[j] << 16), b = (double)__uint_as_float(w[j] & 0xffff0000u);
      o[j] = pack_bf16x2((float)(a * inv), (float)(b * inv));
    }
    *reinterpret_cast<uint4 *>(orow + c) = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

// The same for d_model <= 512 * NCH with the token's row held in registers: one read, all loads in
// flight at once.
template <int NCH>
__global__ __launch_bounds__(256) void ff_rmsnorm_reg_kernel(const bf16_t *__restrict__ h,
                                                             bf16_t *__restrict__ x, int T, int d_model,
                                                             float eps) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + wave;
  if (t >= T) return;
  const bf16_t *row = h + (size_t)t * d_model;
  uint4 v[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane * 8 + i * 512;
    v[i] = c < d_model ? *reinterpret_cast<const uint4 *>(row + c) : make_uint4(0, 0, 0, 0);
  }
  double ss = 0.0;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {          // same order of additions as the two-pass kernel
    const uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
    if (lane * 8 + i * 512 < d_model) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const double a = (double)__uint_as_float(w[j] << 16), b = (double)__uint_as_float(w[j] & 0xffff0000u);
        ss = fma(a, a, ss);
        ss = fma(b, b, ss);
      }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  const double inv = 1.0 / sqrt(ss / (double)d_model + (double)eps);
  bf16_t *orow = x + (size_t)t * d_model;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane * 8 + i * 512;
    if (c < d_model) {
      const uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
      uint32_t o[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const double a = (double)__uint_as_float(w[j] << 16), b = (double)__uint_as_float(w[j] & 0xffff0000u);
        o[j] = pack_bf16x2((float)(a * inv), (float)(b * inv));
      }
      *reinterpret_cast<uint4 *>(orow + c) = make_uint4(o[0], o[1], o[2], o[3]);
    }
  }
}

// h = bf16(h + y), 8 elements per thread
__global__ __launch_bounds__(256) void ff_residual_kernel(bf16_t *__restrict__ h,
                                                          const bf16_t *__restrict__ y, size_t n8) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n8) return;
  const uint4 a = reinterpret_cast<const uint4 *>(h)[i], b = reinterpret_cast<const uint4 *>(y)[i];
  const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
  uint32_t o[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
    o[j] = pack_bf16x2(__uint_as_float(aw[j] << 16) + __uint_as_float(bw[j] << 16),
                       __uint_as_float(aw[j] & 0xffff0000u) + __uint_as_float(bw[j] & 0xffff0000u));
  reinterpret_cast<uint4 *>(h)[i] = make_uint4(o[0], o[1], o[2], o[3]);
}

// plain copy, 16 bytes per thread (also the calibration kernel for the HBM byte counters)
__global__ __launch_bounds__(256) void ff_copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src, size_t n16) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) dst[i] = src[i];
}

// one workgroup per block: entries [0,K) strictly ascending in [0,d_ffn), entries [K,k_stride) == -1
__global__ __launch_bounds__(256) void ff_validate_kernel(const int32_t *__restrict__ idx, int k_stride,
                                                          KSpec ks, int d_ffn, int32_t *flag) {
  const int b = blockIdx.x;
  const int32_t *row = idx + (size_t)b * k_stride;
  int K = ks.per_block ? ks.per_block[b] : ks.uniform;
  bool bad = false;
  for (int i = threadIdx.x; i < k_stride; i += 256) {
    const int v = row[i];
    if (i < K) {
      if (v < 0 || v >= d_ffn) bad = true;
      if (i > 0 && row[i - 1] >= v) bad = true;
    } else if (v != -1) {
      bad = true;
    }
  }
  if (bad) atomicMax(flag, b + 1);
}

// ---- lists of g neighbouring short blocks merged into one list per group of g blocks --------------
// One workgroup of 1024 threads per group.  A byte per neuron in LDS collects which of the group's
// blocks selected it (bit s = block g * group + s); the neurons with a non-zero byte, in ascending order,
// are the group's list, their bytes its membership masks.  Entries of a list beyond its K, negative or
// out of range are ignored.
__global__ __launch_bounds__(1024) void ff_merge_lists_kernel(const int32_t *__restrict__ idx, int k_stride, KSpec ks,
                                                              int n_blocks, int g, int d_ffn,
                                                              int32_t *__restrict__ u_idx, uint8_t *__restrict__ u_mask,
                                                              int u_stride, int32_t *__restrict__ u_k) {
  extern __shared__ uint32_t member[];                  // d_ffn bytes, four neurons per word
  __shared__ int wsum[17];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int vb = blockIdx.x;
  const int n_words = (d_ffn + 3) / 4;
  for (int i = tid; i < n_words; i += 1024) member[i] = 0u;
  __syncthreads();
  for (int s = 0; s < g; ++s) {
    const int b = vb * g + s;
    if (b >= n_blocks) break;
    int K = ks.per_block ? ks.per_block[b] : ks.uniform;
    K = max(1, min(K, min(d_ffn, k_stride)));
    const int32_t *row = idx + (size_t)b * k_stride;
    for (int i0 = tid; i0 < K; i0 += 8 * 1024) {          // eight entries per thread in flight
      int n[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) n[u] = row[min(i0 + u * 1024, K - 1)];
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (i0 + u * 1024 < K && n[u] >= 0 && n[u] < d_ffn) atomicOr(&member[n[u] >> 2], 1u << (8 * (n[u] & 3) + s));
    }
  }
  __syncthreads();
  // thread t owns the words [t * per, (t + 1) * per): count, scan over the workgroup, write in order
  const int per = (n_words + 1023) / 1024;
  const int w0 = tid * per, w1 = min(n_words, w0 + per);
  int cnt = 0;
  for (int w = w0; w < w1; ++w) {
    const uint32_t m = member[w];
    cnt += ((m & 0xffu) != 0) + ((m & 0xff00u) != 0) + ((m & 0xff0000u) != 0) + ((m >> 24) != 0);
  }
  int inc = cnt;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __shfl_up(inc, d);
    if (lane >= d) inc += t;
  }
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int w = 0; w < 16; ++w) { const int t = wsum[w]; wsum[w] = run; run += t; }
    wsum[16] = run;
  }
  __syncthreads();
  int pos = wsum[wave] + inc - cnt;
  int32_t *out = u_idx + (size_t)vb * u_stride;
  uint8_t *outm = u_mask + (size_t)vb * u_stride;
  for (int w = w0; w < w1; ++w) {
    const uint32_t m = member[w];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t bits = (m >> (8 * q)) & 0xffu;
      if (bits != 0 && pos < u_stride) {
        out[pos] = 4 * w + q;
        outm[pos] = (uint8_t)bits;
        ++pos;
      }
    }
  }
  if (tid == 0) u_k[vb] = min(wsum[16], u_stride);
}

}  // namespace

hipError_t ff_launch_merge_lists(const int32_t *idx, int k_stride, KSpec ks, int n_blocks, int g, int d_ffn,
                                 int32_t *u_idx, uint8_t *u_mask, int u_stride, int32_t *u_k, int lds_limit,
                                 hipStream_t s) {
  static int raised = 0;
  const size_t lds = (size_t)((d_ffn + 3) / 4) * 4;
  if (lds + 256 > (size_t)lds_limit) return hipErrorInvalidValue;
  if (!raised) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(ff_merge_lists_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_limit - 256);
    if (e != hipSuccess) return e;
    raised = 1;
  }
  const int n_groups = (n_blocks + g - 1) / g;
  hipLaunchKernelGGL(ff_merge_lists_kernel, dim3(n_groups), dim3(1024), lds, s, idx, k_stride, ks, n_blocks, g, d_ffn,
                     u_idx, u_mask, u_stride, u_k);
  return hipGetLastError();
}

hipError_t ff_launch_rmsnorm(const bf16_t *h, bf16_t *x, int T, int d_model, float eps, hipStream_t s) {
  if (d_model <= 512 * 8)
    hipLaunchKernelGGL(ff_rmsnorm_reg_kernel<8>, dim3((T + 3) / 4), dim3(256), 0, s, h, x, T, d_model, eps);
  else if (d_model <= 512 * 16)
    hipLaunchKernelGGL(ff_rmsnorm_reg_kernel<16>, dim3((T + 3) / 4), dim3(256), 0, s, h, x, T, d_model, eps);
  else
    hipLaunchKernelGGL(ff_rmsnorm_kernel, dim3((T + 3) / 4), dim3(256), 0, s, h, x, T, d_model, eps);
  return hipGetLastError();
}

hipError_t ff_launch_residual(bf16_t *h, const bf16_t *y, size_t n, hipStream_t s) {
  const size_t n8 = n / 8;
  hipLaunchKernelGGL(ff_residual_kernel, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, s, h, y, n8);
  return hipGetLastError();
}

// ---- what the matrix pipes sustain with nothing else going on --------------------------------
// A register-only loop of v_mfma_f32_32x32x16_bf16 over 8 independent accumulators, two wavefronts
// per SIMD over the whole chip.  Operands are either zero or pseudo-random bf16 of magnitude 1/2..1
// (the clock the chip holds under this load depends on how many bits toggle), built in registers.
namespace {
typedef __attribute__((ext_vector_type(8))) __bf16 pk_bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float pk_f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t pk_u32x4_t;
constexpr int kPeakGrid = 1024, kPeakThreads = 512, kPeakAcc = 8;

__device__ __forceinline__ uint32_t peak_hash(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

__global__ __launch_bounds__(kPeakThreads) __attribute__((amdgpu_waves_per_eu(2)))
void ff_mfma_peak_kernel(int iters, int zero_operands, float *sink) {
  pk_u32x4_t a[2], b[4];
  const uint32_t id = blockIdx.x * kPeakThreads + threadIdx.x;
#pragma unroll
  for (int i = 0; i < 6; ++i) {
    pk_u32x4_t v;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t h = peak_hash(id * 24u + i * 4u + j);
      // two bf16 per dword: random sign and mantissa, exponent of 1/2
      v[j] = zero_operands ? 0u : ((h & 0x807f807fu) | 0x3f003f00u);
    }
    if (i < 2) a[i] = v; else b[i - 2] = v;
  }
  pk_f32x16_t acc[kPeakAcc];
#pragma unroll
  for (int m = 0; m < kPeakAcc; ++m)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[m][e] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < kPeakAcc; ++m)
      acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(pk_bf16x8_t, a[m & 1]),
                                                       __builtin_bit_cast(pk_bf16x8_t, b[m >> 1]), acc[m], 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int m = 0; m < kPeakAcc; ++m)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[m][e];
  if (s == 12345.6789f) sink[0] = s;   // keeps the loop alive; practically never taken
}
}  // namespace

hipError_t ff_launch_mfma_peak(int iters, int zero_operands, float *sink, double *flops, hipStream_t s) {
  hipLaunchKernelGGL(ff_mfma_peak_kernel, dim3(kPeakGrid), dim3(kPeakThreads), 0, s, iters, zero_operands, sink);
  *flops = (double)kPeakGrid * (kPeakThreads / 64) * (double)iters * kPeakAcc * (2.0 * 32 * 32 * 16);
  return hipGetLastError();
}

hipError_t ff_launch_copy(void *dst, const void *src, size_t bytes, hipStream_t s) {
  const size_t n16 = bytes / 16;
  hipLaunchKernelGGL(ff_copy_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, s,
                     static_cast<uint4 *>(dst), static_cast<const uint4 *>(src), n16);
  return hipGetLastError();
}

hipError_t ff_launch_validate(const int32_t *idx, int n_blocks, int k_stride, KSpec k, int d_ffn,
                              int32_t *flag, hipStream_t s) {
  hipLaunchKernelGGL(ff_validate_kernel, dim3(n_blocks), dim3(256), 0, s, idx, k_stride, k, d_ffn, flag);
  return hipGetLastError();
}

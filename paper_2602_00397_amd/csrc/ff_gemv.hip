// Few-token path of the sparse FFN (Eq. 15-18, 20-21 for prompts of at most kGemvMaxTokens
// tokens: the generation-time regime, where a block is a handful of tokens or a single one).
// With so few rows the work is a gather of 3 K weight rows per block read exactly once, i.e.
// bound by HBM, and the MFMA tiles of the prefill kernels would leave most of the chip idle
// (one block gives the down GEMM only d_model / 512 workgroups).  Three plain-ALU kernels:
//   gemv1: H[t][p] = bf16( SiLU(x_t . Wgate[r]) * (x_t . Wup[r]) ), r = idx_b[p]   (p <  K_b)
//          H[t][p] = bf16( act(x_t . Wc1[p - K_b]) )                                (compensator units)
//          one wavefront per list position, the lanes split d_model, fixed-order lane reduction;
//   gemv2: partial Y over a chunk of list positions for 256 output columns per wavefront
//          (split along the list so that one block still fills the chip), fp32;
//   gemv3: Y[t] = sum of the chunk partials in a fixed order, rounded once (or added to the
//          residual stream).
// Same rounding points as the prefill kernels (H in bf16, fp32 accumulation); every reduction has
// a fixed order, so results are reproducible.
#include "ff_internal.h"

namespace {

constexpr int kMaxPosPerWg = 32;   // gemv1: most list positions per workgroup (8 per wavefront)

// list length of block b; without a list (dense: position p is row p) the pitch does not bound it
__device__ __forceinline__ int gv_block_k(const GemvParams &p, int b) {
  int K = p.k.per_block ? p.k.per_block[b] : p.k.uniform;
  K = max(1, min(K, p.d_ffn));
  return p.idx ? min(K, p.k_stride) : K;
}
__device__ __forceinline__ int gv_row(const int32_t *list, int pos, int d_ffn) {
  return min(max(list ? list[pos] : pos, 0), d_ffn - 1);
}
__device__ __forceinline__ float gv_act(int act, float g) {
  if (act == FF_ACT_SILU) return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g));
  if (act == FF_ACT_RELU) return fmaxf(g, 0.0f);
  return g;
}
__device__ __forceinline__ void unpack8(const uint4 &v, float (&f)[8]) {
  f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
  f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
  f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
  f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
}
// sum over the 64 lanes in a fixed butterfly order; every lane ends with the total
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// grid (ceil(max list length / pos_per_wg), n_blocks), 256 or 1024 threads, LDS = nt * d_model bf16
__global__ __launch_bounds__(1024) void ff_gemv1_kernel(GemvParams p) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
  const int b = blockIdx.y;
  const int t0 = b * p.block;
  const int nt = min(p.T, t0 + p.block) - t0;          // <= kGemvMaxTokens by the launcher's check
  const int Kb = gv_block_k(p, b);
  const int ntot = Kb + p.rc;
  const int pos0 = blockIdx.x * p.pos_per_wg;
  if (pos0 >= ntot) return;
  // the block's tokens, as they are
  const uint4 *xg = reinterpret_cast<const uint4 *>(p.x + (size_t)t0 * p.d_model);
  uint4 *xs = reinterpret_cast<uint4 *>(smem);
  const int n16 = nt * (p.d_model / 8);
  for (int i = tid; i < n16; i += blockDim.x) xs[i] = xg[i];
  __syncthreads();
  const int32_t *list = p.idx ? p.idx + (size_t)b * p.k_stride : nullptr;
  for (int pp = wave; pp < p.pos_per_wg; pp += nw) {
    const int pos = pos0 + pp;
    if (pos >= ntot) break;
    const bool gated = pos < Kb;
    const uint32_t member = (p.mask != nullptr && gated) ? (uint32_t)p.mask[(size_t)b * p.k_stride + pos] : 0xffffffffu;
    const bf16_t *grow, *urow;
    if (gated) {
      const int r = gv_row(list, pos, p.d_ffn);
      grow = p.wg + (size_t)r * p.d_model;
      urow = p.wu + (size_t)r * p.d_model;
    } else {
      grow = urow = p.wc1 + (size_t)(pos - Kb) * p.d_model;
    }
    float ag[kGemvMaxTokens], au[kGemvMaxTokens];
#pragma unroll
    for (int t = 0; t < kGemvMaxTokens; ++t) { ag[t] = 0.0f; au[t] = 0.0f; }
    // lanes take 8-element chunks l, l + 64, ...; four chunks of each matrix in flight
    for (int c0 = lane * 8; c0 < p.d_model; c0 += 4 * 512) {
      uint4 gv[4], uv[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = c0 + j * 512;
        const bool in = c < p.d_model;
        gv[j] = in ? *reinterpret_cast<const uint4 *>(grow + c) : make_uint4(0, 0, 0, 0);
        uv[j] = (in && gated) ? *reinterpret_cast<const uint4 *>(urow + c) : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = c0 + j * 512;
        if (c < p.d_model) {
          float gf[8], uf[8];
          unpack8(gv[j], gf);
          unpack8(uv[j], uf);
#pragma unroll
          for (int t = 0; t < kGemvMaxTokens; ++t)
            if (t < nt) {
              float xf[8];
              unpack8(xs[t * (p.d_model / 8) + c / 8], xf);
#pragma unroll
              for (int e = 0; e < 8; ++e) {
                ag[t] = fmaf(gf[e], xf[e], ag[t]);
                au[t] = fmaf(uf[e], xf[e], au[t]);
              }
            }
        }
      }
    }
#pragma unroll
    for (int t = 0; t < kGemvMaxTokens; ++t)
      if (t < nt) {
        const float g = wave_sum(ag[t]);
        const float u = wave_sum(au[t]);
        if (lane == 0) {
          float hv = gated ? gv_act(FF_ACT_SILU, g) * u : gv_act(p.comp_act, g);
          if (p.mask != nullptr && !((member >> (t / p.sub_block)) & 1u)) hv = 0.0f;   // not selected for this token
          p.h[(size_t)(t0 + t) * p.hs + pos] = f32_to_bf16(hv);
        }
      }
  }
}

// grid (ceil(column groups / 4), n_chunks, n_blocks), 256 threads: a wavefront owns a group of
// NV * 512 output columns (NV units of 512, a lane holding 8 adjacent columns of each) for at most
// NT tokens and walks its chunk of the list, two groups of U weight rows in flight; nothing is shared
// between the wavefronts, so there is no barrier.  Wider groups read longer contiguous pieces of a
// gathered row; they cost NT * NV * 8 accumulators, hence fewer tokens.
template <int NV, int NT, int U>
__global__ __launch_bounds__(256) void ff_gemv2_kernel(GemvParams p) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.z, ch = blockIdx.y;
  const int t0 = b * p.block;
  const int nt = min(min(p.T, t0 + p.block) - t0, NT);
  const int Kb = gv_block_k(p, b);
  const int ntot = Kb + p.rc;
  const int cl = ((ntot + p.n_chunks - 1) / p.n_chunks + 7) / 8 * 8;   // chunk length
  const int pb = ch * cl, pe = min(ntot, pb + cl);
  const int col0 = (blockIdx.x * 4 + wave) * (NV * 512) + lane * 8;
  if (col0 - lane * 8 >= p.d_model) return;
  // d_model is a multiple of 8, so a lane's 8 columns of a unit are in or out together; a unit that is
  // out reads the last 8 columns instead and stores nothing
  int colj[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) colj[j] = min(col0 + j * 512, p.d_model - 8);
  const int32_t *list = p.idx ? p.idx + (size_t)b * p.k_stride : nullptr;
  // lane t < nt reads token t's H values; the other lanes' values are never used
  const bf16_t *hrow = p.h + (size_t)(t0 + min(lane, nt - 1)) * p.hs;
  float acc[NT][NV][8];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int j = 0; j < NV; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[t][j][e] = 0.0f;
  // Loads never branch: a position past the chunk's end re-reads the last row and its H value
  // counts as zero.  Two groups of U rows alternate, so that the next group's rows are on their
  // way while this one is multiplied.
  const int last = pe - 1;
  auto load = [&](int q0, uint4 (&wv)[U][NV], bf16_t (&hv)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int pos = min(q0 + u, last);
      const bf16_t *row = pos < Kb ? p.wd + (size_t)gv_row(list, pos, p.d_ffn) * p.d_model
                                   : p.wc2 + (size_t)(pos - Kb) * p.d_model;
#pragma unroll
      for (int j = 0; j < NV; ++j) wv[u][j] = *reinterpret_cast<const uint4 *>(row + colj[j]);
      hv[u] = hrow[pos];
    }
  };
  auto fma_rows = [&](int q0, const uint4 (&wv)[U][NV], const bf16_t (&hv)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float hm = q0 + u < pe ? bf16_to_f32(hv[u]) : 0.0f;
      float hs[NT];
#pragma unroll
      for (int t = 0; t < NT; ++t) hs[t] = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(hm), t));
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        float wf[8];
        unpack8(wv[u][j], wf);
#pragma unroll
        for (int t = 0; t < NT; ++t)
          if (t < nt) {
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[t][j][e] = fmaf(hs[t], wf[e], acc[t][j][e]);
          }
      }
    }
  };
  if (pb < pe) {
    uint4 wa[U][NV], wb[U][NV];
    bf16_t ha[U], hb[U];
    load(pb, wa, ha);
    for (int q0 = pb; q0 < pe; q0 += 2 * U) {
      load(q0 + U, wb, hb);
      fma_rows(q0, wa, ha);
      load(q0 + 2 * U, wa, ha);
      fma_rows(q0 + U, wb, hb);
    }
  }
#pragma unroll
  for (int t = 0; t < NT; ++t)
    if (t < nt) {
#pragma unroll
      for (int j = 0; j < NV; ++j)
        if (col0 + j * 512 < p.d_model) {
          float *o = p.part + ((size_t)ch * p.T + (t0 + t)) * p.d_model + col0 + j * 512;
          *reinterpret_cast<float4 *>(o) = make_float4(acc[t][j][0], acc[t][j][1], acc[t][j][2], acc[t][j][3]);
          *reinterpret_cast<float4 *>(o + 4) = make_float4(acc[t][j][4], acc[t][j][5], acc[t][j][6], acc[t][j][7]);
        }
    }
}

struct Gemv2Variant {
  void (*fn)(GemvParams);
  int nv, nt;
};
const Gemv2Variant kGemv2[] = {
    {ff_gemv2_kernel<1, 2, 8>, 1, 2},   // one or two tokens per block
    {ff_gemv2_kernel<2, 2, 8>, 2, 2},   // the same with four or more blocks: enough wavefronts for longer row pieces
    {ff_gemv2_kernel<1, 4, 4>, 1, 4},
    {ff_gemv2_kernel<1, 8, 4>, 1, 8},
};

// grid (ceil(d_model / 256), T), 1024 threads: wavefront w adds the chunks w, w + 16, ... for 256
// columns (4 per lane), then thread c < 256 adds the 16 wavefronts' sums for column c in order.
__global__ __launch_bounds__(1024) void ff_gemv3_kernel(GemvParams p) {
  __shared__ __align__(16) float red[16][256];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, t = blockIdx.y;
  const int col = blockIdx.x * 256 + lane * 4;
  float4 s4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  if (col < p.d_model) {
    constexpr int R = kGemvChunks / 16;
    float4 v[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const int ch = wave + 16 * j;
      v[j] = ch < p.n_chunks ? *reinterpret_cast<const float4 *>(p.part + ((size_t)ch * p.T + t) * p.d_model + col)
                             : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    }
#pragma unroll
    for (int j = 0; j < R; ++j) { s4.x += v[j].x; s4.y += v[j].y; s4.z += v[j].z; s4.w += v[j].w; }
  }
  *reinterpret_cast<float4 *>(&red[wave][lane * 4]) = s4;
  __syncthreads();
  const int c = blockIdx.x * 256 + tid;
  if (tid >= 256 || c >= p.d_model) return;
  float s = 0.0f;
#pragma unroll
  for (int w = 0; w < 16; ++w) s += red[w][tid];
  const size_t o = (size_t)t * p.d_model + c;
  if (p.res) {
    p.res[o] = f32_to_bf16(bf16_to_f32(p.res[o]) + bf16_to_f32(f32_to_bf16(s)));
  } else if (p.out_f32) {
    reinterpret_cast<float *>(p.y)[o] = s;
  } else {
    reinterpret_cast<bf16_t *>(p.y)[o] = f32_to_bf16(s);
  }
}

int g_gemv_lds_raised = 0;

}  // namespace

size_t ff_gemv_part_bytes(int n_tokens, int d_model) {
  return n_tokens <= kGemvMaxTokens ? (size_t)kGemvChunks * n_tokens * d_model * sizeof(float) : 0;
}

bool ff_gemv_eligible(int n_tokens, int block, int d_model, int lds_limit) {
  const int nt = block < n_tokens ? block : n_tokens;
  return n_tokens <= kGemvMaxTokens && (size_t)nt * d_model * 2 <= (size_t)lds_limit;
}

hipError_t ff_launch_gemv(const GemvParams &p_in, int lds_limit, hipStream_t s, Profiler *prof) {
  GemvParams p = p_in;
  if (!ff_gemv_eligible(p.T, p.block, p.d_model, lds_limit)) return hipErrorInvalidValue;
  if (!g_gemv_lds_raised) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(ff_gemv1_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_limit);
    if (e != hipSuccess) return e;
    g_gemv_lds_raised = 1;
  }
  const int nt = p.block < p.T ? p.block : p.T;
  const int n_extent = p.k.k_max + p.rc;
  // Both grids aim at about 2048 units of work (workgroups of gemv1, wavefronts of gemv2): eight
  // or more per compute unit, each with 4 to 16 KB of weight rows in flight, which is what it takes
  // to keep HBM busy from so few tokens.
  constexpr int kTarget = 2048;
  // gemv1 copies the block's tokens into LDS once per workgroup: with more than two tokens a
  // workgroup of 16 wavefronts shares that copy
  const int threads1 = nt > 2 ? 1024 : 256, nw1 = threads1 / 64;
  int ppw = (int)(((long)n_extent * p.n_blocks / kTarget) / nw1 * nw1);
  p.pos_per_wg = ppw < nw1 ? nw1 : (ppw > kMaxPosPerWg ? kMaxPosPerWg : ppw);
  // gemv2: chunks of at least 32 rows, so that a wavefront's row reads outweigh the fp32 partials
  // it writes (nt * 32 bytes per lane against 32 * 16)
  const int gv = nt <= 2 ? (p.n_blocks >= 4 ? 1 : 0) : nt <= 4 ? 2 : 3;
  const int col_groups = (p.d_model + kGemv2[gv].nv * 512 - 1) / (kGemv2[gv].nv * 512);
  int nc = kTarget / (col_groups * p.n_blocks);
  if (nc > n_extent / 32) nc = n_extent / 32;
  p.n_chunks = nc < 1 ? 1 : (nc > kGemvChunks ? kGemvChunks : nc);
  prof_begin(prof, FF_STAGE_GEMM1, s);
  hipLaunchKernelGGL(ff_gemv1_kernel, dim3((n_extent + p.pos_per_wg - 1) / p.pos_per_wg, p.n_blocks), dim3(threads1),
                     (size_t)nt * p.d_model * 2, s, p);
  prof_end(prof, s);
  prof_begin(prof, FF_STAGE_GEMM2, s);
  hipLaunchKernelGGL(kGemv2[gv].fn, dim3((col_groups + 3) / 4, p.n_chunks, p.n_blocks), dim3(256), 0, s, p);
  hipLaunchKernelGGL(ff_gemv3_kernel, dim3((p.d_model + 255) / 256, p.T), dim3(1024), 0, s, p);
  prof_end(prof, s);
  return hipGetLastError();
}

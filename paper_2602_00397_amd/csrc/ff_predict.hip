// Expert-neuron predictor (Sec. 3.2): pooling (Eq. 12), two-layer MLP (Eq. 13)
// and top-K selection (Eq. 14), all in float64 so that the selected set is the
// one the real-number scores define.  Every reduction has a fixed order, so
// results are bitwise reproducible from run to run.
#include "ff_internal.h"

namespace {

__device__ __forceinline__ void unpack8(const uint4 &v, double *o) {
  o[0] = (double)__uint_as_float(v.x << 16); o[1] = (double)__uint_as_float(v.x & 0xffff0000u);
  o[2] = (double)__uint_as_float(v.y << 16); o[3] = (double)__uint_as_float(v.y & 0xffff0000u);
  o[4] = (double)__uint_as_float(v.z << 16); o[5] = (double)__uint_as_float(v.z & 0xffff0000u);
  o[6] = (double)__uint_as_float(v.w << 16); o[7] = (double)__uint_as_float(v.w & 0xffff0000u);
}

// ---- Eq. 12, logits z_t = q . x_t / sqrt(d_model): one wavefront per token ----
__global__ __launch_bounds__(256) void ff_logits_kernel(const bf16_t *__restrict__ x,
                                                        const bf16_t *__restrict__ q,
                                                        double *__restrict__ z, int T, int d_model) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + wave;
  if (t >= T) return;
  const bf16_t *row = x + (size_t)t * d_model;
  double acc = 0.0;
  for (int c = lane * 8; c < d_model; c += 512) {
    double xv[8], qv[8];
    unpack8(*reinterpret_cast<const uint4 *>(row + c), xv);
    unpack8(*reinterpret_cast<const uint4 *>(q + c), qv);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc = fma(xv[j], qv[j], acc);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
  if (lane == 0) z[t] = acc / sqrt((double)d_model);
}

// ---- Eq. 12, a_b = sum_t p_t x_t over one block, and its share of Eq. 13's first layer ----
// grid (ceil(d_model/512), n_blocks), 256 threads: each lane owns 8 channels,
// the four wavefronts take every fourth token and are summed in wave order.  The workgroup
// then multiplies its 512 pooled channels into the first predictor layer, hpart[b][slice][j] =
// sum_{c in slice} a_b[c] W1[c][j]; the next kernel adds the slices in slice order.
template <bool SOFTMAX>
__global__ __launch_bounds__(256) void ff_pool_kernel(const bf16_t *__restrict__ x,
                                                      const double *__restrict__ z,
                                                      const bf16_t *__restrict__ w1,
                                                      double *__restrict__ hpart, int T,
                                                      int d_model, int Nb, int r) {
  extern __shared__ double p_s[];          // SOFTMAX: Nb weights
  __shared__ double red[4][512];
  __shared__ double red1[256];
  __shared__ double a_s[512];              // this workgroup's pooled channels
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int b = blockIdx.y;
  const int t0 = b * Nb;
  const int n = min(T, t0 + Nb) - t0;
  if (SOFTMAX) {
    double m = -INFINITY;
    for (int i = tid; i < n; i += 256) m = fmax(m, z[t0 + i]);
    red1[tid] = m;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
      if (tid < s) red1[tid] = fmax(red1[tid], red1[tid + s]);
      __syncthreads();
    }
    m = red1[0];
    for (int i = tid; i < n; i += 256) p_s[i] = exp(z[t0 + i] - m);
    __syncthreads();
    if (tid == 0) {
      double s = 0.0;
      for (int i = 0; i < n; ++i) s += p_s[i];
      red1[1] = s;
    }
    __syncthreads();
    const double s = red1[1];
    for (int i = tid; i < n; i += 256) p_s[i] = p_s[i] / s;
    __syncthreads();
  }
  const int c = blockIdx.x * 512 + lane * 8;
  double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (c < d_model) {
    const bf16_t *xc = x + (size_t)t0 * d_model + c;
    int i = wave;
    for (; i + 28 < n; i += 32) {          // 8 token rows in flight, added in token order
      uint4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const uint4 *>(xc + (size_t)(i + 4 * u) * d_model);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        double xv[8];
        unpack8(v[u], xv);
        if (SOFTMAX) {
          const double w = p_s[i + 4 * u];
#pragma unroll
          for (int j = 0; j < 8; ++j) acc[j] = fma(w, xv[j], acc[j]);
        } else {
#pragma unroll
          for (int j = 0; j < 8; ++j) acc[j] += xv[j];
        }
      }
    }
    for (; i < n; i += 4) {
      double xv[8];
      unpack8(*reinterpret_cast<const uint4 *>(xc + (size_t)i * d_model), xv);
      if (SOFTMAX) {
        const double w = p_s[i];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = fma(w, xv[j], acc[j]);
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += xv[j];
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) red[wave][lane * 8 + j] = acc[j];
  __syncthreads();
  for (int ch = tid; ch < 512; ch += 256) {
    const int cc = blockIdx.x * 512 + ch;
    double tot = 0.0;
    if (cc < d_model) {
      tot = ((red[0][ch] + red[1][ch]) + red[2][ch]) + red[3][ch];
      if (!SOFTMAX) tot = tot / (double)n;
    }
    a_s[ch] = tot;                       // channels past d_model count as zero
  }
  __syncthreads();
  // First layer over this slice: hpart[b][slice][j] = sum_c a_s[c] W1[c_base + c][j].
  const int c_base = blockIdx.x * 512;
  const int n_ch = min(512, d_model - c_base);
  const int n_slices = gridDim.x;
  double *dst = hpart + ((size_t)b * n_slices + blockIdx.x) * r;
  if ((r & 7) == 0) {
    // Thread (cl, o) takes the 8 outputs 8 o .. 8 o + 7 (one 16-byte load per channel) over the channels
    // cl, cl + CL, ... in ascending order, eight loads in flight; the CL partial sums of an output are then
    // added in cl order.
    const int n_oct = r >> 3;                                   // <= 128
    int o_ceil = 1;
    while (o_ceil < n_oct) o_ceil <<= 1;
    const int CL = 256 / o_ceil;                                // >= 2 channel lanes
    const int o = tid % o_ceil, cl = tid / o_ceil;
    double acc8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (o < n_oct) {
      const bf16_t *wp = w1 + (size_t)c_base * r + 8 * o;
      int cq = cl;
      for (; cq + 7 * CL < n_ch; cq += 8 * CL) {
        uint4 wv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) wv[u] = *reinterpret_cast<const uint4 *>(wp + (size_t)(cq + u * CL) * r);
        __builtin_amdgcn_sched_barrier(0);                      // all eight loads go out before the first use
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          double wd[8];
          unpack8(wv[u], wd);
          const double av = a_s[cq + u * CL];
#pragma unroll
          for (int q = 0; q < 8; ++q) acc8[q] = fma(av, wd[q], acc8[q]);
        }
      }
      for (; cq < n_ch; cq += CL) {
        double wd[8];
        unpack8(*reinterpret_cast<const uint4 *>(wp + (size_t)cq * r), wd);
        const double av = a_s[cq];
#pragma unroll
        for (int q = 0; q < 8; ++q) acc8[q] = fma(av, wd[q], acc8[q]);
      }
    }
    double *ps = &red[0][0];                                    // [CL][8 o_ceil] = 2048 doubles: red is free by now
#pragma unroll
    for (int q = 0; q < 8; ++q) ps[(cl * o_ceil + o) * 8 + q] = acc8[q];
    __syncthreads();
    for (int j = tid; j < r; j += 256) {
      double tot = 0.0;
      for (int q = 0; q < CL; ++q) tot += ps[q * o_ceil * 8 + j];
      dst[j] = tot;
    }
  } else {
    // any r: a thread per output, channels in ascending order
    for (int j = tid; j < r; j += 256) {
      const bf16_t *col = w1 + (size_t)c_base * r + j;
      double acc = 0.0;
      for (int cq = 0; cq < n_ch; ++cq) acc = fma(a_s[cq], (double)bf16_to_f32(col[(size_t)cq * r]), acc);
      dst[j] = acc;
    }
  }
}

// ---- Eq. 13 in float64 ---------------------------------------------------------------------
// The first layer (long contraction over d_model, few outputs) is cut into slices of 512 channels that
// ride along with the pooling kernel above; the second (short contraction, d_ffn outputs) takes MLP_BB
// blocks per workgroup so that every weight is loaded once per MLP_BB blocks, each thread keeping
// MLP_LD weight loads in flight.
constexpr int MLP_BB = 4;    // blocks per workgroup: 8 halves the weight loads but leaves too few wavefronts to hide the scalar loads
constexpr int MLP_LD = 16;   // rows of W2 a thread has in flight

// ---- Eq. 13, second layer with the hidden units formed on the way in -------------------------
// scores[b][n] = sum_j h_b[j] W2[j][n], h_b[j] = ReLU(sum_s hpart[b][s][j]) (slices added in slice order).
// grid (ceil(d_ffn / 1024), ceil(n_blocks / MLP_BB)), 256 threads: a workgroup first forms the r hidden units of its
// MLP_BB blocks in LDS (every workgroup of a block group repeats these few sums rather than wait for a launch of
// their own), then every thread owns four adjacent score columns and reads the hidden units as LDS broadcasts.
__global__ __launch_bounds__(256) void ff_scores_kernel(const double *__restrict__ hpart,
                                                        const bf16_t *__restrict__ w2,
                                                        double *__restrict__ scores, int n_blocks, int r,
                                                        int n_slices, int d_ffn) {
  extern __shared__ double hid[];          // [MLP_BB][r]
  const int tid = threadIdx.x;
  const int b0 = blockIdx.y * MLP_BB;
  const int nb = min(MLP_BB, n_blocks - b0);
  for (int e = tid; e < MLP_BB * r; e += 256) {
    const int i = e / r, j = e - i * r;
    double acc = 0.0;
    if (i < nb) {
      const double *src = hpart + (size_t)(b0 + i) * n_slices * r + j;
      int s = 0;
      for (; s + 8 <= n_slices; s += 8) {      // eight loads in flight, added in slice order
        double v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[(size_t)(s + u) * r];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u];
      }
      for (; s < n_slices; ++s) acc += src[(size_t)s * r];
    }
    hid[e] = fmax(acc, 0.0);
  }
  __syncthreads();
  // A hidden unit read from LDS (the same address in every lane) costs a full-width LDS access, and a
  // load instruction costs the same whether a lane asks for 2 bytes or 8: every thread takes four
  // adjacent score columns, one 8-byte load per row of W2 (d_ffn is a multiple of 8, so a group of
  // four columns is whole and aligned), and each hidden unit read feeds 4 x MLP_BB multiply-adds.
  const int n_quads = d_ffn >> 2;
  const int quad = (int)(blockIdx.x * 256) + tid;
  const int n0 = 4 * min(quad, n_quads - 1);               // past the end: the last group again, not stored
  double acc[4][MLP_BB];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int i = 0; i < MLP_BB; ++i) acc[q][i] = 0.0;
  const bf16_t *wp = w2 + n0;
  auto mac_row = [&](const uint2 &wv, int jrow) __attribute__((always_inline)) {
    const double wd[4] = {(double)__uint_as_float(wv.x << 16), (double)__uint_as_float(wv.x & 0xffff0000u),
                          (double)__uint_as_float(wv.y << 16), (double)__uint_as_float(wv.y & 0xffff0000u)};
    double hv[MLP_BB];
#pragma unroll
    for (int i = 0; i < MLP_BB; ++i) hv[i] = hid[i * r + jrow];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int i = 0; i < MLP_BB; ++i) acc[q][i] = fma(hv[i], wd[q], acc[q][i]);
  };
  int j = 0;
  for (; j + MLP_LD <= r; j += MLP_LD) {   // MLP_LD rows of W2 in flight
    uint2 wv[MLP_LD];
#pragma unroll
    for (int u = 0; u < MLP_LD; ++u) wv[u] = *reinterpret_cast<const uint2 *>(wp + (size_t)(j + u) * d_ffn);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < MLP_LD; ++u) mac_row(wv[u], j + u);
  }
  for (; j < r; ++j) mac_row(*reinterpret_cast<const uint2 *>(wp + (size_t)j * d_ffn), j);
  if (quad < n_quads) {
#pragma unroll
    for (int i = 0; i < MLP_BB; ++i)
      if (i < nb) {
        double *dst = scores + (size_t)(b0 + i) * d_ffn + n0;
        *reinterpret_cast<double2 *>(dst) = make_double2(acc[0][i], acc[1][i]);
        *reinterpret_cast<double2 *>(dst + 2) = make_double2(acc[2][i], acc[3][i]);
      }
  }
}

// ---- Eq. 14: top-K, one workgroup of 1024 threads per block -----------------------
// Scores become 64-bit keys whose unsigned order is the score order (-0 == +0).  The
// selected set is {key > theta} plus the lowest-index (K - count) keys equal to theta,
// where theta is the key of the K-th largest score; it is written in ascending index
// order through two prefix sums.  theta is found exactly in two steps: a histogram over
// 4096 buckets of a monotone map of the score range locates the bucket holding the K-th
// largest, then the few keys of that bucket are ranked against each other.  When that
// bucket holds too many keys (heavy ties) an 8-pass MSB-first radix select on the keys
// finds theta instead.
__device__ __forceinline__ unsigned long long score_key(double s) {
  s = s + 0.0;  // -0.0 -> +0.0
  unsigned long long u = (unsigned long long)__double_as_longlong(s);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}
__device__ __forceinline__ double key_score(unsigned long long k) {
  const unsigned long long u = (k >> 63) ? (k & 0x7fffffffffffffffull) : ~k;
  return __longlong_as_double((long long)u);
}

__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __shfl_up(v, d);
    if (lane >= d) v += t;
  }
  return v;
}

// exclusive prefix over the 1024 threads of the block; total returned too
__device__ __forceinline__ int block_excl_scan(int v, int *wsum, int &total) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int inc = wave_incl_scan(v, lane);
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  if (wave == 0) {
    const int w = lane < 16 ? wsum[lane] : 0;
    const int ws = wave_incl_scan(w, lane);
    if (lane < 16) wsum[lane] = ws - w;
    if (lane == 15) wsum[16] = ws;
  }
  __syncthreads();
  total = wsum[16];
  const int res = wsum[wave] + inc - v;
  __syncthreads();
  return res;
}

constexpr int TOPK_BUCKETS = 4096;
constexpr int TOPK_CAND = 1024;   // most keys the threshold bucket may hold for the ranking step

// LDS of the threshold search, shared by both top-K kernels
struct TopkShared {
  unsigned int hist[TOPK_BUCKETS];           // also the 256-bin histogram of the radix path
  unsigned long long cand[TOPK_CAND];
  int wsum[17];
  unsigned int wtot[4];
  unsigned int sel_bin, sel_rem, n_cand;
  unsigned long long theta;
  int ties;
};

// The key theta of the K-th largest score and the number of keys equal to theta that are kept, found
// exactly by the 1024 threads of a workgroup.  each(fn) calls fn(key) once for every key the calling thread
// owns.  [lo_v, hi_v] encloses the scores (it only shapes the bucket map); need_radix skips the buckets.
// On entry sh.hist is zero, sh.n_cand is 0 and a barrier has been passed.
template <class Each>
__device__ __forceinline__ void topk_threshold(TopkShared &sh, int K, double lo_v, double hi_v, bool need_radix,
                                               Each each, unsigned long long &theta, int &ties_taken) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const double scale = need_radix ? 0.0 : (double)TOPK_BUCKETS / (hi_v - lo_v);
  // monotone: s1 <= s2 implies bucket(s1) <= bucket(s2), so a key in a higher bucket is a larger key
  auto bucket_of = [&](unsigned long long k) -> int {
    const double t = (key_score(k) - lo_v) * scale;
    return min(TOPK_BUCKETS - 1, max(0, (int)t));
  };
  if (!need_radix) {
    each([&](unsigned long long k) { atomicAdd(&sh.hist[bucket_of(k)], 1u); });
    __syncthreads();
    // thread t owns buckets 4095-4t .. 4092-4t (descending); prefix over threads = keys in higher buckets
    int local = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) local += (int)sh.hist[TOPK_BUCKETS - 1 - (4 * tid + q)];
    int total;
    int above = block_excl_scan(local, sh.wsum, total);
    if (above < K && K <= above + local) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int bk = TOPK_BUCKETS - 1 - (4 * tid + q);
        const int h = (int)sh.hist[bk];
        if (above < K && K <= above + h) { sh.sel_bin = (unsigned int)bk; sh.sel_rem = (unsigned int)(K - above); }
        above += h;
      }
    }
    __syncthreads();
    const int tb = (int)sh.sel_bin;
    const int need = (int)sh.sel_rem;             // rank of theta inside bucket tb (1 = largest)
    const int c = (int)sh.hist[tb];
    if (c > TOPK_CAND) {
      need_radix = true;                          // uniform: every thread reads the same hist[tb]
    } else {
      each([&](unsigned long long k) {
        if (bucket_of(k) == tb) sh.cand[atomicAdd(&sh.n_cand, 1u)] = k;
      });
      __syncthreads();
      if (tid < c) {
        const unsigned long long mine = sh.cand[tid];
        int n_gt = 0, n_eq = 0;
        for (int j = 0; j < c; ++j) {
          const unsigned long long o = sh.cand[j];
          n_gt += o > mine;
          n_eq += o == mine;
        }
        // the need-th largest of the bucket: n_gt < need <= n_gt + n_eq (all holders of that key agree)
        if (n_gt < need && need <= n_gt + n_eq) { sh.theta = mine; sh.ties = need - n_gt; }
      }
      __syncthreads();
    }
  }
  if (need_radix) {
    // 8-pass MSB-first radix select on the keys themselves (heavy ties, or no ordered range)
    unsigned long long prefix = 0;  // digits decided so far (high part of theta)
    unsigned int rem = (unsigned int)K;
    for (int pass = 7; pass >= 0; --pass) {
      const int shift = pass * 8;
      __syncthreads();
      if (tid < 256) sh.hist[tid] = 0;
      __syncthreads();
      each([&](unsigned long long k) {
        const bool match = (pass == 7) || ((k >> (shift + 8)) == prefix);
        if (match) atomicAdd(&sh.hist[(unsigned int)(k >> shift) & 255u], 1u);
      });
      __syncthreads();
      // suffix sums S[d] = sum_{d' >= d} hist[d'] over the 256 digits
      unsigned int hv = 0, suf = 0;
      if (tid < 256) {
        hv = sh.hist[tid];
        suf = hv;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
          const unsigned int t = __shfl_down(suf, off);
          if (lane + off < 64) suf += t;
        }
        if (lane == 0) sh.wtot[wave] = suf;
      }
      __syncthreads();
      if (tid < 256) {
        for (int w = wave + 1; w < 4; ++w) suf += sh.wtot[w];
        // the digit of the K-th largest: S[d] >= rem > S[d+1]
        if (suf >= rem && suf - hv < rem) {
          sh.sel_bin = (unsigned int)tid;
          sh.sel_rem = rem - (suf - hv);
        }
      }
      __syncthreads();
      prefix = (prefix << 8) | (unsigned long long)sh.sel_bin;
      rem = sh.sel_rem;
    }
    if (tid == 0) { sh.theta = prefix; sh.ties = (int)rem; }
    __syncthreads();
  }
  theta = sh.theta;        // key of the K-th largest score
  ties_taken = sh.ties;    // keys equal to theta that are kept
}

// The general kernel, for d_ffn beyond what ff_topk_reg_kernel keeps in registers: every pass
// re-reads the scores (coalesced, from L2).  LDS_MODE 1: a byte per key (above / equal to / below
// theta) is kept in LDS for the two passes of the ordered compaction.  0: not even that fits.
template <int LDS_MODE>
__global__ __launch_bounds__(1024) void ff_topk_kernel(const double *__restrict__ scores,
                                                       int32_t *__restrict__ indices, int d_ffn,
                                                       int k_stride, KSpec ks) {
  extern __shared__ unsigned long long dyn[];
  __shared__ TopkShared sh;
  __shared__ double red_lo[16], red_hi[16];
  __shared__ int wsum[17], wcnt_eq[16];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x;
  const double *sc = scores + (size_t)b * d_ffn;
  int32_t *out = indices + (size_t)b * k_stride;
  int K = ks.per_block ? ks.per_block[b] : ks.uniform;
  K = max(1, min(K, min(d_ffn, k_stride)));

  unsigned char *cls = reinterpret_cast<unsigned char *>(dyn);
  auto key_at = [&](int i) -> unsigned long long { return score_key(sc[i]); };

  // keys, and the score range
  double lo_v = INFINITY, hi_v = -INFINITY;
  int not_finite = 0;
  for (int base = 0; base < d_ffn; base += 8 * 1024) {   // 8 loads in flight per thread
    double v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = sc[min(base + u * 1024 + tid, d_ffn - 1)] + 0.0;   // past the end: the last score again
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      lo_v = fmin(lo_v, v[u]);
      hi_v = fmax(hi_v, v[u]);
      not_finite |= !(fabs(v[u]) <= 1.7976931348623157e308);
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    lo_v = fmin(lo_v, __shfl_xor(lo_v, off));
    hi_v = fmax(hi_v, __shfl_xor(hi_v, off));
  }
  if (lane == 0) { red_lo[wave] = lo_v; red_hi[wave] = hi_v; }
  for (int i = tid; i < TOPK_BUCKETS; i += 1024) sh.hist[i] = 0;
  if (tid == 0) sh.n_cand = 0;
  // fmin/fmax skip a NaN, whose key nevertheless ranks above (or below) every number: the bucket map
  // would not be monotone over the keys.  The radix path orders the keys themselves, whatever they are.
  not_finite = __syncthreads_or(not_finite);
  lo_v = red_lo[0]; hi_v = red_hi[0];
#pragma unroll
  for (int w = 1; w < 16; ++w) { lo_v = fmin(lo_v, red_lo[w]); hi_v = fmax(hi_v, red_hi[w]); }
  const bool need_radix = not_finite || !(hi_v > lo_v);   // all scores equal (or not ordered): no range to cut into buckets
  unsigned long long theta;
  int ties_taken;
  topk_threshold(sh, K, lo_v, hi_v, need_radix,
                 [&](auto fn) __attribute__((always_inline)) { for (int i = tid; i < d_ffn; i += 1024) fn(key_at(i)); },
                 theta, ties_taken);

  if (LDS_MODE == 1) {
    for (int i = tid; i < d_ffn; i += 1024) {
      const unsigned long long key = score_key(sc[i]);
      cls[i] = key > theta ? 2 : (key == theta ? 1 : 0);
    }
    __syncthreads();
  }
  // 2 = above theta, 1 = equal, 0 = below
  auto class_at = [&](int i) -> int {
    if (LDS_MODE == 1) return cls[i];
    const unsigned long long key = key_at(i);
    return key > theta ? 2 : (key == theta ? 1 : 0);
  };
  // Ordered compaction.  Wavefront w owns the index range [w * span, (w + 1) * span) and walks it 64
  // consecutive indices at a time, so the rank of a kept index among the kept ones is the count over
  // lower wavefronts (one scan over 16 totals) plus the count over earlier rows and lower lanes
  // (ballots).  Ties keep exactly the ties_taken lowest indices.
  const int span = ((d_ffn + 15) / 16 + 63) / 64 * 64;
  const int w0 = wave * span;
  int n_gt = 0, n_eq = 0;
  for (int j = 0; j < span; j += 64) {
    const int i = w0 + j + lane;
    const int c = i < d_ffn ? class_at(i) : 0;
    n_gt += __popcll(__ballot(c == 2));
    n_eq += __popcll(__ballot(c == 1));
  }
  if (lane == 0) { wsum[wave] = n_gt; wcnt_eq[wave] = n_eq; }
  __syncthreads();
  // every wavefront scans the 16 pairs itself: lane l < 16 holds wavefront l's totals
  const int e_l = lane < 16 ? wcnt_eq[lane] : 0;
  const int e_incl = wave_incl_scan(e_l, lane);
  const int quota_l = max(0, min(e_l, ties_taken - (e_incl - e_l)));
  const int kept_l = (lane < 16 ? wsum[lane] : 0) + quota_l;
  const int kept_incl = wave_incl_scan(kept_l, lane);
  int eq_seen = __shfl(e_incl - e_l, wave);          // ties at lower indices than this wavefront's range
  int pos = __shfl(kept_incl - kept_l, wave);        // kept indices below this wavefront's range
  const unsigned long long lower = (1ull << lane) - 1ull;
  for (int j = 0; j < span; j += 64) {
    const int i = w0 + j + lane;
    const int c = i < d_ffn ? class_at(i) : 0;
    const unsigned long long m_eq = __ballot(c == 1);
    const bool take = c == 2 || (c == 1 && eq_seen + (int)__popcll(m_eq & lower) < ties_taken);
    const unsigned long long m_take = __ballot(take);
    const int at = pos + __popcll(m_take & lower);
    if (take && at < K) out[at] = i;               // never past the list, whatever the scores were
    pos += __popcll(m_take);
    eq_seen += __popcll(m_eq);
  }
  for (int i = K + tid; i < k_stride; i += 1024) out[i] = -1;
}

// min or max of a 32-bit value over the wavefront with data-parallel-primitive lane exchanges inside
// the rows of 16 lanes (xor 1, xor 2, mirror in 8, mirror in 16) and four lane reads across the rows
template <bool MAX, int CTRL>
__device__ __forceinline__ unsigned int dpp_minmax_step(unsigned int v) {
  const unsigned int o = (unsigned int)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xf, 0xf, false);
  return MAX ? max(v, o) : min(v, o);
}
template <bool MAX>
__device__ __forceinline__ unsigned int wave_minmax_u32(unsigned int v) {
  v = dpp_minmax_step<MAX, 0xB1>(v);    // quad_perm [1,0,3,2]
  v = dpp_minmax_step<MAX, 0x4E>(v);    // quad_perm [2,3,0,1]
  v = dpp_minmax_step<MAX, 0x141>(v);   // row_half_mirror
  v = dpp_minmax_step<MAX, 0x140>(v);   // row_mirror
  const unsigned int a = __builtin_amdgcn_readlane(v, 0), b = __builtin_amdgcn_readlane(v, 16);
  const unsigned int c = __builtin_amdgcn_readlane(v, 32), d = __builtin_amdgcn_readlane(v, 48);
  return MAX ? max(max(a, b), max(c, d)) : min(min(a, b), min(c, d));
}

// The same selection for d_ffn <= 1024 * ROWS with every key in a register: thread t owns the
// indices t, t + 1024, ... (row u = index / 1024), so the scores are read with all loads in flight
// and no pass reads keys back from LDS.  Index order is row-major over (row, wavefront, lane): the rank
// of a kept index among the kept ones is a scan over the ROWS x 16 per-(row, wavefront) ballot counts
// (one wavefront does it) plus the count over lower lanes of its own ballot.
template <int ROWS>
__global__ __launch_bounds__(1024) void ff_topk_reg_kernel(const double *__restrict__ scores,
                                                           int32_t *__restrict__ indices, int d_ffn,
                                                           int k_stride, KSpec ks) {
  __shared__ TopkShared sh;
  __shared__ unsigned int red_lo[16], red_hi[16];
  __shared__ int cnt_gt[ROWS * 16], cnt_eq[ROWS * 16];  // per (row, wavefront); then their exclusive scans

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x;
  const double *sc = scores + (size_t)b * d_ffn;
  int32_t *out = indices + (size_t)b * k_stride;
  int K = ks.per_block ? ks.per_block[b] : ks.uniform;
  K = max(1, min(K, min(d_ffn, k_stride)));

  // keys; a row past the end repeats the last score and is masked by `valid`.  The score range only
  // shapes the bucket map, so bounds that enclose it are as good as the exact ends: the high words of
  // the smallest and largest key, which cost 32-bit wavefront reductions.
  unsigned long long key[ROWS];
  unsigned int lo_w = 0xffffffffu, hi_w = 0u;
#pragma unroll
  for (int u0 = 0; u0 < ROWS; u0 += 16) {
    double v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u)
      if (u0 + u < ROWS) v[u] = sc[min((u0 + u) * 1024 + tid, d_ffn - 1)];
#pragma unroll
    for (int u = 0; u < 16; ++u)
      if (u0 + u < ROWS) {
        key[u0 + u] = score_key(v[u]);
        lo_w = min(lo_w, (unsigned int)(key[u0 + u] >> 32));
        hi_w = max(hi_w, (unsigned int)(key[u0 + u] >> 32));
      }
  }
  auto valid = [&](int u) -> bool { return u * 1024 + tid < d_ffn; };
  lo_w = wave_minmax_u32<false>(lo_w);
  hi_w = wave_minmax_u32<true>(hi_w);
  if (lane == 0) { red_lo[wave] = lo_w; red_hi[wave] = hi_w; }
  for (int i = tid; i < TOPK_BUCKETS; i += 1024) sh.hist[i] = 0;
  if (tid == 0) sh.n_cand = 0;
  __syncthreads();
  lo_w = red_lo[0]; hi_w = red_hi[0];
#pragma unroll
  for (int w = 1; w < 16; ++w) { lo_w = min(lo_w, red_lo[w]); hi_w = max(hi_w, red_hi[w]); }
  const double lo_v = key_score((unsigned long long)lo_w << 32);
  const double hi_v = key_score(((unsigned long long)hi_w << 32) | 0xffffffffull);
  const bool need_radix = !(hi_v > lo_v);   // no ordered range to cut into buckets (not finite)
  unsigned long long theta;
  int ties_taken;
  topk_threshold(sh, K, lo_v, hi_v, need_radix,
                 [&](auto fn) __attribute__((always_inline)) {
#pragma unroll
                   for (int u = 0; u < ROWS; ++u)
                     if (valid(u)) fn(key[u]);
                 },
                 theta, ties_taken);

  // ordered compaction
  unsigned long long m_gt[ROWS], m_eq[ROWS];
#pragma unroll
  for (int u = 0; u < ROWS; ++u) {
    m_gt[u] = __ballot(valid(u) && key[u] > theta);
    m_eq[u] = __ballot(valid(u) && key[u] == theta);
  }
  // lane u < ROWS publishes row u of this wavefront
  {
    int g = 0, e = 0;
#pragma unroll
    for (int u = 0; u < ROWS; ++u)
      if (lane == u) { g = __popcll(m_gt[u]); e = __popcll(m_eq[u]); }
    if (lane < ROWS) { cnt_gt[lane * 16 + wave] = g; cnt_eq[lane * 16 + wave] = e; }
  }
  __syncthreads();
  if (wave == 0) {
    // lane l scans entries [l * PER, (l + 1) * PER) of the (row, wavefront) order
    constexpr int PER = ROWS * 16 / 64;
    int e[PER], g[PER], es = 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) { e[q] = cnt_eq[lane * PER + q]; g[q] = cnt_gt[lane * PER + q]; es += e[q]; }
    int eq_before = wave_incl_scan(es, lane) - es;   // ties at lower indices than this lane's entries
    int ks_ = 0, kept[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int eq_q = e[q];
      const int quota = max(0, min(eq_q, ties_taken - eq_before));
      kept[q] = g[q] + quota;
      e[q] = eq_before;                               // ties at lower indices than the entry
      eq_before += eq_q;
      ks_ += kept[q];
    }
    int pos = wave_incl_scan(ks_, lane) - ks_;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      cnt_eq[lane * PER + q] = e[q];
      cnt_gt[lane * PER + q] = pos;                   // kept indices below the entry
      pos += kept[q];
    }
  }
  __syncthreads();
  int eq_row = 0, pos_row = 0;
  if (lane < ROWS) { eq_row = cnt_eq[lane * 16 + wave]; pos_row = cnt_gt[lane * 16 + wave]; }
  const unsigned long long lower = (1ull << lane) - 1ull;
#pragma unroll
  for (int u = 0; u < ROWS; ++u) {
    const int eq_seen = __builtin_amdgcn_readlane(eq_row, u);
    const int pos = __builtin_amdgcn_readlane(pos_row, u);
    const bool is_gt = (m_gt[u] >> lane) & 1ull, is_eq = (m_eq[u] >> lane) & 1ull;
    const bool take = is_gt || (is_eq && eq_seen + (int)__popcll(m_eq[u] & lower) < ties_taken);
    const unsigned long long m_take = __ballot(take);
    const int at = pos + __popcll(m_take & lower);
    if (take && at < K) out[at] = u * 1024 + tid;   // never past the list, whatever the scores were
  }
  for (int i = K + tid; i < k_stride; i += 1024) out[i] = -1;
}

}  // namespace

static int g_topk_lds_raised = 0;

hipError_t ff_launch_predict(const PredictParams &p, int lds_limit, hipStream_t s, Profiler *prof) {
  const int n_slices = (p.d_model + 511) / 512;
  prof_begin(prof, FF_STAGE_POOL, s);
  if (p.q_pred) {
    hipLaunchKernelGGL(ff_logits_kernel, dim3((p.T + 3) / 4), dim3(256), 0, s, p.x, p.q_pred, p.z,
                       p.T, p.d_model);
    hipLaunchKernelGGL(ff_pool_kernel<true>, dim3(n_slices, p.n_blocks), dim3(256),
                       (size_t)p.block * sizeof(double), s, p.x, p.z, p.w1, p.hpart, p.T, p.d_model,
                       p.block, p.r);
  } else {
    hipLaunchKernelGGL(ff_pool_kernel<false>, dim3(n_slices, p.n_blocks), dim3(256),
                       0, s, p.x, (const double *)nullptr, p.w1, p.hpart, p.T, p.d_model, p.block, p.r);
  }
  prof_end(prof, s);
  prof_begin(prof, FF_STAGE_MLP, s);
  const int n_groups = (p.n_blocks + MLP_BB - 1) / MLP_BB;
  hipLaunchKernelGGL(ff_scores_kernel, dim3((p.d_ffn + 1023) / 1024, n_groups), dim3(256),
                     (size_t)MLP_BB * p.r * sizeof(double), s, p.hpart, p.w2, p.scores, p.n_blocks, p.r,
                     n_slices, p.d_ffn);
  prof_end(prof, s);
  prof_begin(prof, FF_STAGE_TOPK, s);
  if (p.d_ffn <= 16 * 1024) {
    hipLaunchKernelGGL(ff_topk_reg_kernel<16>, dim3(p.n_blocks), dim3(1024), 0, s, p.scores, p.indices,
                       p.d_ffn, p.k_stride, p.k);
  } else if (p.d_ffn <= 24 * 1024) {
    hipLaunchKernelGGL(ff_topk_reg_kernel<24>, dim3(p.n_blocks), dim3(1024), 0, s, p.scores, p.indices,
                       p.d_ffn, p.k_stride, p.k);
  } else if (p.d_ffn <= 32 * 1024) {
    hipLaunchKernelGGL(ff_topk_reg_kernel<32>, dim3(p.n_blocks), dim3(1024), 0, s, p.scores, p.indices,
                       p.d_ffn, p.k_stride, p.k);
  } else {
    // the kernel's own static arrays (bucket histogram, candidates, scan scratch) take under 26 KiB
    const size_t dyn_limit = (size_t)lds_limit - 26 * 1024;
    if (!g_topk_lds_raised) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(ff_topk_kernel<1>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn_limit);
      if (e != hipSuccess) return e;
      g_topk_lds_raised = 1;
    }
    const size_t cls_bytes = ((size_t)p.d_ffn + 15) / 16 * 16;
    if (cls_bytes <= dyn_limit) {
      hipLaunchKernelGGL(ff_topk_kernel<1>, dim3(p.n_blocks), dim3(1024), cls_bytes, s, p.scores,
                         p.indices, p.d_ffn, p.k_stride, p.k);
    } else {
      hipLaunchKernelGGL(ff_topk_kernel<0>, dim3(p.n_blocks), dim3(1024), 0, s, p.scores,
                         p.indices, p.d_ffn, p.k_stride, p.k);
    }
  }
  prof_end(prof, s);
  return hipGetLastError();
}

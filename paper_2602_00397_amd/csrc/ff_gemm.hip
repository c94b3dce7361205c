// Gathered SwiGLU GEMMs on bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 accumulate.
//
//   gemm1 (Eq. 15, 16, 18 and the first half of Eq. 20):
//       H[t][p] = bf16( SiLU(x_t . Wgate[idx_b[p]]) * (x_t . Wup[idx_b[p]]) )   p <  K_b
//       H[t][p] = bf16( act(x_t . Wc1[p - K_b]) )                    K_b <= p <  K_b + rc
//       H[t][p] = 0                                                   up to the next multiple of 64
//   gemm2 (Eq. 17, 18 and the second half of Eq. 20, the sum of Eq. 21):
//       Y[t][:] = sum_p H[t][p] * R_b[p][:],  R_b[p] = Wdown[idx_b[p]] for p < K_b,
//                                              R_b[p] = Wc2[p - K_b] for the compensator units.
// The compensator is thus rc extra, always selected, un-gated "neurons" appended to
// every block's list, and its add happens in the accumulator of gemm2.
// With idx == nullptr the list is 0..d_ffn-1 and the pair computes Eq. 10.
//
// Weight rows are gathered straight from the neuron-major matrices by per-thread row
// pointers; nothing is packed per block.  A workgroup owns all tokens of one block
// (or an M-slice of it) and a range of list positions (gemm1) or of output columns
// (gemm2).  Workgroup ids are mapped so that the ids one XCD receives (id mod 8) walk
// the position/column ranges in the same order over that XCD's own group of blocks:
// blocks that selected the same weight rows then hit them in that XCD's L2.
#include "ff_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

__device__ __forceinline__ f32x16_t mfma32(const u32x4_t &a, const u32x4_t &b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                 __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// Workgroup id -> (virtual block, n tile).  XCD x = id mod 8 owns virtual blocks
// x, x+8, ...; its ids enumerate n tiles outermost, its blocks innermost.
struct TileCoord { int vb, nt; bool valid; };
__device__ __forceinline__ TileCoord map_tile(int w, int V, int N) {
  const int cnt = (V + 7) >> 3;
  const int xcd = w & 7, l = w >> 3;
  const int nt = l / cnt, j = l - nt * cnt;
  const int vb = xcd + 8 * j;
  TileCoord t = {vb, nt, vb < V && nt < N};
  return t;
}

// 16-byte chunk swizzle of a k-contiguous tile row (conflict-free ds_read_b128 over
// 8 consecutive rows): rows of 64 B hold 4 chunks, rows of 128 B hold 8.
template <int BK>
__device__ __forceinline__ int swz(int row) { return BK == 32 ? ((row >> 1) & 3) : (row & 7); }

__device__ __forceinline__ int block_k(const KSpec &k, int b, int d_ffn, int k_stride, bool has_idx) {
  int K = k.per_block ? k.per_block[b] : k.uniform;
  K = max(1, min(K, d_ffn));
  if (has_idx) K = min(K, k_stride);
  return K;
}

__device__ __forceinline__ float act_apply(int act, float g) {
  if (act == FF_ACT_SILU) return g / (1.0f + __expf(-g));
  if (act == FF_ACT_RELU) return fmaxf(g, 0.0f);
  return g;
}

__device__ __forceinline__ u32x4_t mk4(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  u32x4_t v = {a, b, c, d};
  return v;
}

// ============================ gemm1 =========================================
// WM x WN wavefronts; a wavefront computes 32*TM tokens x 32*TN list positions, for the
// gate and the up projection at once (the SiLU(g)*u epilogue is lane-local).
// Position p = wave_base + TN*c + f is held by MFMA tile f, column c, so a lane owns TN
// consecutive positions of a token row and H is written in contiguous runs.
template <int WM, int WN, int TM, int TN, int BK>
__global__ __launch_bounds__(WM * WN * 64) __attribute__((amdgpu_waves_per_eu(TM * TN * 2 <= 8 ? 2 : 1)))
void ff_gemm1_kernel(Gemm1Params p, int V, int mt, int N) {
  constexpr int NT = WM * WN * 64;
  constexpr int BM = WM * TM * 32;
  constexpr int WNn = TN * 32;
  constexpr int BNn = WN * WNn;
  constexpr int CPR = BK / 8;
  constexpr int ROWB = BK * 2;
  constexpr int A_BYTES = BM * ROWB;
  constexpr int B_BYTES = 2 * BNn * ROWB;
  constexpr int STAGE = A_BYTES + B_BYTES;
  constexpr int A_CH = BM * CPR, B_CH = 2 * BNn * CPR;
  constexpr int A_PER = (A_CH + NT - 1) / NT, B_PER = (B_CH + NT - 1) / NT;
  extern __shared__ __align__(16) uint8_t smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int c = lane & 31, half = lane >> 5;

  const TileCoord tc = map_tile(blockIdx.x, V, N);
  if (!tc.valid) return;
  const int b = tc.vb / mt, m = tc.vb - b * mt;
  const int t0 = b * p.block + m * BM;
  const int rows_valid = min(p.T, (b + 1) * p.block) - t0;
  if (rows_valid <= 0) return;
  const int Kb = block_k(p.k, b, p.d_ffn, p.k_stride, p.idx != nullptr);
  const int ntot = Kb + p.rc;
  const int n0 = tc.nt * BNn;
  if (n0 >= ntot) return;

  const bf16_t *a_src[A_PER];
  int a_dst[A_PER];
#pragma unroll
  for (int i = 0; i < A_PER; ++i) {
    const int q = tid + i * NT;
    const int row = q / CPR, ch = q % CPR;
    const int tok = t0 + min(row, rows_valid - 1);
    a_src[i] = p.x + (size_t)tok * p.d_model + ch * 8;
    a_dst[i] = row * ROWB + ((ch ^ swz<BK>(row)) << 4);
  }
  const bf16_t *b_src[B_PER];
  int b_dst[B_PER];
#pragma unroll
  for (int i = 0; i < B_PER; ++i) {
    const int q = tid + i * NT;
    const int rho = q / CPR, ch = q % CPR;
    const int mat = rho / BNn, rp = rho % BNn;
    const int w = rp / WNn, f = (rp % WNn) >> 5, cc = rp & 31;
    const int pos = n0 + w * WNn + TN * cc + f;
    const bf16_t *base = p.wg;
    int row = 0;
    if (pos < Kb) {
      row = p.idx ? p.idx[(size_t)b * p.k_stride + pos] : pos;
      row = min(max(row, 0), p.d_ffn - 1);
      base = mat ? p.wu : p.wg;
    } else if (pos < ntot) {
      row = pos - Kb;
      base = p.wc1;
    }
    b_src[i] = base + (size_t)row * p.d_model + ch * 8;
    b_dst[i] = A_BYTES + rho * ROWB + ((ch ^ swz<BK>(rho)) << 4);
  }

  f32x16_t accg[TM][TN], accu[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) { accg[i][j][e] = 0.0f; accu[i][j][e] = 0.0f; }

  u32x4_t a_reg[A_PER], b_reg[B_PER];
  auto g_load = [&](int kt) __attribute__((always_inline)) {
    const int koff = kt * BK;
#pragma unroll
    for (int i = 0; i < A_PER; ++i)
      if (A_CH % NT == 0 || tid + i * NT < A_CH) a_reg[i] = *reinterpret_cast<const u32x4_t *>(a_src[i] + koff);
#pragma unroll
    for (int i = 0; i < B_PER; ++i)
      if (B_CH % NT == 0 || tid + i * NT < B_CH) b_reg[i] = *reinterpret_cast<const u32x4_t *>(b_src[i] + koff);
  };
  auto s_store = [&](uint8_t *st) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < A_PER; ++i)
      if (A_CH % NT == 0 || tid + i * NT < A_CH) *reinterpret_cast<u32x4_t *>(st + a_dst[i]) = a_reg[i];
#pragma unroll
    for (int i = 0; i < B_PER; ++i)
      if (B_CH % NT == 0 || tid + i * NT < B_CH) *reinterpret_cast<u32x4_t *>(st + b_dst[i]) = b_reg[i];
  };

  const int nk = p.d_model / BK;
  g_load(0);
  s_store(smem);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const uint8_t *cur = smem + (kt & 1) * STAGE;
    const bool more = kt + 1 < nk;
    if (more) g_load(kt + 1);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int q = 2 * kk + half;
      u32x4_t af[TM], bg[TN], bu[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = (wm * TM + i) * 32 + c;
        af[i] = *reinterpret_cast<const u32x4_t *>(cur + row * ROWB + ((q ^ swz<BK>(row)) << 4));
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int rho = wn * WNn + j * 32 + c;
        const int off = rho * ROWB + ((q ^ swz<BK>(rho)) << 4);
        bg[j] = *reinterpret_cast<const u32x4_t *>(cur + A_BYTES + off);
        bu[j] = *reinterpret_cast<const u32x4_t *>(cur + A_BYTES + BNn * ROWB + off);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          accg[i][j] = mfma32(af[i], bg[j], accg[i][j]);
          accu[i][j] = mfma32(af[i], bu[j], accu[i][j]);
        }
    }
    if (more) s_store(smem + ((kt + 1) & 1) * STAGE);
    __syncthreads();
  }

  // epilogue: H = bf16(SiLU(g) * u) (FFN neurons), bf16(act(g)) (compensator units), 0 (padding)
  const int pos0 = n0 + wn * WNn + TN * c;
  if (pos0 < p.hs) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int rowl = (wm * TM + i) * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
        if (rowl < rows_valid) {
          float hv[TN];
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            const int pos = pos0 + j;
            const float g = accg[i][j][e], u = accu[i][j][e];
            hv[j] = pos < Kb ? act_apply(FF_ACT_SILU, g) * u : (pos < ntot ? act_apply(p.comp_act, g) : 0.0f);
          }
          bf16_t *dst = p.h + (size_t)(t0 + rowl) * p.hs + pos0;
          if (TN == 1) {
            dst[0] = f32_to_bf16(hv[0]);
          } else if (TN == 2) {
            *reinterpret_cast<uint32_t *>(dst) = pack_bf16x2(hv[0], hv[1]);
          } else {
#pragma unroll
            for (int j = 0; j < TN; j += 2)
              *reinterpret_cast<uint32_t *>(dst + j) = pack_bf16x2(hv[j], hv[j + 1]);
          }
        }
      }
  }
}

// ============================ gemm2 =========================================
// WM x WN wavefronts; a wavefront computes 32*TM tokens x 128 output columns.  The B
// operand tile is [BK list positions][BN columns] as it lies in memory (a gathered row is
// contiguous along the columns); the k-contiguous MFMA fragments are formed by reading
// 8 rows x 4 columns per lane (ds_read_b64) and interleaving row pairs in registers.
// MFMA tile f, column c holds output column wave_base + 4c + f: a lane ends up with 4
// consecutive columns of a row.
template <int WM, int WN, int TM, int BK>
__global__ __launch_bounds__(WM * WN * 64) __attribute__((amdgpu_waves_per_eu(TM * 4 <= 8 ? 2 : 1)))
void ff_gemm2_kernel(Gemm2Params p, int V, int mt, int N) {
  constexpr int NT = WM * WN * 64;
  constexpr int BM = WM * TM * 32;
  constexpr int BN = WN * 128;
  constexpr int CPR = BK / 8;
  constexpr int ROWB = BK * 2;
  constexpr int A_BYTES = BM * ROWB;
  constexpr int ROWB_B = BN * 2;
  constexpr int B_BYTES = BK * ROWB_B;
  constexpr int STAGE = A_BYTES + B_BYTES;
  constexpr int CPR_B = BN / 8;
  constexpr int A_CH = BM * CPR, B_CH = BK * CPR_B;
  constexpr int A_PER = (A_CH + NT - 1) / NT, B_PER = (B_CH + NT - 1) / NT;
  static_assert(B_CH % NT == 0, "B tile must split evenly over the threads");
  extern __shared__ __align__(16) uint8_t smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int c = lane & 31, half = lane >> 5;

  const TileCoord tc = map_tile(blockIdx.x, V, N);
  if (!tc.valid) return;
  const int b = tc.vb / mt, m = tc.vb - b * mt;
  const int t0 = b * p.block + m * BM;
  const int rows_valid = min(p.T, (b + 1) * p.block) - t0;
  if (rows_valid <= 0) return;
  const int Kb = block_k(p.k, b, p.d_ffn, p.k_stride, p.idx != nullptr);
  const int ntot = Kb + p.rc;
  const int n0 = tc.nt * BN;
  const int nk = (ntot + BK - 1) / BK;

  const bf16_t *a_src[A_PER];
  int a_dst[A_PER];
#pragma unroll
  for (int i = 0; i < A_PER; ++i) {
    const int q = tid + i * NT;
    const int row = q / CPR, ch = q % CPR;
    const int tok = t0 + min(row, rows_valid - 1);
    a_src[i] = p.h + (size_t)tok * p.hs + ch * 8;
    a_dst[i] = row * ROWB + ((ch ^ swz<BK>(row)) << 4);
  }
  // B: thread loads chunk b_ch of tile rows b_row0 + i * (NT / CPR_B)
  const int b_ch = tid % CPR_B, b_row0 = tid / CPR_B;
  const int b_col = min(n0 + b_ch * 8, p.d_model - 8);
  const int32_t *idx_row = p.idx ? p.idx + (size_t)b * p.k_stride : nullptr;
  // source row id of list position pos: < d_ffn -> Wdown row, else compensator unit
  auto src_row = [&](int pos) __attribute__((always_inline)) -> int {
    if (pos < Kb) {
      const int r = idx_row ? idx_row[pos] : pos;
      return min(max(r, 0), p.d_ffn - 1);
    }
    return pos < ntot ? p.d_ffn + (pos - Kb) : 0;
  };
  auto row_ptr = [&](int r) __attribute__((always_inline)) -> const bf16_t * {
    return (r < p.d_ffn ? p.wd + (size_t)r * p.d_model : p.wc2 + (size_t)(r - p.d_ffn) * p.d_model) + b_col;
  };

  f32x16_t acc[TM][4];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][f][e] = 0.0f;

  u32x4_t a_reg[A_PER], b_reg[B_PER];
  int rows_next[B_PER];
  auto fetch_rows = [&](int kt) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < B_PER; ++i) rows_next[i] = src_row(kt * BK + b_row0 + i * (NT / CPR_B));
  };
  auto g_load = [&](int kt) __attribute__((always_inline)) {  // uses rows_next == rows of tile kt
    const int koff = kt * BK;
#pragma unroll
    for (int i = 0; i < A_PER; ++i)
      if (A_CH % NT == 0 || tid + i * NT < A_CH) a_reg[i] = *reinterpret_cast<const u32x4_t *>(a_src[i] + koff);
#pragma unroll
    for (int i = 0; i < B_PER; ++i) b_reg[i] = *reinterpret_cast<const u32x4_t *>(row_ptr(rows_next[i]));
  };
  auto s_store = [&](uint8_t *st) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < A_PER; ++i)
      if (A_CH % NT == 0 || tid + i * NT < A_CH) *reinterpret_cast<u32x4_t *>(st + a_dst[i]) = a_reg[i];
#pragma unroll
    for (int i = 0; i < B_PER; ++i)
      *reinterpret_cast<u32x4_t *>(st + A_BYTES + (b_row0 + i * (NT / CPR_B)) * ROWB_B + b_ch * 16) = b_reg[i];
  };

  fetch_rows(0);
  g_load(0);
  if (nk > 1) fetch_rows(1);
  s_store(smem);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const uint8_t *cur = smem + (kt & 1) * STAGE;
    const bool more = kt + 1 < nk;
    if (more) {
      g_load(kt + 1);
      if (kt + 2 < nk) fetch_rows(kt + 2);
    }
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int q = 2 * kk + half;
      u32x4_t af[TM];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = (wm * TM + i) * 32 + c;
        af[i] = *reinterpret_cast<const u32x4_t *>(cur + row * ROWB + ((q ^ swz<BK>(row)) << 4));
      }
      u32x2_t d[8];
      const uint8_t *bb = cur + A_BYTES + (kk * 16 + 8 * half) * ROWB_B + (wn * 128 + 4 * c) * 2;
#pragma unroll
      for (int i = 0; i < 8; ++i) d[i] = *reinterpret_cast<const u32x2_t *>(bb + i * ROWB_B);
      u32x4_t bf[4];
      // column 4c+f of rows (2j, 2j+1) -> one dword, lower row in the low half
#define FF_LO(e, o) (((e) & 0xffffu) | ((o) << 16))
#define FF_HI(e, o) (((e) >> 16) | ((o) & 0xffff0000u))
      bf[0] = mk4(FF_LO(d[0].x, d[1].x), FF_LO(d[2].x, d[3].x), FF_LO(d[4].x, d[5].x), FF_LO(d[6].x, d[7].x));
      bf[1] = mk4(FF_HI(d[0].x, d[1].x), FF_HI(d[2].x, d[3].x), FF_HI(d[4].x, d[5].x), FF_HI(d[6].x, d[7].x));
      bf[2] = mk4(FF_LO(d[0].y, d[1].y), FF_LO(d[2].y, d[3].y), FF_LO(d[4].y, d[5].y), FF_LO(d[6].y, d[7].y));
      bf[3] = mk4(FF_HI(d[0].y, d[1].y), FF_HI(d[2].y, d[3].y), FF_HI(d[4].y, d[5].y), FF_HI(d[6].y, d[7].y));
#undef FF_LO
#undef FF_HI
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int f = 0; f < 4; ++f) acc[i][f] = mfma32(af[i], bf[f], acc[i][f]);
    }
    if (more) s_store(smem + ((kt + 1) & 1) * STAGE);
    __syncthreads();
  }

  const int col = n0 + wn * 128 + 4 * c;
  if (col < p.d_model) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int rowl = (wm * TM + i) * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
        if (rowl < rows_valid) {
          const size_t o = (size_t)(t0 + rowl) * p.d_model + col;
          if (p.out_f32) {
            *reinterpret_cast<float4 *>(reinterpret_cast<float *>(p.y) + o) =
                make_float4(acc[i][0][e], acc[i][1][e], acc[i][2][e], acc[i][3][e]);
          } else {
            *reinterpret_cast<uint2 *>(reinterpret_cast<bf16_t *>(p.y) + o) =
                make_uint2(pack_bf16x2(acc[i][0][e], acc[i][1][e]), pack_bf16x2(acc[i][2][e], acc[i][3][e]));
          }
        }
      }
  }
}

// ---- variant tables --------------------------------------------------------
struct Variant {
  const void *fn;
  int bm, bn, threads, lds;
};

template <int WM, int WN, int TM, int TN, int BK>
Variant g1v() {
  return Variant{reinterpret_cast<const void *>(&ff_gemm1_kernel<WM, WN, TM, TN, BK>), WM * TM * 32,
                 WN * TN * 32, WM * WN * 64, 2 * (WM * TM * 32 + 2 * WN * TN * 32) * BK * 2};
}
template <int WM, int WN, int TM, int BK>
Variant g2v() {
  return Variant{reinterpret_cast<const void *>(&ff_gemm2_kernel<WM, WN, TM, BK>), WM * TM * 32,
                 WN * 128, WM * WN * 64, 2 * (WM * TM * 32 * BK * 2 + BK * WN * 128 * 2)};
}

const Variant kGemm1[] = {
    g1v<2, 4, 2, 2, 32>(),  // 0: 128 tokens x 256 positions, 8 waves
    g1v<2, 2, 2, 2, 32>(),  // 1: 128 x 128, 4 waves
    g1v<4, 2, 2, 2, 32>(),  // 2: 256 x 128, 8 waves
    g1v<1, 4, 2, 2, 32>(),  // 3: 64 x 256, 4 waves
    g1v<1, 8, 2, 2, 32>(),  // 4: 64 x 512, 8 waves
    g1v<2, 2, 2, 2, 64>(),  // 5: 128 x 128, 4 waves, BK 64
    g1v<1, 4, 4, 2, 32>(),  // 6: 128 x 256, 4 waves with 128 x 64 wave tiles
};
const Variant kGemm2[] = {
    g2v<2, 4, 2, 32>(),  // 0: 128 tokens x 512 columns, 8 waves
    g2v<2, 2, 2, 32>(),  // 1: 128 x 256, 4 waves
    g2v<4, 2, 2, 32>(),  // 2: 256 x 256, 8 waves
    g2v<1, 4, 2, 32>(),  // 3: 64 x 512, 4 waves
    g2v<1, 8, 2, 32>(),  // 4: 64 x 1024, 8 waves
    g2v<2, 2, 2, 64>(),  // 5: 128 x 256, 4 waves, BK 64
};
constexpr int kNumGemm1 = sizeof(kGemm1) / sizeof(Variant);
constexpr int kNumGemm2 = sizeof(kGemm2) / sizeof(Variant);

// Tile choice by the block size: the largest M tile a block fills.
int choose(int block, int v64, int v128, int v256) {
  if (block >= 256) return v256;
  if (block > 64) return v128;
  return v64;
}

}  // namespace

int ff_gemm1_num_variants() { return kNumGemm1; }
int ff_gemm2_num_variants() { return kNumGemm2; }

hipError_t ff_gemm_init() {
  for (int i = 0; i < kNumGemm1; ++i)
    if (kGemm1[i].lds > 48 * 1024) {
      hipError_t e = hipFuncSetAttribute(kGemm1[i].fn, hipFuncAttributeMaxDynamicSharedMemorySize, kGemm1[i].lds);
      if (e != hipSuccess) return e;
    }
  for (int i = 0; i < kNumGemm2; ++i)
    if (kGemm2[i].lds > 48 * 1024) {
      hipError_t e = hipFuncSetAttribute(kGemm2[i].fn, hipFuncAttributeMaxDynamicSharedMemorySize, kGemm2[i].lds);
      if (e != hipSuccess) return e;
    }
  return hipSuccess;
}

static hipError_t launch_variant(const Variant &v, const void *params, int block, int n_blocks,
                                 int n_extent, hipStream_t s) {
  // virtual blocks: each block is cut into M tiles of v.bm tokens
  int mt = (block + v.bm - 1) / v.bm;
  int V = n_blocks * mt;
  int N = (n_extent + v.bn - 1) / v.bn;
  int grid = 8 * ((V + 7) / 8) * N;
  void *args[] = {const_cast<void *>(params), &V, &mt, &N};
  return hipLaunchKernel(v.fn, dim3(grid), dim3(v.threads), args, v.lds, s);
}

hipError_t ff_launch_gemm1(const Gemm1Params &p, int variant, hipStream_t s) {
  if (variant < 0) variant = choose(p.block, 3, 0, 2);
  if (variant >= kNumGemm1) return hipErrorInvalidValue;
  return launch_variant(kGemm1[variant], &p, p.block, p.n_blocks, p.k.k_max + p.rc, s);
}

hipError_t ff_launch_gemm2(const Gemm2Params &p, int variant, hipStream_t s) {
  if (variant < 0) variant = choose(p.block, 3, 0, 2);
  if (variant >= kNumGemm2) return hipErrorInvalidValue;
  return launch_variant(kGemm2[variant], &p, p.block, p.n_blocks, p.d_model, s);
}

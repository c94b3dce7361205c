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

#include <algorithm>
#include <type_traits>

namespace {

// MFMA groups over which a two-stage ring spreads a stage's copies (all of them would leave the
// last copies no time to land before the next barrier; measured 1, 2, 3 of 4: 2 is best)
constexpr int kSpreadGroupsTwoStage = 2;

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

// Lists of unequal length.  The few blocks longer than the common length ("heavy": the first
// and last block when those stay dense) would otherwise leave their extra tiles for the end of
// the launch, all on the one XCD that owns the block, sharing weight rows with nobody.  Their
// tiles get the first ids instead (they start at once, next to everybody else's), and
// consecutive ids go to consecutive XCDs.
__device__ __forceinline__ int heavy_block(const KSpec &k, int h) {
  int b = k.heavy[0];
#pragma unroll
  for (int i = 1; i < kMaxHeavy; ++i) b = __builtin_amdgcn_readfirstlane((h == i) ? k.heavy[i] : b);   // keeps the chain scalar
  return b;
}
__device__ __forceinline__ bool is_heavy(const KSpec &k, int b) {
  bool r = false;
#pragma unroll
  for (int i = 0; i < kMaxHeavy; ++i) r = r || (i < k.n_heavy && k.heavy[i] == b);
  return r;
}

// which entry of heavy[] block b is, or -1
__device__ __forceinline__ int heavy_index(const KSpec &k, int b) {
  int r = -1;
#pragma unroll
  for (int i = 0; i < kMaxHeavy; ++i) r = (i < k.n_heavy && k.heavy[i] == b) ? i : r;
  return r;
}

// 16-byte chunk swizzle of a k-contiguous tile row: logical chunk q of row r is stored
// at chunk q ^ swz(r).  A ds_read_b128 of one chunk column over consecutive rows must
// spread over all banks both for 8 rows (128-byte bank window) and for 16 rows
// (256-byte window); rows of 64 B hold 4 chunks, rows of 128 B hold 8.  Period 16 rows.
template <int BK>
__device__ __forceinline__ int swz(int row) {
  return BK == 32 ? (((row >> 1) & 3) ^ ((row >> 3) & 1)) : (((row >> 1) & 7) ^ ((row & 1) << 2));
}

__device__ __forceinline__ int block_k(const KSpec &k, int b, int d_ffn, int k_stride, bool has_idx) {
  int K = k.per_block ? k.per_block[b] : k.uniform;
  K = max(1, min(K, d_ffn));
  if (has_idx) K = min(K, k_stride);
  return K;
}

__device__ __forceinline__ float act_apply(int act, float g) {
  if (act == FF_ACT_SILU) return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g));   // 1-ulp reciprocal: far below bf16 rounding
  if (act == FF_ACT_RELU) return fmaxf(g, 0.0f);
  return g;
}

__device__ __forceinline__ u32x4_t mk4(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  u32x4_t v = {a, b, c, d};
  return v;
}

// ---- asynchronous global -> LDS staging --------------------------------------
// One wavefront instruction moves 64 x 16 bytes from per-lane global addresses to
// 1 KiB of LDS starting at a wave-uniform address (lane l lands at +16 l).  The copy
// bypasses the registers and is tracked by vmcnt only, so loads for later k-steps stay
// in flight across barriers; they are waited for with explicit counts.
// m0 (the LDS base of the copy) is written without being listed as clobbered: it is a reserved register
// that the compiler never allocates and never keeps a value in across statements (it rewrites m0 in front
// of each of its own uses); naming it in the clobber list only draws a "reserved register" warning.
__device__ __forceinline__ void gload_lds16(const void *gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(gptr), "s"(lds_addr)
               : "memory");
}
// the 4-byte form: lane l lands at +4 l (256 bytes per wavefront instruction)
__device__ __forceinline__ void gload_lds4(const void *gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
               :
               : "v"(gptr), "s"(lds_addr)
               : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm_barrier() {
  // lgkmcnt(0): this wavefront's own LDS reads of the slot about to be refilled have completed
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" : : "n"(N) : "memory");
}
__device__ __forceinline__ uint32_t lds_addr_of(const void *p) {
  return (uint32_t)(size_t)(__attribute__((address_space(3))) const uint8_t *)p;
}

// ============================ gemm1 =========================================
// KG groups of WM x WN wavefronts; a wavefront computes 32*TM tokens x 32*TN list positions
// for the gate and the up projection at once (the SiLU(g)*u epilogue is lane-local); with
// KG = 2 the two groups split each stage's k range and exchange halves of their
// accumulators through LDS at the end (fixed order, so results stay reproducible).
// Position p = wave_base + TN*c + f is held by MFMA tile f, column c, so a lane owns TN
// consecutive positions of a token row and H is written in contiguous runs.
// Operands stream through a ring of S LDS stages filled by asynchronous copies issued S-1
// k-steps ahead, one barrier per k-step.  A wave-load covers 1 KiB of a stage = 1024 / (2 BK)
// tile rows; lane l fills 16-byte slot l of it, and fetches the chunk that the read-side
// swizzle expects there.  BK = 64 makes every request a whole 128-byte line.
template <int WM, int WN, int TM, int TN, int BK, int S, int KG = 1>
__global__ __launch_bounds__(WM * WN * KG * 64) __attribute__((amdgpu_waves_per_eu(TM * TN * 2 <= 8 ? 2 : 1)))
void ff_gemm1_kernel(Gemm1Params p, int V, int mt, int N, int NX) {
  constexpr int NW = WM * WN * KG;                 // KG groups of WM x WN wavefronts split each stage's k range
  constexpr int BM = WM * TM * 32;
  constexpr int WNn = TN * 32;
  constexpr int BNn = WN * WNn;
  constexpr int CPR = BK / 8;
  constexpr int ROWB = BK * 2;
  constexpr int A_BYTES = BM * ROWB;
  constexpr int B_BYTES = 2 * BNn * ROWB;
  constexpr int STAGE = A_BYTES + B_BYTES;
  constexpr int RPL = 1024 / ROWB;                 // tile rows per wave-load
  constexpr int NL = STAGE / 1024;                 // wave-loads per stage
  constexpr int L = NL / NW;                       // wave-loads per wavefront per stage
  static_assert(NL % NW == 0, "stage must split evenly over the wavefronts");
  static_assert(A_BYTES % 1024 == 0, "A tile must be whole wave-loads");
  extern __shared__ __align__(16) uint8_t smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kgrp = wave / (WM * WN), wq = wave % (WM * WN);
  const int wm = wq / WN, wn = wq % WN;
  const int c = lane & 31, half = lane >> 5;

  // ids [0, heavy virtual blocks x NX): the NX tiles beyond the common N of the heavy blocks;
  // then the common region, N tiles for every block
  TileCoord tc;
  const int n_first = p.k.n_heavy * mt * NX;
  if ((int)blockIdx.x < n_first) {
    const int h = __builtin_amdgcn_readfirstlane((int)blockIdx.x / NX);
    const int hb = __builtin_amdgcn_readfirstlane(h / mt);
    tc.vb = heavy_block(p.k, hb) * mt + (h - hb * mt);
    tc.nt = N + ((int)blockIdx.x - h * NX);
    tc.valid = true;
  } else {
    tc = map_tile((int)blockIdx.x - n_first, V, N);
  }
  if (!tc.valid) return;
  // wave-uniform by construction; say so, so that everything derived from it stays scalar
  tc.vb = __builtin_amdgcn_readfirstlane(tc.vb);
  tc.nt = __builtin_amdgcn_readfirstlane(tc.nt);
  const int b = tc.vb / mt, m = tc.vb - b * mt;
  const int t0 = b * p.block + m * BM;
  const int rows_valid = min(p.T, (b + 1) * p.block) - t0;
  if (rows_valid <= 0) return;
  const int Kb = __builtin_amdgcn_readfirstlane(block_k(p.k, b, p.d_ffn, p.k_stride, p.idx != nullptr));
  const int ntot = Kb + p.rc;
  const int n0 = __builtin_amdgcn_readfirstlane(p.rem_bn ? min(ntot / p.rem_bn * p.rem_bn, p.rem_cap) : 0) + tc.nt * BNn;
  if (n0 >= ntot) return;
  if (p.full_only && n0 + BNn > ntot) return;   // the remainder launch takes this part-filled tile
  if (p.skip_heavy && is_heavy(p.k, b)) return;  // a launch of their own has covered the heavy blocks' ends

  // wave-load j = wave + i * NW of a stage covers stage bytes [1024 j, 1024 j + 1024)
  const bf16_t *src[L];
  // list position of the B row that copy i of a stage fills (-1: an A row)
  auto b_pos = [&](int i) __attribute__((always_inline)) -> int {
    const int trow = (wave + i * NW) * RPL + lane / CPR;
    if (trow < BM) return -1;
    const int rp = (trow - BM) % BNn;
    return n0 + rp / WNn * WNn + TN * (rp & 31) + ((rp % WNn) >> 5);
  };
  // the list entries first, all loads in flight at once (from a clamped position, so that none is
  // conditional: left inside the branches below, every load is waited for before the next is issued)
  int entry[L];
#pragma unroll
  for (int i = 0; i < L; ++i) {
    const int pos = b_pos(i);
    entry[i] = (p.idx != nullptr && pos >= 0) ? p.idx[(size_t)b * p.k_stride + min(pos, Kb - 1)] : pos;
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < L; ++i) {
    const int j = wave + i * NW;
    const int trow = j * RPL + lane / CPR;          // row within the stage (A rows, then B rows)
    const int ch = (lane % CPR) ^ swz<BK>(trow);  // BM is a multiple of 32: the B rows keep the swizzle phase
    if (trow < BM) {
      const int tok = t0 + min(trow, rows_valid - 1);
      src[i] = p.x + (size_t)tok * p.d_model + ch * 8;
    } else {
      const int mat = (trow - BM) / BNn;
      const int pos = b_pos(i);
      const bf16_t *base = p.wg;
      int row = 0;
      if (pos < Kb) {
        row = min(max(entry[i], 0), p.d_ffn - 1);
        base = mat ? p.wu : p.wg;
      } else if (pos < ntot) {
        row = pos - Kb;
        base = p.wc1;
      }
      src[i] = base + (size_t)row * p.d_model + ch * 8;
    }
  }
  const uint32_t lds0 = lds_addr_of(smem);
  auto issue = [&](int kt) __attribute__((always_inline)) {
    const uint32_t st = lds0 + (uint32_t)(kt % S) * STAGE + (uint32_t)wave * 1024u;
#pragma unroll
    for (int i = 0; i < L; ++i) gload_lds16(src[i] + kt * BK, st + (uint32_t)i * (NW * 1024u));
  };

  auto issue_one = [&](int kt, int i) __attribute__((always_inline)) {
    const uint32_t st = lds0 + (uint32_t)(kt % S) * STAGE + (uint32_t)wave * 1024u;
    gload_lds16(src[i] + kt * BK, st + (uint32_t)i * (NW * 1024u));
  };

  f32x16_t accg[TM][TN], accu[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) { accg[i][j][e] = 0.0f; accu[i][j][e] = 0.0f; }

  // Pipeline.  Stage kt+1 is waited for (and the workgroup synchronised) in front of the LAST
  // MFMA group of stage kt, and the first fragments of stage kt+1 are requested from LDS there, so
  // the matrix pipe has work while they arrive.  After that barrier every wavefront is done reading
  // stage kt, so its ring slot takes the copies of stage kt+S: they are issued one at a time
  // between the MFMAs of the next KQ groups (a burst would park the wavefront on a full
  // memory-issue queue with its matrix pipe idle).
  constexpr int KQ = BK / 16 / KG;                     // MFMA groups (16 k each) per stage and k-group
  static_assert(KQ % 2 == 0, "fragment double buffer needs an even number of groups per stage");
  constexpr int NMF = TM * TN;                         // gate/up MFMA pairs per group
  constexpr int NSP = S == 2 ? (kSpreadGroupsTwoStage < KQ ? kSpreadGroupsTwoStage : KQ) : KQ;  // groups the copies of a stage are spread over
  constexpr int LQ = (L + NSP - 1) / NSP;              // copies issued during one group
  constexpr int PER = (LQ + NMF - 1) / NMF;            // copies behind one MFMA pair
  constexpr int EVERY = NMF / LQ > 0 ? NMF / LQ : 1;
  constexpr int SLOTS = (NMF + EVERY - 1) / EVERY * PER;  // copy slots between the MFMAs of a group
  const int nk = p.d_model / BK;
  u32x4_t af[2][TM], bg[2][TN], bu[2][TN];
  auto frags = [&](int kt, int kq, int buf) __attribute__((always_inline)) {
    const uint8_t *cur = smem + (kt % S) * STAGE;
    const int q = 2 * (kgrp * KQ + kq) + half;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int row = (wm * TM + i) * 32 + c;
      af[buf][i] = *reinterpret_cast<const u32x4_t *>(cur + row * ROWB + ((q ^ swz<BK>(row)) << 4));
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int rho = wn * WNn + j * 32 + c;
      const int off = rho * ROWB + ((q ^ swz<BK>(rho)) << 4);
      bg[buf][j] = *reinterpret_cast<const u32x4_t *>(cur + A_BYTES + off);
      bu[buf][j] = *reinterpret_cast<const u32x4_t *>(cur + A_BYTES + BNn * ROWB + off);
    }
  };
  // MFMA group kq of the current stage from fragment buffer kq & 1, with part `part` (of KQ) of
  // stage `st`'s copies issued in between when `load` is set
  auto group = [&](int kq, int st, int part, bool load) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        accg[i][j] = mfma32(af[kq & 1][i], bg[kq & 1][j], accg[i][j]);
        accu[i][j] = mfma32(af[kq & 1][i], bu[kq & 1][j], accu[i][j]);
        if ((i * TN + j) % EVERY == 0) {
#pragma unroll
          for (int r = 0; r < PER; ++r) {
            const int n = (i * TN + j) / EVERY * PER + r;
            if (n < LQ && part * LQ + n < L) {
              if (load) issue_one(st, part * LQ + n);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        }
      }
#pragma unroll
    for (int n = SLOTS; n < LQ; ++n)
      if (load && part * LQ + n < L) issue_one(st, part * LQ + n);
    __builtin_amdgcn_sched_barrier(0);
  };
  // MAIN: stages kt+S-1 and kt+S both exist (no conditions in the loop body)
  auto step = [&](int kt, auto main_tag) __attribute__((always_inline)) {
    constexpr bool MAIN = decltype(main_tag)::value;
    const bool la = MAIN || kt + S - 1 < nk;
    const bool lb = MAIN || kt + S < nk;
#pragma unroll
    for (int kq = 0; kq < KQ - 1; ++kq) {
      frags(kt, kq + 1, (kq + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
      group(kq, kt + S - 1, kq + 1, la);
    }
    if (MAIN || kt + 1 < nk) {
      // stage kt+1 must have landed; stages kt+2 .. kt+S-1 may still be in flight
      if (MAIN || kt + S - 1 < nk) wait_vm_barrier<(S - 2) * L>(); else wait_vm_barrier<0>();
      frags(kt + 1, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    group(KQ - 1, kt + S, 0, lb);
  };
#pragma unroll
  for (int s = 0; s < S - 1; ++s)
    if (s < nk) issue(s);
  if (S - 1 <= nk) wait_vm_barrier<(S - 2) * L>(); else wait_vm_barrier<0>();
  if (S - 1 < nk) {
#pragma unroll
    for (int i = 0; i < (LQ < L ? LQ : L); ++i) issue_one(S - 1, i);
  }
  frags(0, 0, 0);
  const int n_main = max(nk - S, 0);
  for (int kt = 0; kt < n_main; ++kt) step(kt, std::true_type{});
  for (int kt = n_main; kt < nk; ++kt) step(kt, std::false_type{});

  // k-groups: group g keeps token tiles i with i % KG == g and hands the others over through LDS
  if (KG > 1) {
    static_assert(KG == 1 || (KG == 2 && TM % 2 == 0), "two k-groups need an even number of token tiles per wavefront");
    static_assert(KG == 1 || S * STAGE >= WM * WN * 2 * (TM / 2) * TN * 2 * 16 * 64 * 4, "ring too small for the hand-over");
    __syncthreads();                                    // everyone is done with the ring
    float *red = reinterpret_cast<float *>(smem);
    constexpr int PER = (TM / 2) * TN * 2 * 4;          // float4 slots a wavefront hands over
    const int slot0 = ((kgrp * (WM * WN) + wq) * PER) * 64 + lane;
    int sl = 0;
#pragma unroll
    for (int i = 0; i < TM; ++i)
      if ((i & 1) != kgrp) {                            // token tiles the other group keeps
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) {
            reinterpret_cast<float4 *>(red)[slot0 + (sl++) * 64] = make_float4(accg[i][j][4 * e4], accg[i][j][4 * e4 + 1], accg[i][j][4 * e4 + 2], accg[i][j][4 * e4 + 3]);
            reinterpret_cast<float4 *>(red)[slot0 + (sl++) * 64] = make_float4(accu[i][j][4 * e4], accu[i][j][4 * e4 + 1], accu[i][j][4 * e4 + 2], accu[i][j][4 * e4 + 3]);
          }
      }
    __syncthreads();
    const int other0 = (((1 - kgrp) * (WM * WN) + wq) * PER) * 64 + lane;
    sl = 0;
#pragma unroll
    for (int i = 0; i < TM; ++i)
      if ((i & 1) == kgrp) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) {
            const float4 g4 = reinterpret_cast<const float4 *>(red)[other0 + (sl++) * 64];
            const float4 u4 = reinterpret_cast<const float4 *>(red)[other0 + (sl++) * 64];
            accg[i][j][4 * e4] += g4.x; accg[i][j][4 * e4 + 1] += g4.y; accg[i][j][4 * e4 + 2] += g4.z; accg[i][j][4 * e4 + 3] += g4.w;
            accu[i][j][4 * e4] += u4.x; accu[i][j][4 * e4 + 1] += u4.y; accu[i][j][4 * e4 + 2] += u4.z; accu[i][j][4 * e4 + 3] += u4.w;
          }
      }
  }

  const int pos0 = n0 + wn * WNn + TN * c;
  // the usual tile: every position a selected neuron of every token row (no compensator unit, no padding, no masks)
  const bool plain = p.mask == nullptr && n0 + BNn <= Kb;
  if (pos0 < p.hs) {
    // merged lists: which sub-blocks' rows each of this lane's positions belongs to (all of them otherwise)
    uint32_t member[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j)
      member[j] = (p.mask != nullptr && pos0 + j < Kb) ? (uint32_t)p.mask[(size_t)b * p.k_stride + pos0 + j] : 0xffffffffu;
#pragma unroll
    for (int i = 0; i < TM; ++i)
      if (KG == 1 || (i & 1) == kgrp)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int rowl = (wm * TM + i) * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
        if (rowl < rows_valid) {
          const int sub = p.mask != nullptr ? ((m * BM + rowl) >> p.sub_shift) : 0;
          float hv[TN];
          if (plain) {
#pragma unroll
            for (int j = 0; j < TN; ++j) hv[j] = act_apply(FF_ACT_SILU, accg[i][j][e]) * accu[i][j][e];
          } else {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
              const int pos = pos0 + j;
              const float g = accg[i][j][e], u = accu[i][j][e];
              hv[j] = pos < Kb ? act_apply(FF_ACT_SILU, g) * u : (pos < ntot ? act_apply(p.comp_act, g) : 0.0f);
              if (!((member[j] >> sub) & 1u)) hv[j] = 0.0f;
            }
          }
          bf16_t *dst = p.h + (size_t)(t0 + rowl) * p.hs + pos0;
          if (TN == 1) {
            dst[0] = f32_to_bf16(hv[0]);
          } else {
#pragma unroll
            for (int j = 0; j < TN; j += 2)
              *reinterpret_cast<uint32_t *>(dst + j) = pack_bf16x2(hv[j], hv[j + 1]);
          }
        }
      }
  }
}

// Four adjacent outputs of one token row on their way out of the down projection: Y in fp32, Y in
// bf16, or the stack's residual add (the same two roundings as a bf16 Y followed by a separate add;
// every element of res is read and written by one lane only).  o = element offset of the first.
__device__ __forceinline__ void store_out4(const Gemm2Params &p, size_t o, float4 v) {
  if (p.res) {
    uint2 *hp = reinterpret_cast<uint2 *>(p.res + o);
    const uint2 hv = *hp;
    const float y0 = bf16_to_f32(f32_to_bf16(v.x)), y1 = bf16_to_f32(f32_to_bf16(v.y));
    const float y2 = bf16_to_f32(f32_to_bf16(v.z)), y3 = bf16_to_f32(f32_to_bf16(v.w));
    *hp = make_uint2(pack_bf16x2(bf16_to_f32((bf16_t)(hv.x & 0xffffu)) + y0, bf16_to_f32((bf16_t)(hv.x >> 16)) + y1),
                     pack_bf16x2(bf16_to_f32((bf16_t)(hv.y & 0xffffu)) + y2, bf16_to_f32((bf16_t)(hv.y >> 16)) + y3));
  } else if (p.out_f32) {
    *reinterpret_cast<float4 *>(reinterpret_cast<float *>(p.y) + o) = v;
  } else {
    *reinterpret_cast<uint2 *>(reinterpret_cast<bf16_t *>(p.y) + o) =
        make_uint2(pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w));
  }
}

// The pieces of the lists that were cut along k, added in piece order (Eq. 17, 21: the same sum in a
// fixed, documented order).  One workgroup per token row of a heavy block and 1024 columns; a thread takes
// four columns and has all pieces' loads in flight before the first add.
constexpr int kMaxPieces = 17;
__global__ __launch_bounds__(256) void ff_gemm2_reduce_kernel(Gemm2Params p) {
  const int hslot = (int)blockIdx.x / p.block, r = (int)blockIdx.x - hslot * p.block;
  const int b = heavy_block(p.k, hslot);
  const int t = b * p.block + r;
  if (t >= p.T) return;
  const size_t piece_stride = (size_t)p.block * p.d_model;
  const float *src = p.part + ((size_t)hslot * p.n_pieces * p.block + r) * p.d_model;
  const int c = p.col0 + 1024 * (int)blockIdx.y + 4 * (int)threadIdx.x;
  if (c < p.d_model) {
    float4 v[kMaxPieces];
#pragma unroll
    for (int j = 0; j < kMaxPieces; ++j)
      if (j < p.n_pieces) v[j] = *reinterpret_cast<const float4 *>(src + j * piece_stride + c);
    __builtin_amdgcn_sched_barrier(0);
    float4 s = v[0];
#pragma unroll
    for (int j = 1; j < kMaxPieces; ++j)
      if (j < p.n_pieces) { s.x += v[j].x; s.y += v[j].y; s.z += v[j].z; s.w += v[j].w; }
    store_out4(p, (size_t)t * p.d_model + c, s);
  }
}

// ============================ gemm2 =========================================
// WM x WN wavefronts; a wavefront computes 32*TM tokens x 128 output columns.  The B
// operand tile is [BK list positions][BN columns] as it lies in memory (a gathered row is
// contiguous along the columns); the k-contiguous MFMA fragments are formed by reading
// 8 rows x 4 columns per lane (ds_read_b64) and interleaving row pairs with one byte
// permute per dword.  MFMA tile f, column c holds output column wave_base + 4c + f: a lane
// ends up with 4 consecutive columns of a row.
// Same S-stage asynchronous LDS ring as gemm1.  A B wave-load is 1 KiB of gathered rows
// (1024 / (2 BN) rows).  Where the row ids come from is a template parameter RM, so that the
// loop has no branches on it: 0 = identity list (Eq. 10, or K = all), computed; 1 = the block's
// whole list (Wdown rows, then the compensator units as ids d_ffn + u, then 0 padding) is
// copied once into an LDS table of 16-bit ids behind the ring and each lane reads the id of
// the row it fills from there, one k-step ahead; 2 = scalar loads of the list through the
// constant address space, the fallback when the table does not fit; 3 = the list streams through
// a small LDS ring of raw entries, one asynchronous 256-byte copy per k-step issued three steps
// before its entries are read (any list length, 2 KB of LDS).  Nothing in the loop is tracked by
// vmcnt except the asynchronous copies themselves.
// With KG = 2 two groups of WM x WN wavefronts split each stage's k range, as in gemm1, and exchange
// halves of their accumulators through LDS at the end (fixed order): eight wavefronts on a 128 x 256
// tile, for launches that give every CU one workgroup at most.
template <int WM, int WN, int TM, int BK, int S, int RM, int KG = 1>
__global__ __launch_bounds__(WM * WN * KG * 64) __attribute__((amdgpu_waves_per_eu(TM * 4 <= 8 ? 2 : 1)))
void ff_gemm2_kernel(Gemm2Params p, int V, int mt, int N) {
  constexpr int NW = WM * WN * KG;
  constexpr int BM = WM * TM * 32;
  constexpr int BN = WN * 128;
  constexpr int CPR = BK / 8;
  constexpr int ROWB = BK * 2;
  constexpr int A_BYTES = BM * ROWB;
  constexpr int ROWB_B = BN * 2;
  constexpr int B_BYTES = BK * ROWB_B;
  constexpr int STAGE = A_BYTES + B_BYTES;
  constexpr int RPLA = 1024 / ROWB;     // A rows per wave-load
  constexpr int RPLB = 1024 / ROWB_B;   // B rows per wave-load
  constexpr int LPR = 64 / RPLB;        // lanes per B row in a wave-load
  constexpr int LA = A_BYTES / 1024 / NW, LB = B_BYTES / 1024 / NW;
  constexpr int L = LA + LB;
  static_assert(ROWB_B <= 1024, "a B tile row must fit one wave-load");
  static_assert(A_BYTES % (1024 * NW) == 0 && B_BYTES % (1024 * NW) == 0, "tiles must split evenly over the wavefronts");
  extern __shared__ __align__(16) uint8_t smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kgrp = wave / (WM * WN), wq = wave % (WM * WN);
  const int wm = wq / WN, wn = wq % WN;
  const int c = lane & 31, half = lane >> 5;

  // The heavy blocks' tiles (the longest k loops) take the first ids, then everybody else's.  With
  // n_pieces > 0 a heavy block's list is cut along k instead: its first cut0 positions are a tile like
  // everybody else's (piece 0, in the common region), the rest goes to n_pieces - 1 short tiles of
  // piece_len positions with the first ids, and every piece writes fp32 partial sums that
  // ff_gemm2_reduce_kernel adds up in a fixed order.
  TileCoord tc;
  const int n_surplus = p.n_pieces > 0 ? p.n_pieces - 1 : 1;
  const int n_first = p.k.n_heavy * mt * N * n_surplus;
  int piece = -1, hslot = 0;   // piece of a cut list (-1: a whole list), and which heavy block
  if ((int)blockIdx.x < n_first) {
    // id = ((surplus piece * heavy virtual blocks) + heavy virtual block) * N + column tile
    const int hv = p.k.n_heavy * mt;
    const int hn = __builtin_amdgcn_readfirstlane((int)blockIdx.x / N);
    const int sp = __builtin_amdgcn_readfirstlane(hn / hv);
    const int h = hn - sp * hv;
    hslot = __builtin_amdgcn_readfirstlane(h / mt);
    tc.vb = heavy_block(p.k, hslot) * mt + (h - hslot * mt);
    tc.nt = (int)blockIdx.x - hn * N;
    tc.valid = true;
    if (p.n_pieces > 0) piece = 1 + sp;
  } else {
    tc = map_tile((int)blockIdx.x - n_first, V, N);
    if (tc.valid && p.k.n_heavy > 0) {
      const int hi = heavy_index(p.k, tc.vb / mt);
      if (hi >= 0) {
        if (p.n_pieces == 0) return;
        piece = 0;
        hslot = hi;
      }
    }
  }
  if (!tc.valid) return;
  tc.vb = __builtin_amdgcn_readfirstlane(tc.vb);   // wave-uniform by construction
  tc.nt = __builtin_amdgcn_readfirstlane(tc.nt);
  piece = __builtin_amdgcn_readfirstlane(piece);
  hslot = __builtin_amdgcn_readfirstlane(hslot);
  const int b = tc.vb / mt, m = tc.vb - b * mt;
  const int t0 = b * p.block + m * BM;
  const int rows_valid = min(p.T, (b + 1) * p.block) - t0;
  if (rows_valid <= 0) return;
  const int Kb = block_k(p.k, b, p.d_ffn, p.k_stride, p.idx != nullptr);
  const int ntot = Kb + p.rc;
  const int n0 = p.col0 + tc.nt * BN;
  // list positions [kofs, kend) of this tile (kofs a multiple of 64; an empty range gives zeros)
  int kofs = 0, kend = ntot;
  if (piece == 0) kend = min(ntot, p.cut0);
  if (piece > 0) {
    kofs = min(p.cut0 + (piece - 1) * p.piece_len, (ntot + 63) / 64 * 64);
    kend = min(ntot, p.cut0 + piece * p.piece_len);
  }
  kofs = __builtin_amdgcn_readfirstlane(kofs);
  const int nk = __builtin_amdgcn_readfirstlane(max(kend - kofs + BK - 1, 0) / BK);

  const bf16_t *a_src[LA];
#pragma unroll
  for (int i = 0; i < LA; ++i) {
    const int trow = (wave + i * NW) * RPLA + lane / CPR;
    const int ch = (lane % CPR) ^ swz<BK>(trow);
    const int tok = t0 + min(trow, rows_valid - 1);
    a_src[i] = p.h + (size_t)tok * p.hs + kofs + ch * 8;
  }
  const int b_sub = lane / LPR;                                   // which of the wave-load's rows this lane fills
  const int b_col = min(n0 + (lane % LPR) * 8, p.d_model - 8);
  typedef const __attribute__((address_space(4))) int32_t *cidx_t;
  const cidx_t idx_row = RM == 2 ? (cidx_t)(p.idx + (size_t)b * p.k_stride) : (cidx_t) nullptr;
  // source row id of list position pos: < d_ffn -> Wdown row, else compensator unit
  auto src_row = [&](int pos, auto load) __attribute__((always_inline)) -> int {
    if (pos < Kb) return min(max(load(pos), 0), p.d_ffn - 1);
    return pos < ntot ? p.d_ffn + (pos - Kb) : 0;
  };
  uint16_t *tab = reinterpret_cast<uint16_t *>(smem + S * STAGE);
  if (RM == 1) {
    // eight list entries per thread in flight at a time (left to itself the loop waits for every load)
    const int32_t *gl = p.idx + (size_t)b * p.k_stride;
    constexpr int U = 8;
    for (int i0 = tid; i0 < nk * BK; i0 += U * NW * 64) {
      int raw[U];
#pragma unroll
      for (int u = 0; u < U; ++u) raw[u] = gl[min(kofs + i0 + u * NW * 64, Kb - 1)];
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = i0 + u * NW * 64;
        if (i < nk * BK) tab[i] = (uint16_t)src_row(kofs + i, [&](int) { return raw[u]; });
      }
    }
    __syncthreads();
  }
  // RM 3: ring of kIdSlots stages' raw list entries behind the operand ring.  Every wavefront issues
  // the same copy (identical bytes to the same place), so all of them count the same number of
  // outstanding loads.  Lane l fetches entry st * BK + l % BK, clamped into the list.
  constexpr int kIdSlots = 8;
  static_assert(RM != 3 || S + 2 <= kIdSlots - 2, "id ring too short for the ring depth");
  const int32_t *idring = reinterpret_cast<const int32_t *>(smem + S * STAGE);
  const uint32_t idring_lds = lds_addr_of(smem) + (uint32_t)(S * STAGE);
  const int32_t *id_src = p.idx + (size_t)b * p.k_stride;
  auto issue_ids = [&](int st) __attribute__((always_inline)) {
    const int q = min(kofs + st * BK + lane % BK, Kb - 1);
    gload_lds4(id_src + q, idring_lds + (uint32_t)(st % kIdSlots) * 256u);
  };
  if (RM == 3) {
    // stages 0 .. S+1 up front; stage j+S+2 follows in step j, right behind that step's barrier
#pragma unroll
    for (int st = 0; st < S + 2; ++st) issue_ids(st);
    wait_vm_barrier<0>();
  }
  // A VGPR zero the compiler cannot see through: keeps the table reads per-lane LDS reads
  // (a wave-uniform address would be turned into a read + wait + readfirstlane in the loop).
  int lane_zero;
  asm volatile("v_mov_b32 %0, 0" : "=v"(lane_zero));
  // rows_v: row id of the B row this lane fills in copy i of the stage issued next; rows_n: the
  // same for the stage after it, fetched a whole step before it is needed
  int rows_v[LB], rows_n[LB];
  auto fetch_rows = [&](int st, int (&dst)[LB]) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < LB; ++i) {
      const int rel0 = st * BK + (wave + i * NW) * RPLB;   // within this tile's k range
      const int pos0 = kofs + rel0;
      if (RM == 0) {
        dst[i] = src_row(pos0 + b_sub, [](int q) { return q; });
      } else if (RM == 1) {
        dst[i] = (int)tab[rel0 + b_sub + lane_zero];
      } else if (RM == 3) {
        const int raw = idring[(st % kIdSlots) * 64 + (wave + i * NW) * RPLB + b_sub + lane_zero];
        dst[i] = src_row(pos0 + b_sub, [&](int) { return raw; });
      } else {
        int r = src_row(pos0, [&](int q) { return idx_row[q]; });
#pragma unroll
        for (int u = 1; u < RPLB; ++u) {
          const int ru = src_row(pos0 + u, [&](int q) { return idx_row[q]; });
          r = (b_sub == u) ? ru : r;
        }
        dst[i] = r;
      }
    }
  };
  const uint32_t lds0 = lds_addr_of(smem);
  const uint32_t row_bytes = (uint32_t)p.d_model * 2u;
  const uint64_t base_w = reinterpret_cast<uint64_t>(p.wd + b_col);
  const uint64_t base_c = reinterpret_cast<uint64_t>(p.wc2 + b_col) - (uint64_t)p.d_ffn * row_bytes;
  // copy i of stage st (uses rows == row ids of stage st): i < LA -> A tile, else gathered B rows
  auto issue_one = [&](int st, int i) __attribute__((always_inline)) {
    const uint32_t base = lds0 + (uint32_t)(st % S) * STAGE + (uint32_t)wave * 1024u;
    if (i < LA) {
      gload_lds16(a_src[i] + st * BK, base + (uint32_t)i * (NW * 1024u));
    } else {
      const int ib = i - LA;
      // row id r < d_ffn: Wdown row r; else compensator unit r - d_ffn.  One compare, one 64-bit
      // select and one 32 x 32 + 64 multiply-add per copy (this arithmetic sits between the MFMAs).
      const uint32_t r = (uint32_t)rows_v[ib];
      const uint64_t src = (uint64_t)r * row_bytes + (r < (uint32_t)p.d_ffn ? base_w : base_c);
      gload_lds16(reinterpret_cast<const void *>(src), base + A_BYTES + (uint32_t)ib * (NW * 1024u));
    }
  };
  auto issue = [&](int st) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < L; ++i) issue_one(st, i);
  };

  f32x16_t acc[TM][4];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][f][e] = 0.0f;

  // Same pipeline as gemm1: stage kt+1 is waited for in front of the last MFMA group of stage
  // kt, its first fragments are requested there, and the copies of stage kt+S go out one at a
  // time between the MFMAs of the following KQ groups.  The row ids of stage kt+S are fetched
  // at the start of step kt and take the place of stage kt+S-1's once its last copy is out.
  constexpr int KQ = BK / 16 / KG;                     // MFMA groups (16 k each) per stage and k-group
  static_assert(KQ % 2 == 0, "fragment double buffer needs an even number of groups per stage");
  constexpr int NMF = TM * 4;
  constexpr int LQ = (L + KQ - 1) / KQ;
  constexpr int PER = (LQ + NMF - 1) / NMF;
  constexpr int EVERY = NMF / LQ > 0 ? NMF / LQ : 1;
  constexpr int SLOTS = (NMF + EVERY - 1) / EVERY * PER;
  u32x4_t af[2][TM];
  u32x2_t d[2][8];
  auto frags = [&](int kt, int kk, int buf) __attribute__((always_inline)) {
    const uint8_t *cur = smem + (kt % S) * STAGE;
    const int kg = kgrp * KQ + kk;                     // 16-k group within the stage
    const int q = 2 * kg + half;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int row = (wm * TM + i) * 32 + c;
      af[buf][i] = *reinterpret_cast<const u32x4_t *>(cur + row * ROWB + ((q ^ swz<BK>(row)) << 4));
    }
    const uint8_t *bb = cur + A_BYTES + (kg * 16 + 8 * half) * ROWB_B + (wn * 128 + 4 * c) * 2;
#pragma unroll
    for (int i = 0; i < 8; ++i) d[buf][i] = *reinterpret_cast<const u32x2_t *>(bb + i * ROWB_B);
  };
  auto group = [&](int kk, int st, int part, bool load) __attribute__((always_inline)) {
    const u32x2_t *dd = d[kk & 1];
    u32x4_t bf[4];
    // One byte permute per dword: low halves (even columns) or high halves (odd columns) of the
    // rows (2j, 2j+1), lower row in the low half.  The four permutes of column tile f are issued
    // right in front of its first MFMA, so all but the first four hide under the previous MFMA.
#define FF_LO(e, o) __builtin_amdgcn_perm((o), (e), 0x05040100u)
#define FF_HI(e, o) __builtin_amdgcn_perm((o), (e), 0x07060302u)
    auto make_bf = [&](int f) __attribute__((always_inline)) {
      if (f == 0) bf[0] = mk4(FF_LO(dd[0].x, dd[1].x), FF_LO(dd[2].x, dd[3].x), FF_LO(dd[4].x, dd[5].x), FF_LO(dd[6].x, dd[7].x));
      if (f == 1) bf[1] = mk4(FF_HI(dd[0].x, dd[1].x), FF_HI(dd[2].x, dd[3].x), FF_HI(dd[4].x, dd[5].x), FF_HI(dd[6].x, dd[7].x));
      if (f == 2) bf[2] = mk4(FF_LO(dd[0].y, dd[1].y), FF_LO(dd[2].y, dd[3].y), FF_LO(dd[4].y, dd[5].y), FF_LO(dd[6].y, dd[7].y));
      if (f == 3) bf[3] = mk4(FF_HI(dd[0].y, dd[1].y), FF_HI(dd[2].y, dd[3].y), FF_HI(dd[4].y, dd[5].y), FF_HI(dd[6].y, dd[7].y));
    };
    // (with a gathered list the copies' address arithmetic already fills those slots, and spreading
    //  the permutes as well measured 5% slower; with the identity list it is 6% faster)
    constexpr bool SPREAD_PERM = RM == 0;
    make_bf(0);
    if (!SPREAD_PERM) { make_bf(1); make_bf(2); make_bf(3); }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int f = 0; f < 4; ++f) {
        acc[i][f] = mfma32(af[kk & 1][i], bf[f], acc[i][f]);
        if (SPREAD_PERM && i == 0 && f < 3) make_bf(f + 1);
        bool fenced = false;
        if ((i * 4 + f) % EVERY == 0) {
#pragma unroll
          for (int r = 0; r < PER; ++r) {
            const int n = (i * 4 + f) / EVERY * PER + r;
            if (n < LQ && part * LQ + n < L) {
              if (load) issue_one(st, part * LQ + n);
              __builtin_amdgcn_sched_barrier(0);
              fenced = true;
            }
          }
        }
        if (SPREAD_PERM && i == 0 && !fenced) __builtin_amdgcn_sched_barrier(0);
      }
#undef FF_LO
#undef FF_HI
#pragma unroll
    for (int n = SLOTS; n < LQ; ++n)
      if (load && part * LQ + n < L) issue_one(st, part * LQ + n);
    __builtin_amdgcn_sched_barrier(0);
  };
  // MAIN: stages kt+S-1 and kt+S both exist (no conditions in the loop body)
  auto step = [&](int kt, auto main_tag) __attribute__((always_inline)) {
    constexpr bool MAIN = decltype(main_tag)::value;
    const bool la = MAIN || kt + S - 1 < nk;
    const bool lb = MAIN || kt + S < nk;
    if (lb) fetch_rows(kt + S, rows_n);
#pragma unroll
    for (int kk = 0; kk < KQ - 1; ++kk) {
      frags(kt, kk + 1, (kk + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
      group(kk, kt + S - 1, kk + 1, la);
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) rows_v[i] = rows_n[i];   // the last copy of stage kt+S-1 is out
    if (MAIN || kt + 1 < nk) {
      // stage kt+1 must have landed; stages kt+2 .. kt+S-1 may still be in flight
      if (MAIN || kt + S - 1 < nk) wait_vm_barrier<(S - 2) * L>(); else wait_vm_barrier<0>();
      frags(kt + 1, 0, 0);
      // older than every copy the next wait lets stay in flight, so it has landed by then, one
      // step before fetch_rows reads it
      if (RM == 3) issue_ids(kt + S + 2);
    }
    __builtin_amdgcn_sched_barrier(0);
    group(KQ - 1, kt + S, 0, lb);
  };
#pragma unroll
  for (int s = 0; s < S - 1; ++s)
    if (s < nk) {
      fetch_rows(s, rows_v);
      issue(s);
    }
  if (S - 1 < nk) fetch_rows(S - 1, rows_v);
#pragma unroll
  for (int i = 0; i < LB; ++i) rows_n[i] = rows_v[i];
  if (S - 1 <= nk) wait_vm_barrier<(S - 2) * L>(); else wait_vm_barrier<0>();
  if (S - 1 < nk) {
#pragma unroll
    for (int i = 0; i < (LQ < L ? LQ : L); ++i) issue_one(S - 1, i);
  }
  frags(0, 0, 0);
  const int n_main = max(nk - S, 0);
  for (int kt = 0; kt < n_main; ++kt) step(kt, std::true_type{});
  for (int kt = n_main; kt < nk; ++kt) step(kt, std::false_type{});
  if (RM == 3) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the last id copies (nobody reads them)

  // k-groups: group g keeps token tiles i with i % KG == g and hands the others over through LDS
  if (KG > 1) {
    static_assert(KG == 1 || (KG == 2 && TM % 2 == 0), "two k-groups need an even number of token tiles per wavefront");
    static_assert(KG == 1 || S * STAGE >= WM * WN * 2 * (TM / 2) * 4 * 16 * 64 * 4, "ring too small for the hand-over");
    __syncthreads();                                    // everyone is done with the ring
    float4 *red = reinterpret_cast<float4 *>(smem);
    constexpr int XPER = (TM / 2) * 4 * 4;              // float4 slots a wavefront hands over
    const int slot0 = ((kgrp * (WM * WN) + wq) * XPER) * 64 + lane;
    int sl = 0;
#pragma unroll
    for (int i = 0; i < TM; ++i)
      if ((i & 1) != kgrp) {                            // token tiles the other group keeps
#pragma unroll
        for (int f = 0; f < 4; ++f)
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4)
            red[slot0 + (sl++) * 64] = make_float4(acc[i][f][4 * e4], acc[i][f][4 * e4 + 1], acc[i][f][4 * e4 + 2], acc[i][f][4 * e4 + 3]);
      }
    __syncthreads();
    const int other0 = (((1 - kgrp) * (WM * WN) + wq) * XPER) * 64 + lane;
    sl = 0;
#pragma unroll
    for (int i = 0; i < TM; ++i)
      if ((i & 1) == kgrp) {
#pragma unroll
        for (int f = 0; f < 4; ++f)
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) {
            const float4 o4 = red[other0 + (sl++) * 64];
            acc[i][f][4 * e4] += o4.x; acc[i][f][4 * e4 + 1] += o4.y; acc[i][f][4 * e4 + 2] += o4.z; acc[i][f][4 * e4 + 3] += o4.w;
          }
      }
  }

  const int col = n0 + wn * 128 + 4 * c;
  if (col < p.d_model) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
      if (KG == 1 || (i & 1) == kgrp)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int rowl = (wm * TM + i) * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
        if (rowl < rows_valid) {
          const float4 v = make_float4(acc[i][0][e], acc[i][1][e], acc[i][2][e], acc[i][3][e]);
          if (piece >= 0) {
            const size_t prow = ((size_t)hslot * p.n_pieces + piece) * p.block + (m * BM + rowl);
            *reinterpret_cast<float4 *>(p.part + prow * p.d_model + col) = v;
          } else {
            store_out4(p, (size_t)(t0 + rowl) * p.d_model + col, v);
          }
        }
      }
  }
}

// ---- variant tables --------------------------------------------------------
struct Variant {
  const void *fn;
  int bm, bn, threads, lds;
  const void *fn_rm[3];  // gemm2 only: the kernels for row-id modes 1, 2 and (or nullptr) 3 (fn is mode 0)
};
int g_lds_limit = 65536;

template <int WM, int WN, int TM, int TN, int BK, int S, int KG = 1>
Variant g1() {
  return Variant{reinterpret_cast<const void *>(&ff_gemm1_kernel<WM, WN, TM, TN, BK, S, KG>), WM * TM * 32,
                 WN * TN * 32, WM * WN * KG * 64, S * (WM * TM * 32 + 2 * WN * TN * 32) * BK * 2, {nullptr, nullptr, nullptr}};
}
template <int WM, int WN, int TM, int BK, int S, int KG = 1>
Variant g2() {
  return Variant{reinterpret_cast<const void *>(&ff_gemm2_kernel<WM, WN, TM, BK, S, 0, KG>), WM * TM * 32,
                 WN * 128, WM * WN * KG * 64, S * (WM * TM * 32 * BK * 2 + BK * WN * 128 * 2),
                 {reinterpret_cast<const void *>(&ff_gemm2_kernel<WM, WN, TM, BK, S, 1, KG>),
                  reinterpret_cast<const void *>(&ff_gemm2_kernel<WM, WN, TM, BK, S, 2, KG>),
                  // the streamed list only where the table may not fit and scalar loads cost too much
                  KG > 1 ? reinterpret_cast<const void *>(&ff_gemm2_kernel<WM, WN, TM, BK, S, (KG > 1 ? 3 : 2), KG>) : nullptr}};
}
constexpr int kIdRingBytes = 8 * 256;   // row-id mode 3: eight stages of 64 raw list entries

// tokens x list positions of the tile, wavefronts, BK, ring stages (LDS)
const Variant kGemm1[] = {
    g1<2, 2, 2, 2, 64, 3, 2>(),  // 0: 128 x 128, 8 waves in 2 k-groups, BK 64, 3 stages (144 KB)
    g1<2, 4, 2, 2, 32, 3>(),     // 1: 128 x 256, 8 waves, BK 32, 3 stages (120 KB)
    g1<2, 2, 2, 2, 32, 3>(),     // 2: 128 x 128, 4 waves, BK 32, 3 stages (72 KB, two workgroups per CU)
    g1<4, 2, 2, 2, 64, 2>(),     // 3: 256 x 128, 8 waves, BK 64, 2 stages (128 KB)
    g1<1, 4, 2, 2, 32, 4>(),     // 4: 64 x 256, 4 waves, BK 32, 4 stages (144 KB)
    g1<1, 4, 2, 2, 64, 2, 2>(),  // 5: 64 x 256, 8 waves in 2 k-groups, BK 64, 2 stages (144 KB)
    g1<2, 4, 2, 2, 64, 2>(),     // 6: 128 x 256, 8 waves, BK 64, 2 stages (160 KB)
    g1<2, 2, 1, 1, 64, 6>(),     // 7: 64 x 64, 4 waves, BK 64, 6 stages (144 KB): remainder tile, latency-bound, deep ring
    g1<2, 2, 2, 1, 64, 4>(),     // 8: 128 x 64, 4 waves, BK 64, 4 stages (128 KB; 2 stages: 67 against 48 us on 224 tiles): the heavy blocks' surplus
    // (tiles whose wavefronts need 256 accumulator registers -- 128 x 256 or 256 x 128 on 4 waves -- were measured
    //  10-25% slower: one wavefront per SIMD cannot keep the matrix pipe issuing back to back)
};
// tokens x output columns of the tile
const Variant kGemm2[] = {
    g2<2, 4, 2, 32, 3>(),  // 0: 128 x 512, 8 waves, 3 stages (120 KB)
    g2<2, 2, 2, 32, 3>(),  // 1: 128 x 256, 4 waves, 3 stages (72 KB)
    g2<4, 2, 2, 32, 3>(),  // 2: 256 x 256, 8 waves, 3 stages (96 KB)
    g2<1, 4, 2, 32, 3>(),  // 3: 64 x 512, 4 waves, 3 stages (108 KB)
    g2<2, 2, 2, 64, 3, 2>(),  // 4: 128 x 256, 8 waves in 2 k-groups, BK 64, 3 stages (144 KB)
};
constexpr int kNumGemm1 = sizeof(kGemm1) / sizeof(Variant);
constexpr int kNumGemm2 = sizeof(kGemm2) / sizeof(Variant);

// Tile choice: the largest M tile the block size fills; among those the first in
// preference order that still gives (nearly) every CU a workgroup.
int choose(const Variant *tab, const int *pref, int n_pref, int block, int n_blocks, int n_extent) {
  int best = pref[0], best_tiles = -1;
  for (int i = 0; i < n_pref; ++i) {
    const Variant &v = tab[pref[i]];
    const int tiles = n_blocks * ((block + v.bm - 1) / v.bm) * ((n_extent + v.bn - 1) / v.bn);
    if (tiles >= 224) return pref[i];
    if (tiles > best_tiles) { best = pref[i]; best_tiles = tiles; }
  }
  return best;
}

}  // namespace

int ff_gemm1_num_variants() { return kNumGemm1; }
int ff_gemm2_num_variants() { return kNumGemm2; }

hipError_t ff_gemm_init(int lds_limit) {
  g_lds_limit = lds_limit;
  for (int i = 0; i < kNumGemm1; ++i) {
    if (kGemm1[i].lds > lds_limit) continue;  // not launchable on this device
    hipError_t e = hipFuncSetAttribute(kGemm1[i].fn, hipFuncAttributeMaxDynamicSharedMemorySize, kGemm1[i].lds);
    if (e != hipSuccess) return e;
  }
  for (int i = 0; i < kNumGemm2; ++i) {  // the ring plus, when there is room, the row-id table
    const void *fns[4] = {kGemm2[i].fn, kGemm2[i].fn_rm[0], kGemm2[i].fn_rm[1], kGemm2[i].fn_rm[2]};
    for (const void *fn : fns) {
      if (fn == nullptr) continue;
      hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds_limit);
      if (e != hipSuccess) return e;
    }
  }
  return hipSuccess;
}

// V virtual blocks (each block cut into M tiles of v.bm tokens) x N tiles, preceded by the
// heavy blocks' n_first_per_vb tiles each
static hipError_t launch_variant(const Variant &v, const void *fn, const void *params, int block, int n_blocks,
                                 int N, int n_heavy, int n_first_per_vb, bool gemm1, hipStream_t s) {
  int mt = (block + v.bm - 1) / v.bm;
  int V = n_blocks * mt;
  int NX = n_first_per_vb;
  int grid = n_heavy * mt * n_first_per_vb + 8 * ((V + 7) / 8) * N;
  if (grid <= 0) return hipSuccess;
  void *args1[] = {const_cast<void *>(params), &V, &mt, &N, &NX};
  void *args2[] = {const_cast<void *>(params), &V, &mt, &N};
  return hipLaunchKernel(fn, dim3(grid), dim3(v.threads), gemm1 ? args1 : args2, v.lds, s);
}

constexpr int kRemainderVariant = 7;
constexpr int kHeavySurplusVariant = 8;
constexpr int kWide128 = 6;
constexpr int kNumCU = 256;

hipError_t ff_launch_gemm1(const Gemm1Params &p, int variant, int split, int heavy_tiles, hipStream_t s) {
  static const int p64[] = {5, 4}, p128[] = {0, 2, 1}, p256[] = {3, 2, 1};
  const int n_extent = p.k.k_max + p.rc;                  // longest list
  const bool ragged = p.k.per_block != nullptr;           // lists of unequal length
  const int base_extent = (p.k.n_heavy > 0 ? p.k.k_base : p.k.k_max) + p.rc;   // what all but the heavy blocks have
  const bool chosen = variant < 0;
  if (variant < 0) {
    if (p.block >= 256) variant = choose(kGemm1, p256, 3, p.block, p.n_blocks, base_extent);
    else if (p.block > 64) {
      variant = choose(kGemm1, p128, 3, p.block, p.n_blocks, base_extent);
      // The 128 x 256 tile moves fewer bytes per FLOP; its part-filled last tile goes to the remainder
      // launch (with lists of unequal length every block's own).  Against the 128 x 128 two-k-group tile, in
      // rounds of 256 workgroups of the wide tile's duration: whole rounds of full wide tiles plus 0.22 per
      // round of remainder tiles, against whole rounds of the smaller tile at 0.52 each.  (Measured, wide
      // against small: 4096/14336 x 64 blocks K 7168 0.888 / 0.916 ms, K 7300 0.895 / 0.920, K 3584 -- 3.5
      // rounds of wide tiles -- 0.520 / 0.490; 3584/18944 x 128 blocks K 13126 2.75 / 2.86; 2048/8192 x 32
      // blocks K 4200 0.155 / 0.172.)
      const Variant &w = kGemm1[kWide128];
      const int rem_w = base_extent % w.bn;
      const long wide_full = (long)p.n_blocks * (base_extent / w.bn);
      const long rem_wgs = (long)p.n_blocks * 2 * ((rem_w + 63) / 64);
      const double cost_wide = (double)((wide_full + kNumCU - 1) / kNumCU) + 0.22 * (double)((rem_wgs + kNumCU - 1) / kNumCU);
      const double cost_small = 0.52 * (double)(((long)p.n_blocks * ((base_extent + 127) / 128) + kNumCU - 1) / kNumCU);
      if (split != 0 && w.lds <= g_lds_limit && base_extent >= w.bn && (ragged || cost_wide <= cost_small) && wide_full >= 224) {
        variant = kWide128;
        if (rem_w > 0 || ragged) split = 1;
      }
    } else variant = choose(kGemm1, p64, 2, p.block, p.n_blocks, base_extent);
  }
  if (variant >= kNumGemm1 || kGemm1[variant].lds > g_lds_limit) return hipErrorInvalidValue;
  const Variant &v = kGemm1[variant];
  Gemm1Params q = p;
  q.full_only = 0;
  q.rem_bn = 0;
  // The positions beyond a block's last full N tile (the compensator's units, typically) would
  // cost the block a whole extra tile.  When that extra tile starts a new round of workgroups
  // over the CUs, they go to a second launch with 64 x 64 tiles instead, which spreads that
  // little work over the whole chip.
  const int rem = n_extent % v.bn;
  bool do_split = false;
  if ((chosen ? split != 0 : split > 0) && (rem > 0 || ragged) && n_extent >= v.bn && variant != kRemainderVariant) {
    const int n_full = base_extent / v.bn;
    const int per_cu = g_lds_limit / v.lds > 0 ? (g_lds_limit / v.lds > 2 ? 2 : g_lds_limit / v.lds) : 1;
    const int slots = kNumCU * per_cu;
    const long vb = (long)p.n_blocks * ((p.block + v.bm - 1) / v.bm);
    const long rounds_all = (vb * (n_full + 1) + slots - 1) / slots;
    const long rounds_full = (vb * n_full + slots - 1) / slots;
    do_split = split > 0 || (rounds_full < rounds_all && 2 * (base_extent % v.bn) <= v.bn);
  }
  const int heavy = p.k.n_heavy;
  if (!do_split) {
    const int N = (base_extent + v.bn - 1) / v.bn, N_all = (n_extent + v.bn - 1) / v.bn;
    return launch_variant(v, v.fn, &q, p.block, p.n_blocks, N, heavy, N_all - N, true, s);
  }
  q.full_only = 1;
  const int N = base_extent / v.bn, N_all = n_extent / v.bn;
  // The heavy blocks' positions beyond the common length.  As tiles of the main launch (with the first ids)
  // they start one more round of workgroups on a mostly idle chip; up to half a round of them run instead
  // as a launch of their own with 128 x 64 tiles, which spreads them over all of it
  // (first and last block dense on 4096/14336, 64 blocks: 0.952 -> 0.920 ms for the three launches).
  const Variant &hv = kGemm1[kHeavySurplusVariant];
  // the remainder's tile: 64 x 64 with a deep ring while that is what it takes to give every CU a workgroup,
  // 128 x 64 (fewer bytes per FLOP) once those fill the chip as well
  const int rem_est = ragged ? (heavy > 0 ? base_extent % v.bn : v.bn / 2) : rem;
  const bool rem_wide = hv.bm <= v.bm && variant != kHeavySurplusVariant &&
                        (long)p.n_blocks * ((p.block + hv.bm - 1) / hv.bm) * ((rem_est + hv.bn - 1) / hv.bn) >= kNumCU;
  const Variant &r = kGemm1[rem_wide ? kHeavySurplusVariant : kRemainderVariant];
  const long surplus_tiles = (long)heavy * ((p.block + v.bm - 1) / v.bm) * (N_all - N);
  const bool heavy_small = heavy > 0 && surplus_tiles > 0 && hv.bm <= v.bm && variant != kHeavySurplusVariant &&
                           (heavy_tiles > 0 || (heavy_tiles < 0 && 2 * surplus_tiles <= kNumCU));
  {
    hipError_t e = launch_variant(v, v.fn, &q, p.block, p.n_blocks, N, heavy, heavy_small ? 0 : N_all - N, true, s);
    if (e != hipSuccess) return e;
  }
  q.full_only = 0;
  q.rem_bn = v.bn;
  if (heavy_small) {
    // everything of a heavy block from where the main launch stopped, its part-filled last tile included
    Gemm1Params qh = q;
    qh.rem_cap = N * v.bn;
    hipError_t e = launch_variant(hv, hv.fn, &qh, p.block, p.n_blocks, 0, heavy, (n_extent - qh.rem_cap + hv.bn - 1) / hv.bn, true, s);
    if (e != hipSuccess) return e;
    q.skip_heavy = 1;
  }
  q.k.n_heavy = heavy_small ? q.k.n_heavy : 0;   // every block has at most one part-filled tile: no heavy region
  const int rem_max = ragged ? v.bn - 1 : rem;
  return launch_variant(r, r.fn, &q, p.block, p.n_blocks, (rem_max + r.bn - 1) / r.bn, 0, 0, true, s);
}

constexpr int kHalf128Wide = 4;     // the 128 x 256 down-GEMM tile with eight wavefronts (144 KB)

constexpr int kMaxShortPieces = kMaxPieces - 1;
constexpr size_t kPartCapBytes = (size_t)48 << 20;

size_t ff_gemm2_part_bytes(int n_tokens, int block, int d_model) {
  if (n_tokens <= block) return 0;   // one block: nothing is longer than the rest
  const size_t want = (size_t)2 * kMaxPieces * block * d_model * sizeof(float);
  return want < kPartCapBytes ? want : kPartCapBytes;
}

hipError_t ff_launch_gemm2(const Gemm2Params &p, int variant, int split, int row_mode, int ksplit, hipStream_t s) {
  // row ids: computed for the identity list; else from an LDS table of 16-bit ids behind the
  // ring when it fits (ids run up to d_ffn + rc - 1), else by scalar loads
  const int n_pad = (p.k.k_max + p.rc + 63) / 64 * 64;   // whole k-steps of the longest BK
  const int tab_bytes = ((2 * n_pad + 15) / 16) * 16;
  // the eight-wavefront 128 x 256 tile leaves 16 KB for that table; a longer list streams through
  // a small LDS ring instead (row-id mode 3)
  const int half128 = kHalf128Wide;
  const int p64[] = {3}, p128[] = {0, half128, 1}, p256[] = {2, 0, half128, 1};
  const bool chosen = variant < 0;
  if (variant < 0) {
    if (p.block >= 256) variant = choose(kGemm2, p256, 4, p.block, p.n_blocks, p.d_model);
    else if (p.block > 64) variant = choose(kGemm2, p128, 3, p.block, p.n_blocks, p.d_model);
    else variant = choose(kGemm2, p64, 1, p.block, p.n_blocks, p.d_model);
  }
  if (variant >= kNumGemm2) return hipErrorInvalidValue;
  Gemm2Params q = p;
  // row_mode > 0 forces one source of the row ids where the tile has it and it fits (else fn = nullptr)
  auto with_row_mode = [&](Variant v) {
    if (p.idx != nullptr) {
      const bool table_fits = p.d_ffn + p.rc <= 65536 && v.lds + tab_bytes <= g_lds_limit;
      const bool ring_fits = v.fn_rm[2] != nullptr && v.lds + kIdRingBytes <= g_lds_limit;
      const int mode = row_mode > 0 ? row_mode : (table_fits ? 1 : (ring_fits ? 3 : 2));
      if (mode == 1 && table_fits) {
        v.lds += tab_bytes;
        v.fn = v.fn_rm[0];
      } else if (mode == 3 && ring_fits) {
        v.lds += kIdRingBytes;
        v.fn = v.fn_rm[2];
      } else if (mode == 2) {
        v.fn = v.fn_rm[1];
      } else {
        v.fn = nullptr;
      }
    }
    return v;
  };
  const Variant v = with_row_mode(kGemm2[variant]);
  if (v.fn == nullptr) return hipErrorInvalidValue;
  const int N = (p.d_model + v.bn - 1) / v.bn;
  // Heavy blocks first only when their k loops are much longer (a dense block among half-sparse
  // ones): moving their tiles off their own XCD costs that XCD's even share of tiles, which
  // for a slightly longer list is all loss (measured 0.48 -> 0.63 ms for one list one longer).
  // Cut along k instead, the long lists cost their XCD nothing, which is worth it from an eighth longer on:
  // the surplus over the common length becomes short pieces, as many as give every CU one (they start at
  // once and take a fraction of a tile time), no shorter than 256 positions, no more than p.part has room for.
  const int cut0 = (p.k.k_base + p.rc + 63) / 64 * 64;
  const int surplus = n_pad - cut0;
  if (ksplit != 0 && split != 1 && p.part != nullptr && p.k.n_heavy > 0 && 8L * surplus >= cut0) {
    const long heavy_tiles = (long)p.k.n_heavy * ((p.block + v.bm - 1) / v.bm) * N;
    const size_t per_piece = (size_t)p.k.n_heavy * p.block * p.d_model * sizeof(float);
    long want = ksplit > 0 ? ksplit : kNumCU / heavy_tiles;
    want = std::min<long>(want, kMaxShortPieces);
    want = std::min<long>(want, (long)(p.part_bytes / per_piece) - 1);
    if (want >= (ksplit > 0 ? 1 : 2)) {
      const int len = std::max(256, (int)((surplus + want - 1) / want + 63) / 64 * 64);
      q.piece_len = len;
      q.cut0 = cut0;
      q.n_pieces = 1 + (surplus + len - 1) / len;
    }
  }
  if (q.n_pieces == 0 && 2L * (p.k.k_max + p.rc) < 3L * (p.k.k_base + p.rc)) q.k.n_heavy = 0;
  // Equal tiles in whole rounds: V x N tiles on kNumCU CUs take ceil(V N / kNumCU) tile times, and a last
  // round that is at most half full wastes the rest of the chip (3584 columns, 128 blocks: 896 tiles,
  // 3.5 rounds).  Then the last nq column tiles of every block leave the main launch, which
  // becomes whole rounds, and run as tiles of half the size in a second launch of one round that
  // takes little more than half a tile time.
  Variant h = with_row_mode(kGemm2[half128]);
  if (h.fn == nullptr) { row_mode = -1; h = with_row_mode(kGemm2[half128]); }   // the second launch's tile picks its own
  const int V = p.n_blocks * ((p.block + v.bm - 1) / v.bm);
  int nq = 0;
  const bool bigger = v.bm * v.bn > h.bm * h.bn;   // the main tile is larger than the second launch's
  if (split == 1 && N >= 2 && bigger) {
    nq = 1;
  } else if (split < 0 && chosen && p.k.per_block == nullptr && bigger && v.lds * 2 > g_lds_limit) {
    const long tiles = (long)V * N;
    const long full = tiles / kNumCU, rem = tiles % kNumCU;
    if (full >= 2 && rem > 0 && 2 * rem <= kNumCU) {
      const int cand = (int)((rem + V - 1) / V);
      const long main_tiles = (long)V * (N - cand);
      const long half_tiles = (long)p.n_blocks * ((p.block + h.bm - 1) / h.bm) * ((p.d_model - (N - cand) * v.bn + h.bn - 1) / h.bn);
      if (cand < N && (main_tiles + kNumCU - 1) / kNumCU == full && half_tiles <= kNumCU) nq = cand;
    }
  }
  if (q.n_pieces > 0) {   // (then nq == 0: the column split is for lists of equal length, or forced)
    hipError_t e = launch_variant(v, v.fn, &q, p.block, p.n_blocks, N, q.k.n_heavy, N * (q.n_pieces - 1), false, s);
    if (e != hipSuccess) return e;
    void *args[] = {&q};
    return hipLaunchKernel(reinterpret_cast<const void *>(&ff_gemm2_reduce_kernel), dim3(q.k.n_heavy * p.block, (p.d_model + 1023) / 1024), dim3(256),
                           args, 0, s);
  }
  if (nq == 0) return launch_variant(v, v.fn, &q, p.block, p.n_blocks, N, q.k.n_heavy, N, false, s);
  hipError_t e = launch_variant(v, v.fn, &q, p.block, p.n_blocks, N - nq, q.k.n_heavy, N - nq, false, s);
  if (e != hipSuccess) return e;
  q.col0 = (N - nq) * v.bn;
  const int N2 = (p.d_model - q.col0 + h.bn - 1) / h.bn;
  return launch_variant(h, h.fn, &q, p.block, p.n_blocks, N2, q.k.n_heavy, N2, false, s);
}

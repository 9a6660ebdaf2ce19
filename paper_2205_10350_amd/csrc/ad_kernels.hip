// gfx950 kernels of the verify / encode / draft forward passes.
//
// Numerical contract of the bf16 mode: weight matrices, GEMM left operands, Q, K, V and the
// softmax numerators that multiply V are bf16 (round to nearest even); accumulation, the
// residual stream, LayerNorm, softmax and logits are fp32.  Every output element is reduced
// in an order that depends on that element alone, never on how many rows or sequences share
// the launch: a row verified in a block of k gives bit-identical results to the same row
// decoded alone, which is what makes draft-and-verify token-identical to greedy decoding
// on this hardware (Section 3.1.1 / Section 3.2 of the paper state the identity for exact
// arithmetic).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "ad_device.h"

namespace ad {

// ------------------------------------------------------------------------------------- embed
// x[m] = E[tok[m]] * sqrt(d) + PE[pos[m]]
template <typename T>
__global__ void k_embed(const T* __restrict__ emb, const float* __restrict__ pe, const int* __restrict__ tok,
                        const int* __restrict__ pos, int d, float sqrt_d, float* __restrict__ x, T* __restrict__ xa) {
  const int m = blockIdx.x;
  const T* e = emb + (size_t)tok[m] * d;
  const float* p = pe + (size_t)pos[m] * d;
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    const float v = embed_value(Store<T>::load(e + c), sqrt_d, p[c]);
    x[(size_t)m * d + c] = v;
    Store<T>::store(xa + (size_t)m * d + c, v);
  }
}

void launch_embed(int dtype, const void* emb, const float* pe, const int* tok, const int* pos, int M, int d,
                  float sqrt_d, float* x, void* xa, hipStream_t s) {
  if (M <= 0) return;
  if (dtype == AD_BF16)
    k_embed<bf16_t><<<M, 128, 0, s>>>((const bf16_t*)emb, pe, tok, pos, d, sqrt_d, x, (bf16_t*)xa);
  else
    k_embed<float><<<M, 128, 0, s>>>((const float*)emb, pe, tok, pos, d, sqrt_d, x, (float*)xa);
}

// ------------------------------------------------------------------------------------- bf16 MFMA GEMM
// C[M,N] = A[M,K] * W[N,K]^T.  One wave owns 16 output columns and MT*16 rows and walks the
// whole K range with v_mfma_f32_16x16x32_bf16, 32 k-values per step in ascending order, into
// one accumulator chain per 16x16 tile.  Weights are stored as B-operand tiles (1 KB per 16
// columns x 32 k, lane slot l = column l%16, k-group l/16) and go from memory straight into the
// operand, one fully coalesced 1 KB fetch per step; for M <= MT*16 each weight is read from
// HBM exactly once.
//   operand layout   A: lane l -> row l%16, k = 8*(l/16) .. +7
//                    B: lane l -> col l%16, k = 8*(l/16) .. +7
//                    C: lane l -> col l%16, rows 4*(l/16) .. +3
template <int MT>
__global__ __launch_bounds__(256) void k_gemm_bf16(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                                   int M, int N, int K, Epi e) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n0 = (blockIdx.x * 4 + wave) * 16;
  const int m0 = blockIdx.y * (MT * 16);
  if (n0 >= N) return;
  const int r = lane & 15, kq = lane >> 4;
  const bf16_t* wp = W + (size_t)n0 * K + lane * 8;   // tile (strip, step u) at + u * 512 elements
  const bf16_t* ap[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    int row = m0 + t * 16 + r;
    row = row < M ? row : M - 1;   // rows past M are computed from a valid row and never stored
    ap[t] = A + (size_t)row * K + kq * 8;
  }
  f32x4 acc[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  // 512 k at a time: all sixteen 1 KB weight fetches of the strip are requested before the first
  // is used (a weight-streaming kernel lives on the bytes it keeps in flight)
  for (int k0 = 0; k0 < K; k0 += 512) {
    uint4 b[16];
#pragma unroll
    for (int u = 0; u < 16; ++u)
      if (k0 + 32 * u < K) b[u] = *(const uint4*)(wp + (k0 + 32 * u) * 16);
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      if (k0 + 32 * u < K) {
        const bf16x8 bv = __builtin_bit_cast(bf16x8, b[u]);
#pragma unroll
        for (int t = 0; t < MT; ++t) {
          const bf16x8 a = __builtin_bit_cast(bf16x8, *(const uint4*)(ap[t] + k0 + 32 * u));
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bv, acc[t], 0, 0, 0);
        }
      }
    }
  }
  strip_epilogue<bf16_t, MT>(e, acc, MT, m0, n0, M, N, lane);
}

// ------------------------------------------------------------------------------------- bf16 MFMA GEMM, many rows, K a multiple of 512
// A stays put, weights stream: a workgroup stages MT*16 rows of A (all K) in LDS once and then
// walks a run of 16-column strips, each wave SP strips at a time (two where rows are many and
// LDS traffic per MFMA matters, one where rows are few and parallelism does).  Work unit = (SP
// strips, 512-k slice): 16*SP weight fragments (fully coalesced 1 KB fetches straight into B operand
// registers).  The registers are refilled on a rolling basis: as soon as step u's MFMAs are
// issued, step u of the NEXT unit is requested into the same registers, so every fetch has a
// whole unit's time before it is needed and one register set suffices; two workgroups share a CU
// and cover each other's gaps.  Per 32-k step the wave reads MT A fragments from LDS and issues
// SP*MT MFMAs.
// Accumulation order per output element as in every other kernel: k ascending, 32 at a time,
// one accumulator.
// EPI_ARGMAX: one (value, column) partial per (row, workgroup) instead of one per strip.
// (Argument order, here and in the other kernels of a forward: the first 64 bytes of a kernel's arguments are in
// scalar registers when a wave starts (kernel-argument preload); what the prologue needs first, the sizes that decide
// the workgroup's place and the pointers of the first loads, comes first, the epilogue's description last.)
// NW waves per workgroup (4, 8 or 16): a wave stages MT*16/NW rows and owns every NW-th run of SP strips.
// (Register budget: two waves per SIMD; four for the 16-wave workgroups and for the 8-wave, 32-row, K = 512
// variant, which then fits a CU twice: forward at 1152 rows 451 -> 446 us.)
template <int MT, int AMAX, int SP, bool ONE, int LNMODE = -1, int EM = -1, int NW = 4>
__global__ __launch_bounds__(64 * NW, NW == 16 || (NW == 8 && ONE && MT == 2 && SP == 1) ? 4 : 2) void k_gemm_bf16_astat(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                                            int M, int N, int K, int strips_per_wg, int groups,
                                                            int chunks, const float* __restrict__ ln_x,
                                                            const float* __restrict__ ln_g, const float* __restrict__ ln_b,
                                                            float* __restrict__ ln_y, Epi e) {
  // (the pending LayerNorm as four plain pointers: a structure among the arguments ends the run of
  // arguments that are preloaded into scalar registers)
  LnA ln;
  ln.x = ln_x; ln.g = ln_g; ln.b = ln_b; ln.y = ln_y;
  constexpr int ROWS = MT * 16, RPW = ROWS / NW;   // rows a wave stages
  static_assert(ROWS % NW == 0, "rows per workgroup must divide among the waves");
  extern __shared__ uint4 astat_lds[];
  bf16_t* At = (bf16_t*)astat_lds;          // [ROWS][K + 16]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, kq = lane >> 4;
  // row stride K + 16 elements = 8 dwords past a multiple of 64 banks: the 16-byte fragment reads of a wave
  // (lane = row + 16 * k-group) then meet no bank twice (measured: K + 8 costs every read 4 extra cycles)
  const int ld = ONE ? 528 : K + 16, n_strips = N >> 4;
  // Workgroup -> (strip group, row chunk).  Consecutive workgroups go to consecutive XCDs, each
  // with its own L2: with eight or more strip groups, group g runs on XCD g % 8 only, its row
  // chunks back to back, so that a group's weights come from HBM once and from that L2 afterwards.
  int group, chunk;
  if (groups >= 8) {
    const int t = blockIdx.x >> 3;
    chunk = t % chunks;
    group = (t / chunks) * 8 + (blockIdx.x & 7);
    if (group >= groups) return;
  } else {
    group = blockIdx.x % groups;
    chunk = blockIdx.x / groups;
  }
  const int m0 = chunk * ROWS;
  const int halves = ONE ? 1 : K >> 9;
  const bf16_t* a_lane = At + r * ld + kq * 8;
  const int s_begin = group * strips_per_wg, s_end = min(n_strips, s_begin + strips_per_wg);
  const int s_first = s_begin + SP * wave;
  const int n_units = s_first < s_end ? ((s_end - s_first + NW * SP - 1) / (NW * SP)) * halves : 0;
  // this lane's fragment addresses of unit q (clamped: the refill after the last unit re-reads it;
  // a wave without strips reads the workgroup's first strip and never uses it)
  auto unit_ptrs = [&](int q, const bf16_t* (&w)[SP]) {
    q = max(0, min(q, n_units - 1));
    const int p = q / halves, k0 = (q - p * halves) << 9;
    const int s0 = n_units > 0 ? s_first + NW * SP * p : s_begin;
#pragma unroll
    for (int j = 0; j < SP; ++j)
      w[j] = W + ((size_t)(min(s0 + j, s_end - 1) << 4) * K + (size_t)k0 * 16 + lane * 8);
  };
  uint4 b[SP][16];
  // Unit 0 is requested right behind the wave's first row loads and is in flight while the rows are
  // staged.  (Loads return in issue order: requested the other way round, the rows, which the
  // whole workgroup waits for at the barrier below, would arrive behind 16 * SP KB of weights.)
  auto prefetch0 = [&]() {
    const bf16_t* w[SP];
    unit_ptrs(0, w);
#pragma unroll
    for (int u = 0; u < 16; ++u)
#pragma unroll
      for (int j = 0; j < SP; ++j) b[j][u] = *(const uint4*)(w[j] + u * 512);
  };
  auto behind_rows = [&]() { prefetch0(); };
  // stage the rows (past M: the last valid row, computed and never stored)
  // (LNMODE 0 / 1: the caller knows at compile time that no LayerNorm / a LayerNorm is pending)
  const bool has_ln = LNMODE < 0 ? ln.x != nullptr : LNMODE == 1;
  if (has_ln) {
    // rows to be normalised first (K = 512 or 1024): the statistics and values of the LayerNorm
    // kernel; the workgroups of strip group 0 also store the fp32 rows
    // (the output projection is the last consumer of its rows: nobody needs them in fp32)
    const bool keep_y = group == 0 && AMAX == 0;
    if (ONE || K == 512) astat_stage_ln<2, (SP == 1 && RPW >= 8 ? 8 : RPW >= 4 ? 4 : RPW), RPW>(ln, At, ld, wave * RPW, m0, M, lane, keep_y, behind_rows);
    else astat_stage_ln<4, (RPW >= 4 ? 4 : RPW), RPW>(ln, At, ld, wave * RPW, m0, M, lane, keep_y, behind_rows);
  } else if (MT == 1 && NW == 4 && !ONE && halves == 4) {
    // few rows of K = 2048: every slice's loads before the weights
    uint4 av[4][4];
#pragma unroll
    for (int h = 0; h < 4; ++h)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        av[h][i] = *(const uint4*)(A + (size_t)min(m0 + wave * 4 + i, M - 1) * K + h * 512 + lane * 8);
    behind_rows();
#pragma unroll
    for (int h = 0; h < 4; ++h)
#pragma unroll
      for (int i = 0; i < 4; ++i) *(uint4*)(At + (wave * 4 + i) * ld + h * 512 + lane * 8) = av[h][i];
  } else
  // a wave's loads of a 512-column slice are all issued before the first LDS store
  for (int h = 0; h < halves; ++h) {
    uint4 av[RPW];
#pragma unroll
    for (int i = 0; i < RPW; ++i)
      av[i] = *(const uint4*)(A + (size_t)min(m0 + wave * RPW + i, M - 1) * K + h * 512 + lane * 8);
    if (h == 0) behind_rows();
#pragma unroll
    for (int i = 0; i < RPW; ++i) *(uint4*)(At + (wave * RPW + i) * ld + h * 512 + lane * 8) = av[i];
  }
  __syncthreads();
  f32x4 acc_x[SP][MT];   // lives across the units of a strip when K has several 512-slices
  // EPI_ARGMAX: every lane keeps the best (value, column) of its MT*4 (row, column-residue) slots
  // over all strips of the wave.  A lane meets its columns in ascending order, so "strictly
  // greater" keeps the smallest column among equal values; the start value (-inf at the lane's
  // first column) makes that hold for a row of -inf too.  A lane without strips keeps the
  // neutral element.
  constexpr int NB = AMAX ? MT * 4 : 1;
  float bv[NB];
  int bi[NB];
#pragma unroll
  for (int x = 0; x < NB; ++x) {
    if constexpr (AMAX == 3) {   // bv = the row's threshold, bi = this lane's count
      const int row = m0 + (x >> 2) * 16 + kq * 4 + (x & 3);
      bv[x] = e.thr[row < M ? row : M - 1];
      bi[x] = 0;
    } else {
      bv[x] = -INFINITY; bi[x] = n_units > 0 ? (s_first << 4) + r : 0x7fffffff;
    }
  }
  // MT = 4: the A fragments in flight across steps and units (see the unit)
  constexpr int AFB = MT < 4 ? 2 : 1;
  uint4 ar[AFB == 1 ? MT : 1];
  if constexpr (AFB == 1) {
#pragma unroll
    for (int t = 0; t < MT; ++t) ar[t] = *(const uint4*)(a_lane + t * 16 * ld);
  }
  // REFILL = false for the wave's last unit: nothing is fetched that nobody will use (the
  // epilogue would wait for it)
  auto unit = [&](auto refill_c, int q) {
    constexpr bool REFILL = decltype(refill_c)::value;
    const int p = q / halves, k0 = (q - p * halves) << 9;
    const bool last = k0 + 512 == K;
    const int s0 = s_first + NW * SP * p;
    const bf16_t* wn[SP];
    unit_ptrs(q + 1, wn);
    // ONE (K = 512): a unit is a whole dot product; its accumulators are the unit's own
    f32x4 acc_l[SP][MT];
    f32x4 (&acc)[SP][MT] = *(ONE ? &acc_l : &acc_x);
    if (ONE || k0 == 0) {
#pragma unroll
      for (int j = 0; j < SP; ++j)
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[j][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // operands of the epilogue that do not depend on the accumulators are requested before the
    // last slice's MFMAs (only where the registers are there for it)
    constexpr bool PRE = !AMAX && MT * SP <= 4;
    EpiRegs<MT> g[SP];
    if constexpr (PRE) {
      if (last) {
#pragma unroll
        for (int j = 0; j < SP; ++j)
          if (s0 + j < s_end) epi_preload<MT, EM>(e, MT, m0, (s0 + j) << 4, M, N, lane, g[j]);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    // A fragments: with MT < 4 a second register set holds the next step's, read while this
    // step's MFMAs run.  With MT = 4 there are no registers for that; instead a row tile's
    // fragment register is refilled with the next step's as soon as the MFMAs that read it are
    // issued (the same rolling scheme as for the weights), so an LDS read has the rest of the
    // step's MFMAs to arrive; the last step reads the first fragments of the next unit.
    uint4 af[AFB][MT];
    if constexpr (AFB == 2) {
#pragma unroll
      for (int t = 0; t < MT; ++t) af[0][t] = *(const uint4*)(a_lane + t * 16 * ld + k0);
      __builtin_amdgcn_sched_group_barrier(0x100, MT, 0);
    }
    const int k0n = ONE ? 0 : (k0 + 512 == K ? 0 : k0 + 512);   // the next unit's slice
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      if constexpr (AFB == 2) {
        if (u + 1 < 16) {
#pragma unroll
          for (int t = 0; t < MT; ++t) af[(u + 1) % 2][t] = *(const uint4*)(a_lane + t * 16 * ld + k0 + 32 * (u + 1));
        }
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
          for (int j = 0; j < SP; ++j)
            acc[j][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, af[u % 2][t]), __builtin_bit_cast(bf16x8, b[j][u]), acc[j][t], 0, 0, 0);
      } else {
#pragma unroll
        for (int t = 0; t < MT; ++t) {
#pragma unroll
          for (int j = 0; j < SP; ++j)
            acc[j][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ar[t]), __builtin_bit_cast(bf16x8, b[j][u]), acc[j][t], 0, 0, 0);
          ar[t] = *(const uint4*)(a_lane + t * 16 * ld + (u + 1 < 16 ? k0 + 32 * (u + 1) : k0n));
        }
      }
      // rolling refill: the same step of the next unit
      if constexpr (REFILL) {
#pragma unroll
        for (int j = 0; j < SP; ++j) b[j][u] = *(const uint4*)(wn[j] + u * 512);
      }
      // issue order per step
      if constexpr (AFB == 2) {
        if (u + 1 < 16) __builtin_amdgcn_sched_group_barrier(0x100, MT, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, SP * MT, 0);
      } else {
#pragma unroll
        for (int t = 0; t < MT; ++t) {
          __builtin_amdgcn_sched_group_barrier(0x008, SP, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
      }
      if constexpr (REFILL) __builtin_amdgcn_sched_group_barrier(0x020, SP, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    // the epilogue's row addressing depends on the chunk only; computed once before the loop it
    // would occupy registers (or scratch) through every unit, so it is tied to this unit
    int m0e = m0;
    asm volatile("" : "+s"(m0e));
    if (last) {
      if constexpr (AMAX) {
#pragma unroll
        for (int j = 0; j < SP; ++j) {
          if (s0 + j >= s_end) break;
          const int n = ((s0 + j) << 4) + r;
#pragma unroll
          for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float v = acc[j][t][i];
              const bool better = v > bv[t * 4 + i];
              if constexpr (AMAX == 3) {
                bi[t * 4 + i] += better ? 1 : 0;
              } else {
                bv[t * 4 + i] = better ? v : bv[t * 4 + i];
                bi[t * 4 + i] = better ? n : bi[t * 4 + i];
              }
            }
          if constexpr (AMAX == 2) {
            for (int t = 0; t < MT; ++t)
              for (int i = 0; i < 4; ++i) {
                const int m = m0e + t * 16 + kq * 4 + i;
                if (m < M) e.logits[(size_t)m * N + n] = acc[j][t][i];
              }
          }
        }
      } else if constexpr (PRE) {
#pragma unroll
        for (int j = 0; j < SP; ++j)
          if (s0 + j < s_end) epi_apply<bf16_t, MT, EM>(e, acc[j], g[j], MT, m0e, (s0 + j) << 4, M, N, lane);
      } else {
#pragma unroll
        for (int j = 0; j < SP; ++j)
          if (s0 + j < s_end) strip_epilogue<bf16_t, MT>(e, acc[j], MT, m0e, (s0 + j) << 4, M, N, lane);
      }
    }
  };
  for (int q = 0; q + 1 < n_units; ++q) unit(std::true_type{}, q);
  if (n_units > 0) unit(std::false_type{}, n_units - 1);
  if constexpr (AMAX) {
    // rows of 16 lanes reduce by lane moves, the waves through LDS
    float* mv = (float*)(At + ROWS * ld);   // [NW waves][ROWS]
    int* mi = (int*)(mv + NW * ROWS);
    // (all lane reductions first: independent chains; then one branch for the LDS writes)
#pragma unroll
    for (int x = 0; x < MT * 4; ++x) {
      if constexpr (AMAX == 3) bi[x] = row16_sum_i(bi[x]);
      else argmax_row16(bv[x], bi[x]);
    }
    if (r == 0) {
#pragma unroll
      for (int x = 0; x < MT * 4; ++x) {
        const int row = (x >> 2) * 16 + kq * 4 + (x & 3);
        mv[wave * ROWS + row] = bv[x];
        mi[wave * ROWS + row] = bi[x];
      }
    }
    __syncthreads();
    if ((int)threadIdx.x < ROWS && m0 + (int)threadIdx.x < M) {
      if constexpr (AMAX == 3) {
        int cnt = mi[threadIdx.x];
#pragma unroll
        for (int w = 1; w < NW; ++w) cnt += mi[w * ROWS + threadIdx.x];
        e.part_idx[(size_t)(m0 + threadIdx.x) * e.n_strips + group] = cnt;
      } else {
        float v = mv[threadIdx.x];
        int idx = mi[threadIdx.x];
#pragma unroll
        for (int w = 1; w < NW; ++w) argmax_merge(v, idx, mv[w * ROWS + threadIdx.x], mi[w * ROWS + threadIdx.x]);
        e.part_val[(size_t)(m0 + threadIdx.x) * e.n_strips + group] = v;
        e.part_idx[(size_t)(m0 + threadIdx.x) * e.n_strips + group] = idx;
      }
    }
  }
}
// Launch shape of the kernel above.  Rough cost model (microseconds) of a shape: the busiest
// XCD runs its workgroups in rounds of (32 CUs x workgroups per CU); a workgroup costs a fixed
// part (launch, staging the rows, drain) plus its units.  Strips per workgroup are a multiple of
// eight (four waves, two strips each).
static size_t astat_lds_bytes(int mt, int K, int nw = 4) { return (size_t)mt * 16 * (K + 16) * 2 + nw * (size_t)mt * 16 * 8; }
static float astat_plan(int mt, int M, int N, int K, bool with_ln, int* per_wg_out) {
  const int chunks = (M + mt * 16 - 1) / (mt * 16), n_strips = N / 16, halves = K / 512;
  const size_t lds = astat_lds_bytes(mt, K);
  const int per_cu = lds * 2 <= 160 * 1024 ? 2 : 1;
  // staging: a wave brings in 4 * mt rows, one after the other when they go through LayerNorm
  const float unit_us = 0.25f * mt + 0.15f, wg_us = 2.0f + 4 * mt * (with_ln ? 0.2f : 0.03f);
  float best = 1e30f;
  for (int per_wg = 8; per_wg <= 128; per_wg += 8) {
    const int groups = (n_strips + per_wg - 1) / per_wg;
    const int wgs_xcd = groups >= 8 ? (groups + 7) / 8 * chunks : (groups * chunks + 7) / 8;
    const int rounds = (wgs_xcd + 32 * per_cu - 1) / (32 * per_cu);
    // co-resident workgroups share the MFMA pipes
    const int together = wgs_xcd > 32 ? per_cu : 1;
    const float cost = rounds * (wg_us + (per_wg / 8) * halves * unit_us * together);
    if (cost < best) { best = cost; *per_wg_out = per_wg; }
    if (groups == 1) break;
  }
  return best;
}
template <int MT, int SP, int NW = 4>
static int launch_astat(const bf16_t* A, const bf16_t* W, int M, int N, int K, const Epi& e, int per_wg, hipStream_t s,
                        const LnA& ln) {
  const int chunks = (M + MT * 16 - 1) / (MT * 16), n_strips = N / 16;
  const size_t lds = astat_lds_bytes(MT, K, NW);
  const int gx = (n_strips + per_wg - 1) / per_wg;
  const int grid = (gx >= 8 ? (gx + 7) / 8 * 8 : gx) * chunks;
  auto go = [&](auto amax_c, auto one_c) {
    constexpr int AMAX = decltype(amax_c)::value;
    constexpr bool ONE = decltype(one_c)::value;
    static size_t set_for = 0;
    if (lds > set_for) {
      (void)hipFuncSetAttribute((const void*)k_gemm_bf16_astat<MT, AMAX, SP, ONE, -1, -1, NW>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      set_for = lds;
    }
    k_gemm_bf16_astat<MT, AMAX, SP, ONE, -1, -1, NW><<<grid, 64 * NW, lds, s>>>(A, W, M, N, K, per_wg, gx, chunks, ln.x, ln.g, ln.b, ln.y, e);
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  const bool amax = e.mode == EPI_ARGMAX;
  if constexpr (MT == 1 && SP == 1 && NW == 4) {
    if (amax && e.logits) {   // launch_gemm sends every request for logits here
      if (K == 512) go(I2{}, std::true_type{});
      else go(I2{}, std::false_type{});
      return gx;
    }
  }
  using I3 = std::integral_constant<int, 3>;
  const bool count = e.mode == EPI_COUNT;
  // a variant with the pending LayerNorm (1) or its absence (0) and, for the layer GEMMs, the epilogue as constants
  auto fixed_variant = [&](auto amax_c, auto ln_c, auto em_c, auto one_c) {
    constexpr int AMAX = decltype(amax_c)::value, LNM = decltype(ln_c)::value, EMV = decltype(em_c)::value;
    constexpr bool ONE = decltype(one_c)::value;
    static size_t set_fixed = 0;
    if (lds > set_fixed) {
      (void)hipFuncSetAttribute((const void*)k_gemm_bf16_astat<MT, AMAX, SP, ONE, LNM, EMV, NW>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      set_fixed = lds;
    }
    k_gemm_bf16_astat<MT, AMAX, SP, ONE, LNM, EMV, NW><<<grid, 64 * NW, lds, s>>>(A, W, M, N, K, per_wg, gx, chunks, ln.x, ln.g, ln.b, ln.y, e);
  };
  if constexpr (NW != 4) {   // the wide workgroups serve the layer GEMMs only
    // (the combinations that occur with the pending LayerNorm and the epilogue as compile-time constants, as for the
    // few-row kernels below: forward at 1152 rows 432.6 -> 425.6 us, at 720 rows 370.5 -> 366.5 us)
    auto wide = [&](auto one_c, auto ln_c, auto em_c) {
      constexpr bool ONE = decltype(one_c)::value;
      constexpr int LNM = decltype(ln_c)::value, EMV = decltype(em_c)::value;
      static size_t set_wide = 0;
      if (lds > set_wide) {
        (void)hipFuncSetAttribute((const void*)k_gemm_bf16_astat<MT, 0, SP, ONE, LNM, EMV, NW>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        set_wide = lds;
      }
      k_gemm_bf16_astat<MT, 0, SP, ONE, LNM, EMV, NW><<<grid, 64 * NW, lds, s>>>(A, W, M, N, K, per_wg, gx, chunks, ln.x, ln.g, ln.b, ln.y, e);
    };
    using L0 = std::integral_constant<int, 0>;
    using L1 = std::integral_constant<int, 1>;
    using EQKV = std::integral_constant<int, EPI_QKV>;
    using ERES = std::integral_constant<int, EPI_RESID>;
    if constexpr (NW == 16) {
      if (K == 512 && ln.x && e.mode == EPI_QKV) { wide(std::true_type{}, L1{}, EQKV{}); return gx; }
      if (K == 512 && !ln.x && e.mode == EPI_QKV) { wide(std::true_type{}, L0{}, EQKV{}); return gx; }
    } else {
      if (K == 512 && !ln.x && e.mode == EPI_RESID) { wide(std::true_type{}, L0{}, ERES{}); return gx; }
      if (K == 2048 && !ln.x && e.mode == EPI_RESID) { wide(std::false_type{}, L0{}, ERES{}); return gx; }
    }
    if (K == 512) go(I0{}, std::true_type{});
    else go(I0{}, std::false_type{});
    return gx;
  } else
  if (K == 512) {
    if (amax) go(I1{}, std::true_type{});
    else if (count) go(I3{}, std::true_type{});
    else if constexpr (MT == 1 && SP == 2 && NW == 4) {
      // FFN1 at many rows (forward at 1152 rows 424.6 -> 412.6 us; the same for the 32-row variant at 720 rows, for FFN2
      // at 192..384 rows and for the many-row output projection measured no gain and was not kept)
      if (ln.x && e.mode == EPI_RELU) fixed_variant(I0{}, std::integral_constant<int, 1>{}, std::integral_constant<int, EPI_RELU>{}, std::true_type{});
      else go(I0{}, std::true_type{});
    }
    else if constexpr (MT == 1 && SP == 1 && NW == 4) {
      // the layer GEMMs of the few-row regime: the pending LayerNorm (or none) and the epilogue mode as
      // compile-time constants, a kernel per combination that occurs (run-time branches around loads in
      // flight make the compiler wait for all of them: 0.1-0.2 us per launch)
      auto hot = [&](auto ln_c, auto em_c) {
        constexpr int LNM = decltype(ln_c)::value, EMV = decltype(em_c)::value;
        static size_t set_hot = 0;
        if (lds > set_hot) {
          (void)hipFuncSetAttribute((const void*)k_gemm_bf16_astat<1, 0, 1, true, LNM, EMV>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
          set_hot = lds;
        }
        k_gemm_bf16_astat<1, 0, 1, true, LNM, EMV><<<grid, 256, lds, s>>>(A, W, M, N, K, per_wg, gx, chunks, ln.x, ln.g, ln.b, ln.y, e);
      };
      using L0 = std::integral_constant<int, 0>;
      using L1 = std::integral_constant<int, 1>;
      if (ln.x && e.mode == EPI_QKV) hot(L1{}, std::integral_constant<int, EPI_QKV>{});
      else if (ln.x && e.mode == EPI_RELU) hot(L1{}, std::integral_constant<int, EPI_RELU>{});
      else if (!ln.x && e.mode == EPI_RESID) hot(L0{}, std::integral_constant<int, EPI_RESID>{});
      else if (!ln.x && e.mode == EPI_QKV) hot(L0{}, std::integral_constant<int, EPI_QKV>{});
      else go(I0{}, std::true_type{});
    } else go(I0{}, std::true_type{});
  } else {
    if (amax) go(I1{}, std::false_type{});
    else if (count) go(I3{}, std::false_type{});
    else go(I0{}, std::false_type{});
  }
  return gx;
}

// ---------------------------------------------------------------- few rows, K of several 512-slices
// C = A . W^T for up to 160 rows when K is 1024, 2048 or 4096 and no LayerNorm is pending (FFN2, the
// attention output projections of the wide model).  The A-in-LDS kernel above walks a strip's
// 512-slices one after the other in one wave, a round trip to memory per slice.  Here a workgroup
// owns one 16-column strip of one 16-row chunk and its wave w owns the slices w, w + 4, ...: every
// wave requests its slice of the rows (into an LDS tile of its own: no barrier before the first
// MFMA; fragments requested straight from the row-major rows, 16 rows x 64 bytes per wave
// instruction, measured 1 us slower per launch) and of the weights at once, so the workgroup waits
// for memory once.  The sum itself stays one chain: the accumulators go from
// wave to wave through LDS in slice order (k ascending, 32 at a time, one accumulator per element:
// the same bits as every other GEMM kernel here), and the wave of the last slice runs the epilogue.
// a 512-slice of 16 rows into a wave's LDS tile (one row per wave instruction, 16 bytes per lane)
// and of a strip's weights into registers; all requests before the first LDS store
__device__ __forceinline__ void kchain_request(const bf16_t* __restrict__ A, const bf16_t* __restrict__ wp, bf16_t* At,
                                               int m0, int M, int K, int slice, int lane, uint4 (&b)[16]) {
  constexpr int LD = 512 + 16;
  uint4 av[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) av[i] = *(const uint4*)(A + (size_t)min(m0 + i, M - 1) * K + slice * 512 + lane * 8);
#pragma unroll
  for (int u = 0; u < 16; ++u) b[u] = *(const uint4*)(wp + (size_t)slice * 8192 + u * 512);
#pragma unroll
  for (int i = 0; i < 16; ++i) *(uint4*)(At + i * LD + lane * 8) = av[i];
}
template <int NS>
__global__ __launch_bounds__(256) void k_gemm_bf16_kchain(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                                         int M, int N, int K, int n_strips, Epi e) {
  constexpr int LD = 512 + 16;               // row stride of a wave's tile (elements): see the kernel above
  __shared__ uint4 tiles[4 * 16 * LD / 8];   // [wave][16 rows][LD]: each wave stages its own slice, no barrier
  __shared__ f32x4 hand[64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, kq = lane >> 4;
  const int strip = blockIdx.x % n_strips, m0 = (blockIdx.x / n_strips) * 16, n0 = strip << 4;
  bf16_t* At = (bf16_t*)tiles + wave * 16 * LD;
  const bf16_t* a_lane = At + r * LD + kq * 8;
  const bf16_t* wp = W + (size_t)n0 * K + lane * 8;
  uint4 b[16];
  if (wave < NS) kchain_request(A, wp, At, m0, M, K, wave, lane, b);
  constexpr int LAST = (NS - 1) & 3;
  EpiRegs<1> g;
  if (wave == LAST) epi_preload<1>(e, 1, m0, n0, M, N, lane, g);
  f32x4 acc[1] = {f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
  for (int p = 0; p < NS; ++p) {
    if (wave == (p & 3)) {
      if (p > 0) acc[0] = hand[lane];
#pragma unroll
      for (int u = 0; u < 16; ++u)
        acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, *(const uint4*)(a_lane + 32 * u)), __builtin_bit_cast(bf16x8, b[u]), acc[0], 0, 0, 0);
      if (p + 1 < NS) hand[lane] = acc[0];
      if (p + 4 < NS) kchain_request(A, wp, At, m0, M, K, p + 4, lane, b);
    }
    if (p + 1 < NS) __syncthreads();
  }
  if (wave == LAST) epi_apply<bf16_t, 1>(e, acc, g, 1, m0, n0, M, N, lane);
}
static void launch_kchain(const bf16_t* A, const bf16_t* W, int M, int N, int K, const Epi& e, hipStream_t s) {
  const int n_strips = N / 16, grid = n_strips * ((M + 15) / 16);
  if (K == 1024) k_gemm_bf16_kchain<2><<<grid, 256, 0, s>>>(A, W, M, N, K, n_strips, e);
  else if (K == 2048) k_gemm_bf16_kchain<4><<<grid, 256, 0, s>>>(A, W, M, N, K, n_strips, e);
  else k_gemm_bf16_kchain<8><<<grid, 256, 0, s>>>(A, W, M, N, K, n_strips, e);
}

// ------------------------------------------------------------------------------------- fp32 GEMM
// Plain fp32 path: one thread per output element, k ascending, fused multiply-add.
__global__ __launch_bounds__(256) void k_gemm_f32(const float* __restrict__ A, const float* __restrict__ W, int M,
                                                  int N, int K, Epi e) {
  __shared__ float As[16][33];
  __shared__ float Ws[16][33];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int n0 = blockIdx.x * 16, m0 = blockIdx.y * 16;
  const int m = m0 + ty, n = n0 + tx;
  float acc = 0.f;
  for (int k0 = 0; k0 < K; k0 += 32) {
    for (int i = threadIdx.x; i < 16 * 32; i += 256) {
      const int rr = i >> 5, cc = i & 31;
      const int am = m0 + rr < M ? m0 + rr : M - 1;
      const int wn = n0 + rr < N ? n0 + rr : N - 1;
      As[rr][cc] = A[(size_t)am * K + k0 + cc];
      Ws[rr][cc] = W[(size_t)wn * K + k0 + cc];
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 32; ++kk) acc = fmaf(As[ty][kk], Ws[tx][kk], acc);
    __syncthreads();
  }
  if (e.mode == EPI_ARGMAX) {
    // 16 columns per strip, reduced by the 16 threads of a row (they sit in one wave)
    float v = acc;
    int idx = n;
    if (e.logits && m < M && n < N) e.logits[(size_t)m * N + n] = v;
    argmax_row16(v, idx);
    if (tx == 0 && m < M) {
      e.part_val[(size_t)m * e.n_strips + blockIdx.x] = v;
      e.part_idx[(size_t)m * e.n_strips + blockIdx.x] = idx;
    }
    return;
  }
  if (e.mode == EPI_COUNT) {
    const int cnt = row16_sum_i(n < N && acc > e.thr[m < M ? m : M - 1] ? 1 : 0);
    if (tx == 0 && m < M) e.part_idx[(size_t)m * e.n_strips + blockIdx.x] = cnt;
    return;
  }
  if (m < M && n < N) epi_store<float>(e, m, n, N, acc);
}

int launch_gemm(int dtype, const void* A, const void* W, int M, int N, int K, const Epi& e, hipStream_t s,
                const LnA& ln_in, bool* a_written) {
  if (M <= 0) return 0;
  if (a_written) *a_written = true;
  LnA ln = ln_in;
  const bool streams = dtype == AD_BF16 && K <= 4096 && K % 512 == 0;   // the A-in-LDS kernel takes it
  if (ln.x && !(streams && (K == 512 || K == 1024))) {
    launch_layernorm(dtype, ln.x, ln.g, ln.b, M, K, ln.y, const_cast<void*>(A), s);
    ln = LnA{};
  }
  if (ln.x && a_written) *a_written = false;
  if (dtype == AD_BF16) {
    const int nb = (N / 16 + 3) / 4;
    if (K <= 4096 && K % 512 == 0) {
      const bf16_t *a = (const bf16_t*)A, *w = (const bf16_t*)W;
      // up to 160 rows of a K of several slices, as they are: the slices side by side in the waves
      // (measured, forward with this kernel up to 64 / 128 / 256 rows: base model 144 rows 253 / 253 / 249 us,
      // 288 rows 285 / 286 / 285 us (293 us with a limit of 512); wide model 100 rows 365 / 352 / 352 us, 200 rows
      // 430 / 430 / 477 us)
      if (M <= 160 && !ln.x && (K == 1024 || K == 2048 || K == 4096) && e.mode != EPI_ARGMAX && e.mode != EPI_COUNT) {
        launch_kchain(a, w, M, N, K, e, s);
        return N / 16;
      }
      // Few rows (measured: up to 64 for the wide output projection, up to 1024 for the layer
      // GEMMs: forward at 792..1008 rows 420-438 us this way, 431-449 us by the cost model below; from
      // 1080 rows the other way round, 520 against 489 us): latency decides, so 16 rows per workgroup
      // (32 from 520 rows, see below), one strip per wave, workgroups of four strips until the chip is
      // covered (at most about 512 workgroups for the layer GEMMs); more rows are more row chunks of
      // the same shape.
      const int mt = 1;
      const bool want_logits = e.mode == EPI_ARGMAX && e.logits != nullptr;
      // 520 rows and more of the d = 512 layer GEMMs: 32 rows per workgroup in workgroups of 16 or 8 waves, one
      // strip and one unit per 512-slice for each wave, while the launch stays within one round of the chip
      // (a wave stages 2 or 4 rows instead of 8, and every wave's weights are requested at once; measured at
      // 1152 rows: QKV with the LayerNorm 12.4 -> 9.6 us, attention output projections 7.0 -> 5.5 us, FFN2
      // 12.9 -> 11.0 us; forward at 576 / 720 / 864 / 1008 / 1152 rows 372 / 411 / 425 / 453 / 517 ->
      // 362 / 393 / 401 / 417 / 458 us, at 432 rows 321 -> 350 us the other way; FFN1's 128 strips would need
      // two rounds and gained nothing in any shape tried, in one round of two 8-wave workgroups per CU either; K = 1024: drafter forward of the wide model at 626
      // rows 983 -> 1073 us, so those shapes keep the rules below)
      if (M >= 520 && e.mode != EPI_ARGMAX && e.mode != EPI_COUNT) {
        const int n_strips = N / 16, chunks2 = (M + 31) / 32;
        if (K == 512 && n_strips >= 64 && n_strips % 16 == 0 && (n_strips / 16) * chunks2 <= 256)
          return launch_astat<2, 1, 16>(a, w, M, N, K, e, 16, s, ln);
        if ((K == 512 || K == 2048) && !ln.x && n_strips % 8 == 0 && (n_strips / 8) * chunks2 <= 256)
          return launch_astat<2, 1, 8>(a, w, M, N, K, e, 8, s, ln);
      }
      if ((M <= 64 || (M <= 1024 && N <= 4096) || want_logits) && astat_lds_bytes(mt, K) <= 150 * 1024) {
        {
          const int n_strips = N / 16, chunks = (M + 15) / 16;
          int per_wg = 4 * std::max(1, (n_strips + 4 * 384 - 1) / (4 * 384));
          // (measured at 33..64 rows of the wide output projection: 12-16 strips per workgroup, about 500
          // workgroups = one round on the chip, 9.0-9.6 us against 11-13 us with 8 strips)
          if (N <= 4096 || chunks > 2) per_wg = 4 * std::max(1, (n_strips * chunks + 4 * 512 - 1) / (4 * 512));
          // wider K (measured at 400..700 rows of the d = 1024 shapes): at most 16 strips per workgroup while
          // two workgroups fit a CU (more rounds beat longer workgroups); one round of 256 workgroups while
          // the A tile leaves room for one only (K = 4096)
          if (K > 512 && N <= 4096) {
            if (astat_lds_bytes(1, K) * 2 <= 160 * 1024) {
              per_wg = std::min(per_wg, 16);
            } else {
              per_wg = 4 * std::max(1, (n_strips * chunks + 4 * 256 - 1) / (4 * 256));
              while (per_wg < n_strips && (n_strips + per_wg - 1) / per_wg * chunks > 256) per_wg += 4;
            }
          }
          // Nine or more strip groups are dealt round the eight XCDs (group g on XCD g % 8): a count that is
          // no multiple of eight leaves some XCDs with one group more than the others, so strips per
          // workgroup grow until the groups divide evenly (measured at 576..756 rows: forward 3-6 % shorter)
          // (layer GEMMs only: the output projection has hundreds of groups, where one more or less per XCD
          // does not matter, and its own measured rule above)
          auto balanced = [&](int pw) {
            if (e.mode == EPI_ARGMAX || e.mode == EPI_COUNT) return pw;
            auto groups_of = [&](int x) { return (n_strips + x - 1) / x; };
            while (groups_of(pw) > 8 && groups_of(pw) % 8 != 0) pw += 4;
            return pw;
          };
          // 520 rows and more (layer GEMMs only): 32 rows per workgroup, so that the weights cross from L2 to
          // the CUs half as often (every 16-row chunk reads the whole matrix: at 576 rows x N 1536 that is
          // 55 MB per launch, more than the launch takes to do anything else); below that the shorter staging
          // of a 16-row tile wins (measured: 504 rows 347 / 362 us forward with 16 / 32 rows, 576 rows 387 / 374,
          // 648 rows 408 / 399, 756 rows 416 / 416)
          if (M >= 520 && e.mode != EPI_ARGMAX && e.mode != EPI_COUNT && astat_lds_bytes(2, K) <= 150 * 1024) {
            const int chunks2 = (M + 31) / 32;
            int pw2 = 4 * std::max(1, (n_strips * chunks2 + 4 * 512 - 1) / (4 * 512));
            if (K > 512 && astat_lds_bytes(2, K) * 2 <= 160 * 1024) pw2 = std::min(pw2, 16);
            return launch_astat<2, 1>(a, w, M, N, K, e, balanced(pw2), s, ln);
          }
          return launch_astat<1, 1>(a, w, M, N, K, e, balanced(per_wg), s, ln);
        }
      } else {
        // rows per workgroup (16, 32 or 64, as far as the A tile fits in LDS) and strips per
        // workgroup by the cost model
        int pw[3] = {8, 8, 8};
        const float c1 = astat_plan(1, M, N, K, ln.x != nullptr, &pw[0]);
        const float c2 = K <= 2048 ? astat_plan(2, M, N, K, ln.x != nullptr, &pw[1]) : 1e30f;
        const float c4 = K <= 1024 ? astat_plan(4, M, N, K, ln.x != nullptr, &pw[2]) : 1e30f;
        if (c4 <= c2 && c4 <= c1) return launch_astat<4, 2>(a, w, M, N, K, e, pw[2], s, ln);
        if (c2 <= c1) return launch_astat<2, 2>(a, w, M, N, K, e, pw[1], s, ln);
        return launch_astat<1, 2>(a, w, M, N, K, e, pw[0], s, ln);
      }
    }
    if (M <= 16)
      k_gemm_bf16<1><<<dim3(nb, 1), 256, 0, s>>>((const bf16_t*)A, (const bf16_t*)W, M, N, K, e);
    else if (M <= 32)
      k_gemm_bf16<2><<<dim3(nb, 1), 256, 0, s>>>((const bf16_t*)A, (const bf16_t*)W, M, N, K, e);
    else
      k_gemm_bf16<4><<<dim3(nb, (M + 63) / 64), 256, 0, s>>>((const bf16_t*)A, (const bf16_t*)W, M, N, K, e);
  } else {
    k_gemm_f32<<<dim3(N / 16, (M + 15) / 16), 256, 0, s>>>((const float*)A, (const float*)W, M, N, K, e);
  }
  return N / 16;
}

// ------------------------------------------------------------------------------------- attention
// One block per (sequence, head, chunk of 64 query rows); see attn_block.
template <typename T, int DH>
__global__ __launch_bounds__(256) void k_attention(const T* __restrict__ q, const T* __restrict__ Kb,
                                                   const T* __restrict__ Vb, T* __restrict__ out,
                                                   const SeqDesc* __restrict__ desc, int d, float scale, int nk_cap) {
  extern __shared__ unsigned att_lds[];
  const SeqDesc sd = desc[blockIdx.x];
  const int row_begin = blockIdx.z * 64;
  if (row_begin >= sd.nq) return;
  const int row_end = min(sd.nq, row_begin + 64);
  attn_block<T, DH>(q, Kb, Vb, out, sd, row_begin, row_end, blockIdx.y, d, scale, att_lds, nk_cap);
}

// The same for launches whose bounds promise at most 64 keys and one chunk of rows (bf16, head width 64): the one path
// that remains (values staged with 2-byte stores, four key tiles at a time, no shared score tiles), a fifth of the
// generic kernel's instructions.  Same device functions, same bits.  (The key count is clamped to the promise, so that
// a bound that does not hold cannot send an access outside the tiles.)
__global__ __launch_bounds__(256) void k_attention_small(const bf16_t* __restrict__ q, const bf16_t* __restrict__ Kb,
                                                         const bf16_t* __restrict__ Vb, bf16_t* __restrict__ out,
                                                         const SeqDesc* __restrict__ desc, int d, float scale) {
  constexpr int DH = 64;
  extern __shared__ unsigned att_small_lds[];
  const SeqDesc sd = desc[blockIdx.x];
  if (sd.nq <= 0) return;
  const int row_begin = 0, row_end = min(sd.nq, 64), h = blockIdx.y;
  const int nk_all = min(sd.causal ? sd.nk_base + row_end : sd.nk_base, 64);
  const int wave = threadIdx.x >> 6;
  const int nkp = (nk_all + 31) & ~31, ldv = nkp + 16;
  bf16_t* Vt = (bf16_t*)att_small_lds;
  bf16_t* Pw = Vt + DH * ldv + wave * 16 * ldv;
  uint4 qf_pre[DH / 32], kf_pre[4][DH / 32];
  attn_preload<DH>(q, Kb, sd, row_begin, row_end, h, d, nk_all, qf_pre, kf_pre);
  {
    constexpr int G = DH / 8;
    const bf16_t* vg = Vb + (size_t)sd.kv_row0 * d + h * DH;
    for (int i = threadIdx.x; i < nkp * G; i += 256) {
      const int g = i / nkp, t = i - g * nkp;
      uint4 v = uint4{0u, 0u, 0u, 0u};
      if (t < nk_all) v = ldg16(vg + (size_t)t * d + g * 8);
      bf16_t* dst = Vt + (size_t)(g * 8) * ldv + t;
      dst[0] = (bf16_t)(v.x & 0xffffu); dst[ldv] = (bf16_t)(v.x >> 16);
      dst[2 * ldv] = (bf16_t)(v.y & 0xffffu); dst[3 * ldv] = (bf16_t)(v.y >> 16);
      dst[4 * ldv] = (bf16_t)(v.z & 0xffffu); dst[5 * ldv] = (bf16_t)(v.z >> 16);
      dst[6 * ldv] = (bf16_t)(v.w & 0xffffu); dst[7 * ldv] = (bf16_t)(v.w >> 16);
    }
  }
  __syncthreads();
  attn_tiles_mfma<DH, 4>(q, Kb, out, sd, row_begin, row_end, h, d, scale, Vt, Pw, ldv, nk_all, qf_pre, kf_pre, nullptr, nkp);
}

template <typename T>
static void attention_dispatch(const void* q, const void* K, const void* V, void* out, const SeqDesc* desc,
                               int n_seq, int max_rows, int H, int dh, int max_keys, hipStream_t s) {
  const float scale = 1.0f / sqrtf((float)dh);
  const size_t sh = attn_lds_bytes(max_keys, dh, sizeof(T), 4);
  dim3 g(n_seq, H, (max_rows + 63) / 64);
#define AD_ATT(DH)                                                                                             \
  do {                                                                                                         \
    static size_t set_for = 0;                                                                                 \
    if (sh > set_for) {                                                                                        \
      (void)hipFuncSetAttribute((const void*)k_attention<T, DH>, hipFuncAttributeMaxDynamicSharedMemorySize,   \
                                (int)sh);                                                                      \
      set_for = sh;                                                                                            \
    }                                                                                                          \
    k_attention<T, DH><<<g, 256, sh, s>>>((const T*)q, (const T*)K, (const T*)V, (T*)out, desc, H * dh, scale, \
                                          max_keys);                                                           \
  } while (0)
  if constexpr (sizeof(T) == 2) {
    // at most 64 keys and 64 rows per problem (the caller's bounds promise both): the compact kernel (measured against the
    // generic one, base model: forward at 8 / 25 rows 183.2 / 186.8 -> 180.2 / 185.0 us, at 32 x 6 / 32 x 36 rows
    // 228.5 / 446.4 -> 224.6 / 434.5 us)
    if (dh == 64 && max_keys <= 64 && max_rows <= 64) {
      k_attention_small<<<dim3(n_seq, H, 1), 256, sh, s>>>((const bf16_t*)q, (const bf16_t*)K, (const bf16_t*)V, (bf16_t*)out, desc, H * dh, scale);
      return;
    }
    if (dh == 64 && max_keys >= kLongKeys) {   // long key ranges: a kernel in a code object of its own
      launch_attention_long(q, K, V, out, desc, g, H * dh, scale, max_keys, sh, s);
      return;
    }
  }
  switch (dh) {
    case 16: AD_ATT(16); break;
    case 32: AD_ATT(32); break;
    case 64: AD_ATT(64); break;
    default: AD_ATT(128); break;
  }
#undef AD_ATT
}
void launch_attention(int dtype, const void* q, const void* K, const void* V, void* out, const SeqDesc* desc,
                      int n_seq, int max_rows, int H, int dh, int max_keys, hipStream_t s) {
  if (n_seq <= 0 || max_rows <= 0) return;
  if (dtype == AD_BF16) attention_dispatch<bf16_t>(q, K, V, out, desc, n_seq, max_rows, H, dh, max_keys, s);
  else attention_dispatch<float>(q, K, V, out, desc, n_seq, max_rows, H, dh, max_keys, s);
}

// ------------------------------------------------- cross-attention with its query projection
// One workgroup per (sequence, head, chunk of 16, 32 or 64 query rows), head width 64, model width 512 or
// 1024, bf16.  The workgroup stages its rows in LDS (through the pending LayerNorm of the
// previous sublayer, the statistics and values of the LayerNorm kernel; the workgroups of head 0
// also keep the fp32 rows), multiplies them by the head's 64 columns of the query matrix (wave w:
// the 16-column strip 4 * head + w; k ascending, 32 at a time, one accumulator per element, bias
// added and the sum rounded to bf16 as the GEMM kernels' epilogue does: the same bits as a
// projection launch), leaves the queries in LDS and goes on with the attention of those rows as
// k_attention does.  What the attention needs that does not depend on the queries (the first key
// tiles, the values when they are few) is requested at the very start, next to the weights, so
// the kernel waits for memory once.  One launch and one trip through memory less per decoder layer.
// LDS: [values, transposed][probability tiles | row tile (until the queries are there)][queries].
bool launch_crossq_attention(int dtype, const LnA& ln, const void* A, const void* W, const float* bias, const void* K,
                             const void* V, void* out, const SeqDesc* desc, int n_seq, int max_rows, int H, int dh,
                             int max_keys, hipStream_t s) {
  const int d = H * dh;
  if (dtype != AD_BF16 || dh != 64 || (d != 512 && d != 1024)) return false;
  // query rows per workgroup: 16 while that keeps the launch within about one workgroup per compute
  // unit (a row tile per workgroup: the shortest staging), else 32 under the same condition, else 64
  // (measured forward times, base model, 16 / 32 / 64 rows per workgroup; batch x rows:
  //  1 x 25: 237 / 248 / 247 us, 1 x 64: 243 / 254 / 271, 8 x 36: 288 / 298 / 306, 12 x 36: 354 / 332 / 342,
  //  16 x 36: 434 / 409 / 418, 24 x 36: 477 / 455 / 431, 32 x 36: 535 / 514 / 487)
  // (Where the tiles of a 64-row chunk do not fit in LDS, 512-token sources of the wide model, the projection and the
  // attention stay two launches: 32-row chunks would fit and measured slower, drafter forward at 626 rows 957 -> 1051 us.)
  const int chunk = n_seq * H * ((max_rows + 15) / 16) <= 256 ? 16 : (n_seq * H * ((max_rows + 31) / 32) <= 256 ? 32 : 64);
  const int mt = (std::min(max_rows, chunk) + 15) / 16;
  // a long source capacity: the kernels of the other code object (the summation order beyond 128 keys; with one row
  // tile per workgroup the waves split the keys)
  if (max_keys >= kLongKeys)
    return launch_crossq_attention_long(ln, A, W, bias, K, V, out, desc, n_seq, max_rows, H, chunk, max_keys, s);
  const size_t sh = crossq_lds_bytes(max_keys, mt, d);
  if (sh > 160 * 1024) return false;
  if (n_seq <= 0 || max_rows <= 0) return true;
  dim3 g(n_seq, H, (max_rows + chunk - 1) / chunk);
  const float scale = 1.0f / sqrtf((float)dh);
  // at most 64 keys (the bound the caller gives promises it): variants that hold that path only, a sixth of the code with
  // one row tile per workgroup, less than half with several
  const int small = max_keys <= 64 ? (mt == 1 ? 1 : 2) : 0;
  auto go = [&](auto nv_c, auto small_c, auto ln_c) {
    constexpr int NV = decltype(nv_c)::value;
    constexpr int SMALL = decltype(small_c)::value;
    constexpr int LNM = decltype(ln_c)::value;
    static size_t set_for = 0;
    if (sh > set_for) {
      (void)hipFuncSetAttribute((const void*)k_crossq_attention<NV, SMALL, false, LNM>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh);
      set_for = sh;
    }
    k_crossq_attention<NV, SMALL, false, LNM><<<g, 256, sh, s>>>(desc, chunk, scale, (const bf16_t*)W, (const bf16_t*)K, (const bf16_t*)V,
                                                                 ln.x, ln.g, ln.b, ln.y, (const bf16_t*)A, bias, (bf16_t*)out);
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I4 = std::integral_constant<int, 4>;
  using LX = std::integral_constant<int, -1>;
  // (in a decoder layer a LayerNorm is always pending here: the compact variants hold that staging path alone)
  if (d == 512) {
    if (small == 1) { if (ln.x) go(I2{}, I1{}, I1{}); else go(I2{}, I1{}, LX{}); }
    else if (small == 2) { if (ln.x) go(I2{}, I2{}, I1{}); else go(I2{}, I2{}, LX{}); }
    else go(I2{}, I0{}, LX{});
  } else {
    if (small == 1) { if (ln.x) go(I4{}, I1{}, I1{}); else go(I4{}, I1{}, LX{}); }
    else if (small == 2) { if (ln.x) go(I4{}, I2{}, I1{}); else go(I4{}, I2{}, LX{}); }
    else go(I4{}, I0{}, LX{});
  }
  return true;
}

// ------------------------------------------------------------------------------------- LayerNorm
// One wave per row; mean, then biased variance of the centred values, eps = 1e-5.
template <typename T, int NV>
__device__ __forceinline__ void layernorm_row4(const float* __restrict__ xr, const float* __restrict__ g,
                                               const float* __restrict__ b, int d, int lane, float* __restrict__ yr,
                                               T* __restrict__ yar) {
  float4 xv[NV];
  float mean, rstd;
  ln_load4<NV>(xr, lane, xv);
  ln_stats4<NV>(xv, d, mean, rstd);
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int c = 4 * lane + 256 * j;
    const float4 gv = *(const float4*)(g + c), bv = *(const float4*)(b + c);
    const float4 o = float4{ln_value(xv[j].x, mean, rstd, gv.x, bv.x), ln_value(xv[j].y, mean, rstd, gv.y, bv.y),
                            ln_value(xv[j].z, mean, rstd, gv.z, bv.z), ln_value(xv[j].w, mean, rstd, gv.w, bv.w)};
    *(float4*)(yr + c) = o;
    Store<T>::store(yar + c, o.x); Store<T>::store(yar + c + 1, o.y);
    Store<T>::store(yar + c + 2, o.z); Store<T>::store(yar + c + 3, o.w);
  }
}
template <typename T>
__global__ __launch_bounds__(256) void k_layernorm(const float* __restrict__ x, const float* __restrict__ g,
                                                   const float* __restrict__ b, int M, int d, float* __restrict__ y,
                                                   T* __restrict__ ya) {
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (m >= M) return;
  const float* xr = x + (size_t)m * d;
  float* yr = y + (size_t)m * d;
  T* yar = ya + (size_t)m * d;
  switch (ln_vector_width(d)) {
    case 1: layernorm_row4<T, 1>(xr, g, b, d, lane, yr, yar); return;
    case 2: layernorm_row4<T, 2>(xr, g, b, d, lane, yr, yar); return;
    case 4: layernorm_row4<T, 4>(xr, g, b, d, lane, yr, yar); return;
    case 8: layernorm_row4<T, 8>(xr, g, b, d, lane, yr, yar); return;
    default: break;
  }
  float mean, rstd, xv[32];
  ln_load_stats(xr, d, lane, xv, mean, rstd);
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const int c = lane + 64 * j;
    if (c < d) {
      const float o = ln_value(xv[j], mean, rstd, g[c], b[c]);
      yr[c] = o;
      Store<T>::store(yar + c, o);
    }
  }
}
void launch_layernorm(int dtype, const float* x, const float* g, const float* b, int M, int d, float* y, void* ya,
                      hipStream_t s) {
  if (M <= 0) return;
  if (dtype == AD_BF16) k_layernorm<bf16_t><<<(M + 3) / 4, 256, 0, s>>>(x, g, b, M, d, y, (bf16_t*)ya);
  else k_layernorm<float><<<(M + 3) / 4, 256, 0, s>>>(x, g, b, M, d, y, (float*)ya);
}

// ------------------------------------------------------------------------------------- counter calibration copy
__global__ __launch_bounds__(256) void k_calibration_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}
hipError_t launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
  const size_t n = bytes / 16;
  if (n == 0) return hipSuccess;
  const int grid = (int)std::min<size_t>((n + 255) / 256, 256 * 32);
  k_calibration_copy<<<grid, 256, 0, s>>>((const uint4*)src, (uint4*)dst, n);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------- MFMA issue-rate calibration
// Every wave issues `iters` x 8 independent v_mfma_f32_16x16x32_bf16 on register operands that never
// change: the rate the matrix cores accept this instruction at, whole chip (2 waves per SIMD).
__global__ __launch_bounds__(256) void k_calibration_mfma(float* __restrict__ out, int iters) {
  f32x4 c[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) c[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  const uint4 av = uint4{0x3c003c00u + threadIdx.x, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
  const uint4 bv = uint4{0x3c003c00u, 0x3c003c00u + blockIdx.x, 0x3c003c00u, 0x3c003c00u};
  const bf16x8 a = __builtin_bit_cast(bf16x8, av), b = __builtin_bit_cast(bf16x8, bv);
  // (written out: left to itself the compiler shuttles the accumulators between register files in the loop)
  for (int i = 0; i < iters; ++i)
    asm volatile(
        "v_mfma_f32_16x16x32_bf16 %0, %8, %9, %0\n v_mfma_f32_16x16x32_bf16 %1, %8, %9, %1\n"
        "v_mfma_f32_16x16x32_bf16 %2, %8, %9, %2\n v_mfma_f32_16x16x32_bf16 %3, %8, %9, %3\n"
        "v_mfma_f32_16x16x32_bf16 %4, %8, %9, %4\n v_mfma_f32_16x16x32_bf16 %5, %8, %9, %5\n"
        "v_mfma_f32_16x16x32_bf16 %6, %8, %9, %6\n v_mfma_f32_16x16x32_bf16 %7, %8, %9, %7\n"
        : "+v"(c[0]), "+v"(c[1]), "+v"(c[2]), "+v"(c[3]), "+v"(c[4]), "+v"(c[5]), "+v"(c[6]), "+v"(c[7])
        : "v"(a), "v"(b));
  float r = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) r += c[j][0] + c[j][1] + c[j][2] + c[j][3];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = r;
}
hipError_t launch_calibration_mfma(float* out, int workgroups, int iters, hipStream_t s) {
  k_calibration_mfma<<<workgroups, 256, 0, s>>>(out, iters);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------- arg max, second stage
__global__ __launch_bounds__(256) void k_argmax_finish(const float* __restrict__ pv, const int* __restrict__ pi,
                                                       int M, int stride, int n_part, int* __restrict__ o_hat,
                                                       float* __restrict__ o_val) {
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (m >= M) return;
  float v;
  int idx;
  argmax_row(pv + (size_t)m * stride, pi + (size_t)m * stride, n_part, lane, v, idx);
  if (lane == 0) {
    o_hat[m] = idx;
    if (o_val) o_val[m] = v;
  }
}
void launch_argmax_finish(const float* pv, const int* pi, int M, int stride, int n_part, int* o_hat, float* o_val,
                          hipStream_t s) {
  if (M <= 0) return;
  k_argmax_finish<<<(M + 3) / 4, 256, 0, s>>>(pv, pi, M, stride, n_part, o_hat, o_val);
}

// Second stage of the arg max for the drafter's mask rows, writing the drafted tokens where the host
// reads them: row r = (l, i) is drafted token i of the l-th unfinished sequence b; its 8-byte slot
// [b * k_max + i] of `slots` (host-visible memory) receives (ticket << 32 | token) in one store, so
// that seeing the call's ticket in a slot is seeing its token.
__global__ __launch_bounds__(256) void k_argmax_draft(const float* __restrict__ pv, const int* __restrict__ pi, int M,
                                                      int stride, int n_part, int* __restrict__ o_hat,
                                                      const int* __restrict__ finished, int B, int k, int k_max,
                                                      const int* __restrict__ ticket_in,
                                                      unsigned long long* __restrict__ slots) {
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (m >= M) return;
  const int ticket = *ticket_in;
  const int l = m / k, i = m - l * k;
  int b = 0;
  for (int seen = 0; b < B; ++b) {
    if (finished[b]) continue;
    if (seen == l) break;
    ++seen;
  }
  float v;
  int idx;
  argmax_row(pv + (size_t)m * stride, pi + (size_t)m * stride, n_part, lane, v, idx);
  if (lane == 0) {
    o_hat[m] = idx;
    __hip_atomic_store(slots + (size_t)b * k_max + i, ((unsigned long long)(unsigned)ticket << 32) | (unsigned)idx,
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  }
}
void launch_argmax_draft(const float* pv, const int* pi, int M, int stride, int n_part, int* o_hat, const int* finished,
                         int B, int k, int k_max, const int* ticket_in, unsigned long long* slots, hipStream_t s) {
  if (M <= 0) return;
  k_argmax_draft<<<(M + 3) / 4, 256, 0, s>>>(pv, pi, M, stride, n_part, o_hat, finished, B, k, k_max, ticket_in, slots);
}


// ------------------------------------------------------------------------------------- row assembly
// Packed row m of a batch whose sequences contribute n[0..B) rows: its sequence and its index there.  The counts may
// live in host memory, where every read is a trip over the bus: the threads read them side by side (one trip per 128
// sequences) into LDS and thread 0 scans them there.  The result is in where[0..1] for the whole workgroup.
__device__ __forceinline__ void locate_packed_row(const int* __restrict__ n, int B, int m, int* chunk, int* where) {
  int acc = 0, bb = 0, ii = 0;
  for (int base = 0; base < B; base += (int)blockDim.x) {
    const int b = base + (int)threadIdx.x;
    chunk[threadIdx.x] = b < B ? n[b] : 0;
    __syncthreads();
    if (threadIdx.x == 0) {
      const int here = min((int)blockDim.x, B - base);
      for (int j = 0; j < here; ++j) {
        const int nb = chunk[j];
        if (m >= acc && m < acc + nb) { bb = base + j; ii = m - acc; }
        acc += nb;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) { where[0] = bb; where[1] = ii; }
  __syncthreads();
}
// row_start[0..B] = running sums of the counts, read the same way
__device__ __forceinline__ void packed_row_starts(const int* __restrict__ n, int B, int* chunk, int* __restrict__ row_start) {
  int acc = 0;
  for (int base = 0; base < B; base += (int)blockDim.x) {
    const int b = base + (int)threadIdx.x;
    chunk[threadIdx.x] = b < B ? n[b] : 0;
    __syncthreads();
    if (threadIdx.x == 0) {
      const int here = min((int)blockDim.x, B - base);
      for (int j = 0; j < here; ++j) { row_start[base + j] = acc; acc += chunk[j]; }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) row_start[B] = acc;
  __syncthreads();
}
// Verify call: sequence b feeds (pending_b, draft_b[0..k_b-2]) at positions len_b .. len_b+k_b-1
// (Section 3.2, the verifier equation conditions row i on the accepted prefix and the first
// i-1 drafted tokens).  The row tables and the embedding of the rows in one launch: workgroup 0
// writes the per-sequence tables the later kernels read; workgroup m + 1 finds row m's (sequence, block
// index) by the same scan, writes the row's table entries and embeds it.  (k and the draft live in host memory:
// a workgroup makes two trips over the bus, one for the counts and one for its token; a workgroup 0 that walked
// the sequences one after the other made two trips per sequence, 10-40 us per call at 32 sequences.)
template <typename T>
__global__ __launch_bounds__(128) void k_assemble_embed_verify(const int* __restrict__ k, const int* __restrict__ draft,
                                                               const int* __restrict__ rows, int rows_stride,
                                                               const int* __restrict__ len,
                                                               const int* __restrict__ pending, const T* __restrict__ emb,
                                                               const float* __restrict__ pe, float* __restrict__ x,
                                                               T* __restrict__ xa, int k_max, int B, int d, float sqrt_d,
                                                               int M, int l_cap, int s_max,
                                                               const int* __restrict__ src_len, VerifyTables t) {
  // k lives in host memory (a trip over the bus); with one sequence it is the row count M
  __shared__ int where[2];
  __shared__ int chunk[128];
  if (blockIdx.x != 0) {
    const int m = blockIdx.x - 1;
    // rows (host memory, written by the caller of several sequences): row m's (sequence << 14 | index) and, behind
    // them, the token it feeds (-1: the sequence's pending token); both requested at once
    int b, i, tok;
    if (rows) {
      const int w = rows[m], fed = rows[rows_stride + m];
      b = w >> 14; i = w & 0x3fff;
      tok = fed < 0 ? pending[b] : fed;
    } else {
      if (B > 1) locate_packed_row(k, B, m, chunk, where);
      b = B > 1 ? where[0] : 0; i = B > 1 ? where[1] : m;
      tok = i == 0 ? pending[b] : draft[b * k_max + i - 1];
    }
    const int L = len[b];
    if (threadIdx.x == 0) {
      t.row_tok[m] = tok;
      t.row_pos[m] = L + i;
      t.row_seq[m] = b;
      t.row_dst[m] = b * l_cap + L + i;
    }
    const T* e = emb + (size_t)tok * d;
    const float* p = pe + (size_t)(L + i) * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
      const float v = embed_value(Store<T>::load(e + c), sqrt_d, p[c]);
      x[(size_t)m * d + c] = v;
      Store<T>::store(xa + (size_t)m * d + c, v);
    }
    return;
  }
  // workgroup 0: the per-sequence tables
  if (B > 1) packed_row_starts(k, B, chunk, t.row_start);
  else {
    if (threadIdx.x == 0) { t.row_start[0] = 0; t.row_start[1] = M; }
    __syncthreads();
  }
  for (int b = threadIdx.x; b < B; b += blockDim.x) {
    SeqDesc s;
    s.q_row0 = t.row_start[b]; s.nq = t.row_start[b + 1] - t.row_start[b]; s.kv_row0 = b * l_cap; s.nk_base = len[b]; s.causal = 1;
    s.pad0 = s.pad1 = s.pad2 = 0;
    t.self_desc[b] = s;
    s.kv_row0 = b * s_max; s.nk_base = src_len[b]; s.causal = 0;
    t.cross_desc[b] = s;
  }
}
void launch_assemble_embed_verify(int dtype, const int* k, const int* draft, const int* rows, int rows_stride, int k_max, const int* len,
                                  const int* pending, const int* src_len, int B, int l_cap, int s_max, VerifyTables t,
                                  int M, const void* emb, const float* pe, int d, float sqrt_d, float* x, void* xa,
                                  hipStream_t s) {
  if (M <= 0) return;
  if (dtype == AD_BF16)
    k_assemble_embed_verify<bf16_t><<<M + 1, 128, 0, s>>>(k, draft, rows, rows_stride, len, pending, (const bf16_t*)emb, pe, x, (bf16_t*)xa, k_max,
                                                      B, d, sqrt_d, M, l_cap, s_max, src_len, t);
  else
    k_assemble_embed_verify<float><<<M + 1, 128, 0, s>>>(k, draft, rows, rows_stride, len, pending, (const float*)emb, pe, x, (float*)xa, k_max, B,
                                                     d, sqrt_d, M, l_cap, s_max, src_len, t);
}

// Encoder: rows = x_1..x_n of every sentence at positions 0..n-1, full self-attention over the
// sentence's own rows (keys live in the packed temporary buffers, row_dst = identity); the
// cross_desc slot describes where the memory keys/values of each sentence go.
// The encoder's tables, the embedding of its rows and the per-call device state in one launch
// (src, src_len, max_out may live in host memory): workgroup 0 writes the per-sequence tables, keeps the
// source lengths and, for the verifier (len != null), the output limits and the start state of a
// decode; workgroup m + 1 writes row m's table entries and embeds it.
template <typename T>
__global__ __launch_bounds__(128) void k_assemble_embed_encoder(const int* __restrict__ src, int max_src,
                                                                const int* __restrict__ src_len,
                                                                const int* __restrict__ max_out_in, int B, int s_max,
                                                                VerifyTables t, int* __restrict__ src_len_out,
                                                                int* __restrict__ max_out, int* __restrict__ len,
                                                                int* __restrict__ pending, int* __restrict__ finished,
                                                                int bos, const T* __restrict__ emb,
                                                                const float* __restrict__ pe, int d, float sqrt_d,
                                                                float* __restrict__ x, T* __restrict__ xa) {
  __shared__ int where[2];
  __shared__ int chunk[128];
  if (blockIdx.x != 0) {
    const int m = blockIdx.x - 1;
    locate_packed_row(src_len, B, m, chunk, where);
    const int b = where[0], i = where[1];
    const int tok = src[b * max_src + i];
    if (threadIdx.x == 0) {
      t.row_tok[m] = tok;
      t.row_pos[m] = i;
      t.row_seq[m] = b;
      t.row_dst[m] = m;                   // own keys/values: packed temporaries
      t.row_dst2[m] = b * s_max + i;      // where this row's memory key/value goes
    }
    const T* e = emb + (size_t)tok * d;
    const float* p = pe + (size_t)i * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
      const float v = embed_value(Store<T>::load(e + c), sqrt_d, p[c]);
      x[(size_t)m * d + c] = v;
      Store<T>::store(xa + (size_t)m * d + c, v);
    }
    return;
  }
  packed_row_starts(src_len, B, chunk, t.row_start);
  for (int b = threadIdx.x; b < B; b += blockDim.x) {
    const int n = t.row_start[b + 1] - t.row_start[b];
    SeqDesc s;
    s.q_row0 = t.row_start[b]; s.nq = n; s.kv_row0 = t.row_start[b]; s.nk_base = n; s.causal = 0;
    s.pad0 = s.pad1 = s.pad2 = 0;
    t.self_desc[b] = s;
    src_len_out[b] = n;
    if (len) { max_out[b] = max_out_in[b]; len[b] = 0; pending[b] = bos; finished[b] = 0; }
  }
}
void launch_assemble_embed_encoder(int dtype, const int* src, int max_src, const int* src_len, const int* max_out_in,
                                   int B, int s_max, VerifyTables t, int* src_len_out, int* max_out, int* len,
                                   int* pending, int* finished, int bos, int M, const void* emb, const float* pe, int d,
                                   float sqrt_d, float* x, void* xa, hipStream_t s) {
  if (M <= 0) return;
  if (dtype == AD_BF16)
    k_assemble_embed_encoder<bf16_t><<<M + 1, 128, 0, s>>>(src, max_src, src_len, max_out_in, B, s_max, t, src_len_out, max_out,
                                                           len, pending, finished, bos, (const bf16_t*)emb, pe, d, sqrt_d, x,
                                                           (bf16_t*)xa);
  else
    k_assemble_embed_encoder<float><<<M + 1, 128, 0, s>>>(src, max_src, src_len, max_out_in, B, s_max, t, src_len_out, max_out,
                                                          len, pending, finished, bos, (const float*)emb, pe, d, sqrt_d, x,
                                                          (float*)xa);
}

// Drafter: rows = (o_0..o_j, [MASK] x k) at positions 0..j+k for every unfinished sequence
// (Section 3.2, draft paragraph), bidirectional self-attention over the sequence's own rows.
// Packed row order: the k mask rows of every unfinished sequence first (sequence l's at
// [l*k, l*k + k)), then the prefix rows, so that whatever only the mask rows need (everything
// after the last layer's key/value projection, the output projection) works on the first live*k
// rows.  A sequence's keys and values stay contiguous (prefix, then masks) through row_dst.
// Descriptors: entries [0, live) = mask rows as queries, [live, 2 live) = prefix rows.
// One launch: workgroup 0 writes the tables and descriptors; workgroup r + 1 finds row r's (token,
// position) itself from the decode state (no workgroup waits for another) and writes
// x[r] = E[token] * sqrt(d) + PE[position] as k_embed does.
template <typename T>
__global__ __launch_bounds__(256) void k_assemble_embed_drafter(const int* __restrict__ out, int max_len,
                                                                const int* __restrict__ len,
                                                                const int* __restrict__ finished,
                                                                const int* __restrict__ src_len, int B, int k, int bos,
                                                                int mask, int s_max, VerifyTables t,
                                                                const T* __restrict__ emb, const float* __restrict__ pe,
                                                                int d, float sqrt_d, float* __restrict__ x,
                                                                T* __restrict__ xa) {
  if (blockIdx.x == 0) {
    __shared__ int s_live;
    if (threadIdx.x == 0) {
      int live = 0;
      for (int b = 0; b < B; ++b) live += finished[b] ? 0 : 1;
      int l = 0, kslot = 0, pre = live * k;
      for (int b = 0; b < B; ++b) {
        t.row_start[b] = kslot;
        if (finished[b]) continue;
        const int L = len[b];
        SeqDesc sd;
        sd.q_row0 = l * k; sd.nq = k; sd.kv_row0 = kslot; sd.nk_base = L + 1 + k; sd.causal = 0;
        sd.pad0 = b; sd.pad1 = pre; sd.pad2 = 0;
        t.self_desc[l] = sd;
        sd.q_row0 = pre; sd.nq = L + 1;
        t.self_desc[live + l] = sd;
        sd.kv_row0 = b * s_max; sd.nk_base = src_len[b];
        t.cross_desc[live + l] = sd;
        sd.q_row0 = l * k; sd.nq = k;
        t.cross_desc[l] = sd;
        kslot += L + 1 + k; pre += L + 1; ++l;
      }
      t.row_start[B] = kslot;
      s_live = live;
    }
    __syncthreads();
    const int live = s_live;
    for (int l = 0; l < live; ++l) {
      const SeqDesc m = t.self_desc[l];
      const int b = m.pad0, pre = m.pad1, L = m.nk_base - 1 - k, kslot = m.kv_row0;
      for (int i = threadIdx.x; i < L + 1 + k; i += blockDim.x) {
        const int row = i <= L ? pre + i : l * k + (i - L - 1);
        t.row_tok[row] = i == 0 ? bos : (i <= L ? out[b * max_len + i - 1] : mask);
        t.row_pos[row] = i;
        t.row_seq[row] = b;
        t.row_dst[row] = kslot + i;
      }
    }
    return;
  }
  const int r = blockIdx.x - 1;
  __shared__ int s_tok, s_pos;
  if (threadIdx.x == 0) {
    int live = 0;
    for (int b = 0; b < B; ++b) live += finished[b] ? 0 : 1;
    int tok = mask, pos = 0;
    if (r < live * k) {
      // mask row j of the l-th unfinished sequence: position L + 1 + j
      const int l = r / k, j = r - l * k;
      int seen = 0;
      for (int b = 0; b < B; ++b) {
        if (finished[b]) continue;
        if (seen == l) { pos = len[b] + 1 + j; break; }
        ++seen;
      }
    } else {
      int pre = live * k;
      for (int b = 0; b < B; ++b) {
        if (finished[b]) continue;
        const int L = len[b];
        if (r < pre + L + 1) {
          pos = r - pre;
          tok = pos == 0 ? bos : out[b * max_len + pos - 1];
          break;
        }
        pre += L + 1;
      }
    }
    s_tok = tok; s_pos = pos;
  }
  __syncthreads();
  const T* e = emb + (size_t)s_tok * d;
  const float* pp = pe + (size_t)s_pos * d;
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    const float v = embed_value(Store<T>::load(e + c), sqrt_d, pp[c]);
    x[(size_t)r * d + c] = v;
    Store<T>::store(xa + (size_t)r * d + c, v);
  }
}
void launch_assemble_embed_drafter(int dtype, const int* out, int max_len, const int* len, const int* finished,
                                   const int* src_len, int B, int k, int bos, int mask, int s_max, VerifyTables t,
                                   int M, const void* emb, const float* pe, int d, float sqrt_d, float* x, void* xa,
                                   hipStream_t s) {
  if (dtype == AD_BF16)
    k_assemble_embed_drafter<bf16_t><<<M + 1, 256, 0, s>>>(out, max_len, len, finished, src_len, B, k, bos, mask, s_max, t,
                                                           (const bf16_t*)emb, pe, d, sqrt_d, x, (bf16_t*)xa);
  else
    k_assemble_embed_drafter<float><<<M + 1, 256, 0, s>>>(out, max_len, len, finished, src_len, B, k, bos, mask, s_max, t,
                                                          (const float*)emb, pe, d, sqrt_d, x, (float*)xa);
}

// Drafted tokens of the unfinished sequences, back in [B, k_max] order (AD_NEVER elsewhere).
__global__ void k_draft_scatter(const int* __restrict__ o_hat, const int* __restrict__ finished, int B, int k,
                                int k_max, int* __restrict__ draft_out) {
  if (threadIdx.x != 0) return;
  int live = 0;
  for (int b = 0; b < B; ++b) {
    for (int i = 0; i < k_max; ++i) draft_out[b * k_max + i] = AD_NEVER;
    if (finished[b]) continue;
    for (int i = 0; i < k; ++i) draft_out[b * k_max + i] = o_hat[live * k + i];
    ++live;
  }
}
void launch_draft_scatter(const int* o_hat, const int* finished, int B, int k, int k_max, int* draft_out,
                          hipStream_t s) {
  k_draft_scatter<<<1, 64, 0, s>>>(o_hat, finished, B, k, k_max, draft_out);
}

// ------------------------------------------------------------------------------------- accept + rollback
// c = first i with draft_i != o_hat_i, else k (Section 3.2, the equation of c; when no position
// differs the whole block is accepted).  Appends o_hat_1..o_hat_c cut after the first [EOS] and
// at the output limit; the cache keeps one row per appended token (len += n), everything past
// it is dead and overwritten by the next call.
// One workgroup per sequence: its waves finish the arg max of the sequence's rows (argmax_row over
// the partials, as k_argmax_finish does), then one thread accepts.
__global__ __launch_bounds__(1024) void k_argmax_accept(const int* __restrict__ k, const int* __restrict__ draft,
                                                       const int* __restrict__ ticket_in, const int* __restrict__ row_start,
                                                       const float* __restrict__ pv, const int* __restrict__ pi,
                                                       int* __restrict__ len, int M, int k_max, int stride, int n_part,
                                                       const int* __restrict__ max_out, int* __restrict__ o_hat,
                                                       float* __restrict__ o_val, int eos, int max_len,
                                                       int* __restrict__ pending, int* __restrict__ finished,
                                                       int* __restrict__ out, int* __restrict__ result,
                                                       unsigned long long* __restrict__ ticket_out, GadppIn gp) {
  const int b = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  // what the end of the kernel needs and nothing here depends on is requested first (k, the draft and the ticket
  // sit in host memory, one trip over the bus for all of them: the draft as all of the sequence's slots, so that
  // its request does not wait for k)
  const int my_draft = (int)threadIdx.x < k_max ? draft[b * k_max + threadIdx.x] : 0;
  const int ticket = threadIdx.x == 0 && ticket_out ? *ticket_in : 0;
  const int kb = gridDim.x == 1 ? M : k[b];   // a lone sequence owns all M rows
  if (kb == 0) {
    if (threadIdx.x == 0) {
      if (ticket_out) __hip_atomic_store(ticket_out + b, (unsigned long long)ticket << 46, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      else { result[2 * b] = 0; result[2 * b + 1] = 0; }
    }
    return;
  }
  const int r0 = row_start[b];
  __shared__ int s_first, s_eos;
  const int L = len[b], lim = max_out[b];
  if (threadIdx.x == 0) { s_first = kb; s_eos = kb; }
  for (int i = wave; i < kb; i += (int)(blockDim.x >> 6)) {
    const int m = r0 + i;
    float v;
    int idx;
    argmax_row(pv + (size_t)m * stride, pi + (size_t)m * stride, n_part, lane, v, idx);
    if (gp.part_cnt) {
      // relaxed verification (both inequalities of the GAD++ requirement, on fp32 scores: log-likelihood
      // differences are score differences): the drafted token stands in for the arg max if fewer than beta
      // columns score above it and the top score exceeds its score by at most tau
      int cnt = 0;
      for (int j = lane; j < gp.n_part; j += 64) cnt += gp.part_cnt[(size_t)m * gp.stride + j];
      cnt = row16_sum_i(cnt);
      cnt = __builtin_amdgcn_readlane(cnt, 0) + __builtin_amdgcn_readlane(cnt, 16) + __builtin_amdgcn_readlane(cnt, 32) +
            __builtin_amdgcn_readlane(cnt, 48);
      const int tok = gp.col[m];
      if (tok >= 0 && cnt < gp.beta && v - gp.lp[m] <= gp.tau) idx = tok;
    }
    if (lane == 0) {
      o_hat[m] = idx;
      if (o_val) o_val[m] = v;
    }
  }
  __syncthreads();   // the sequence's arg maxima are in memory, visible to the whole workgroup
  // first mismatch with the draft and first [EOS], every thread a row at a time
  for (int i = threadIdx.x; i < kb; i += blockDim.x) {
    const int t = o_hat[r0 + i];
    const int dr = i == (int)threadIdx.x ? my_draft : draft[b * k_max + i];
    if (dr != t) atomicMin(&s_first, i);
    if (t == eos) atomicMin(&s_eos, i);
  }
  __syncthreads();
  // accepted block = o_hat_{1..c}, cut after the first [EOS] and at the output limit
  const int c = s_first < kb ? s_first + 1 : kb;
  int n = min(c, max(lim - L, 0));
  if (s_eos < n) n = s_eos + 1;
  for (int i = threadIdx.x; i < n; i += blockDim.x) out[b * max_len + L + i] = o_hat[r0 + i];
  if (threadIdx.x != 0) return;
  const int last = n > 0 ? o_hat[r0 + n - 1] : 0;
  len[b] = L + n;
  if (n > 0) pending[b] = last;
  finished[b] = (n > 0 && last == eos) || (L + n >= lim);
  // a host that waits for this call by watching memory: ticket (18 bits), accepted length (14) and
  // next token (32) in ONE 8-byte store, so that seeing the ticket is seeing the result; no
  // release fence (it would write the whole cache back).  Nothing else is written to host memory
  // then: a plain store could still be on its way when the host, having seen the ticket, goes on.
  if (ticket_out) {
    __hip_atomic_store(ticket_out + b, ((unsigned long long)ticket << 46) | ((unsigned long long)n << 32) | (unsigned)last,
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  } else {
    result[2 * b] = n;
    result[2 * b + 1] = last;
  }
}
void launch_argmax_accept(const float* pv, const int* pi, int stride, int n_part, int* o_hat, float* o_val, const int* k,
                          const int* draft, int k_max, const int* row_start, int B, int eos, int max_len,
                          const int* max_out, int* len, int* pending, int* finished, int* out, int* result,
                          const int* ticket_in, unsigned long long* ticket_out, int max_rows, int M, hipStream_t s,
                          const GadppIn& gp) {
  // as many waves as the longest block has rows (4 to 16): a wave finishes a row at a time
  const int waves = std::min(16, std::max(4, max_rows));
  k_argmax_accept<<<B, 64 * waves, 0, s>>>(k, draft, ticket_in, row_start, pv, pi, len, M, k_max, stride, n_part, max_out,
                                    o_hat, o_val, eos, max_len, pending, finished, out, result, ticket_out, gp);
}
// ------------------------------------------------------------------------------------- GAD++ (Section 3.2.3)
// The drafted token of packed row m: draft[b][i] for row i of sequence b.
__device__ __forceinline__ int drafted_token(const int* __restrict__ row_seq, const int* __restrict__ row_start,
                                             const int* __restrict__ draft, int k_max, int m) {
  const int b = row_seq[m];
  return draft[b * k_max + (m - row_start[b])];
}
// Score of each row's drafted token.  One wave per 16 rows: the MFMA tile whose column j holds
// the weight row of row j's drafted token; its diagonal is what is asked for.  Operand layouts,
// instruction and k order are those of the output projection, and an MFMA output element is a dot
// product of its own, so lp[m] equals the logit that projection computes for (m, token), bit for bit.
__global__ __launch_bounds__(64) void k_draft_logit_bf16(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                                         int M, int N, int K, const int* __restrict__ row_seq,
                                                         const int* __restrict__ row_start,
                                                         const int* __restrict__ draft, int k_max,
                                                         float* __restrict__ lp, int* __restrict__ col) {
  const int lane = threadIdx.x, r = lane & 15, kq = lane >> 4;
  const int m = min((int)blockIdx.x * 16 + r, M - 1);
  const int tok = drafted_token(row_seq, row_start, draft, k_max, m);
  const int c = min(max(tok, 0), N - 1);
  const bf16_t* ap = A + (size_t)m * K + kq * 8;
  const bf16_t* wp = W + (size_t)(c >> 4) * 16 * K + ((c & 15) + 16 * kq) * 8;   // tile (strip, step u) at + u * 512
  f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < K; k0 += 32) {
    const bf16x8 a = __builtin_bit_cast(bf16x8, *(const uint4*)(ap + k0));
    const bf16x8 b = __builtin_bit_cast(bf16x8, *(const uint4*)(wp + k0 * 16));
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
  }
  // lane (r, kq) holds rows 4 kq .. 4 kq + 3 of column r: the diagonal element of row r sits in
  // the lane with kq = r / 4
  if (kq == (r >> 2) && (int)blockIdx.x * 16 + r < M) {
    const int i = r & 3;
    lp[m] = i == 0 ? acc[0] : i == 1 ? acc[1] : i == 2 ? acc[2] : acc[3];
    col[m] = tok;
  }
}
// fp32 path: the fused multiply-add chain of k_gemm_f32, k ascending.
__global__ void k_draft_logit_f32(const float* __restrict__ A, const float* __restrict__ W, int M, int N, int K,
                                  const int* __restrict__ row_seq, const int* __restrict__ row_start,
                                  const int* __restrict__ draft, int k_max, float* __restrict__ lp,
                                  int* __restrict__ col) {
  const int m = blockIdx.x * blockDim.x + threadIdx.x;
  if (m >= M) return;
  const int tok = drafted_token(row_seq, row_start, draft, k_max, m);
  const int c = min(max(tok, 0), N - 1);
  float acc = 0.f;
  for (int k = 0; k < K; ++k) acc = fmaf(A[(size_t)m * K + k], W[(size_t)c * K + k], acc);
  lp[m] = acc;
  col[m] = tok;
}
void launch_draft_logit(int dtype, const void* A, const void* W, int M, int N, int K, const int* row_seq,
                        const int* row_start, const int* draft, int k_max, float* lp, int* col, hipStream_t s) {
  if (M <= 0) return;
  if (dtype == AD_BF16)
    k_draft_logit_bf16<<<(M + 15) / 16, 64, 0, s>>>((const bf16_t*)A, (const bf16_t*)W, M, N, K, row_seq, row_start, draft,
                                                    k_max, lp, col);
  else
    k_draft_logit_f32<<<(M + 63) / 64, 64, 0, s>>>((const float*)A, (const float*)W, M, N, K, row_seq, row_start, draft,
                                                   k_max, lp, col);
}

}  // namespace ad

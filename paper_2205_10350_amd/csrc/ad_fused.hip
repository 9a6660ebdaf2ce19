// Persistent fused forward for small row counts (M <= 64 packed rows, bf16 mode).
//
// At batch 1 a verify forward is ~50 dependent stages that each stream at most a few MB of
// weights: far less than one memory round trip's worth of bandwidth, so one launch per stage
// is bound by launch and first-access latency.  Here ONE cooperative launch (one workgroup per
// compute unit) walks a static stage program; stages are separated by a device-wide barrier
// (relaxed atomics only: cross-workgroup data uses device-coherent accesses).  LayerNorm and the embedding are
// computed as the prologue of the GEMM that consumes them (each workgroup normalises the
// <= 64 rows into LDS itself), the output projection ends in per-strip arg-max partials, and
// the last stage (workgroup 0) finishes the arg max and runs prefix match / accept / rollback.
//
// Every value is produced by the device functions of ad_device.h in the same order as in the
// stand-alone kernels, so rows are bit-identical between the two launch styles.
#include <hip/hip_runtime.h>

#include "ad_device.h"

namespace ad {

// ------------------------------------------------------------------------------------- grid barrier
// Data that crosses workgroups inside this kernel is written and read with device-coherent
// accesses (see ad_device.h), so the barrier itself needs no cache maintenance: relaxed atomics
// only.  Two levels keep contention low: 16 workgroups share a group counter, the last arriver
// of a group bumps the top counter, the last of those publishes the phase number that everyone
// else polls.  Counters are monotonic over the life of the context (`phase` = barriers completed
// so far + 1).  bar layout (64-bit words): [0] top counter, [32] published phase, [64] abort flag,
// [96 + 32 g] counter of group g.  A workgroup that waits longer than the spin limit raises the
// abort flag; every workgroup leaves the kernel once it sees the flag, so the grid always drains.
constexpr int kBarGroup = 16;
__device__ __forceinline__ bool grid_barrier(unsigned long long* bar, unsigned long long phase) {
  __syncthreads();   // includes the wait for this workgroup's outstanding stores
  __shared__ int ok;
  if (threadIdx.x == 0) {
    const int G = gridDim.x;
    const int grp = blockIdx.x / kBarGroup, ngrp = (G + kBarGroup - 1) / kBarGroup;
    const int gsz = min(kBarGroup, G - grp * kBarGroup);
    int good = 1;
    bool last = false;
    const unsigned long long a =
        __hip_atomic_fetch_add(&bar[96 + 32 * grp], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (a + 1 == phase * (unsigned long long)gsz) {
      const unsigned long long t = __hip_atomic_fetch_add(&bar[0], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      last = t + 1 == phase * (unsigned long long)ngrp;
    }
    if (last) {
      __hip_atomic_store(&bar[32], phase, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      unsigned spins = 0;
      while (__hip_atomic_load(&bar[32], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < phase) {
        __builtin_amdgcn_s_sleep(32);
        if ((++spins & 255u) == 0) {
          if (__hip_atomic_load(&bar[64], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0ull) { good = 0; break; }
          if (spins > (1u << 21)) {
            __hip_atomic_store(&bar[64], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            good = 0;
            break;
          }
        }
      }
    }
    ok = good;
  }
  __syncthreads();
  return ok != 0;
}

// ------------------------------------------------------------------------------------- GEMM stage
// A tile in LDS: rows of (K + 8) bf16 so that the 16 lanes of a k-group read 16-byte vectors from
// different banks.
__device__ __forceinline__ void stage_a_to_lds(const Stage& st, const FusedArgs& fa, bf16_t* A) {
  const int K = st.K, ld = K + 8, M = fa.M;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, waves = blockDim.x >> 6;
  const bool write_x = blockIdx.x == 0 && st.x_out != nullptr;
  if (st.a_mode == A_LN) {
    // four rows per wave in flight: all their loads are issued before the first reduction
    const float* s = (const float*)st.a_src;
    for (int m0 = wave; m0 < M; m0 += 4 * waves) {
      float xv[4][32];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int m = m0 + u * waves;
        if (m < M) ln_load<true>(s + (size_t)m * K, K, lane, xv[u]);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int m = m0 + u * waves;
        if (m < M) {
          float mean, rstd;
          ln_stats(xv[u], K, lane, mean, rstd);
#pragma unroll
          for (int j = 0; j < 32; ++j) {
            const int c = lane + 64 * j;
            if (c < K) {
              const float o = ln_value(xv[u][j], mean, rstd, st.ln_g[c], st.ln_b[c]);
              A[m * ld + c] = f2bf(o);
              if (write_x) stg<true>(st.x_out + (size_t)m * K + c, o);
            }
          }
        }
      }
    }
  } else if (st.a_mode == A_EMBED) {
    const bf16_t* emb = (const bf16_t*)st.a_src;
    for (int m0 = wave; m0 < M; m0 += 4 * waves) {
      int tok[4], pos[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int m = m0 + u * waves;
        tok[u] = m < M ? fa.row_tok[m] : 0;
        pos[u] = m < M ? fa.row_pos[m] : 0;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int m = m0 + u * waves;
        if (m < M) {
          const bf16_t* e = emb + (size_t)tok[u] * K;
          const float* p = fa.pe + (size_t)pos[u] * K;
          for (int c = lane; c < K; c += 64) {
            const float o = embed_value(bf2f(e[c]), fa.sqrt_d, p[c]);
            A[m * ld + c] = f2bf(o);
            if (write_x) stg<true>(st.x_out + (size_t)m * K + c, o);
          }
        }
      }
    }
  } else {   // A_COPY
    const uint4* src = (const uint4*)st.a_src;
    const int vec_per_row = K / 8;
    const int n = M * vec_per_row, nt = blockDim.x;
    for (int base = threadIdx.x; base < n; base += 4 * nt) {
      uint4 v4[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = base + u * nt;
        if (i < n) v4[u] = ldg16<true>(src + i);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = base + u * nt;
        if (i < n) {
          const int m = i / vec_per_row, v = i - m * vec_per_row;
          *(uint4*)(A + m * ld + v * 8) = v4[u];
        }
      }
    }
  }
  __syncthreads();
}

template <bool A_IN_LDS>
__device__ __forceinline__ void gemm_stage(const Stage& st, const FusedArgs& fa, bf16_t* A_lds) {
  const int K = st.K, N = st.N, M = fa.M;
  const int n_strips = N >> 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
  const int G = gridDim.x;
  if ((int)blockIdx.x >= n_strips) return;          // this workgroup owns no strip
  const int mt_used = (M + 15) >> 4;
  const int r = lane & 15, kq = lane >> 4;
  const bf16_t* W = (const bf16_t*)st.W;
  const int ld = K + 8;
  // the first strip's weights do not depend on the activations: fetch them while A is staged
  uint4 b[16];
  const int first = blockIdx.x + G * wave;
  if (first < n_strips) {
    const bf16_t* wp = W + (size_t)((first << 4) + r) * K + kq * 8;
#pragma unroll
    for (int u = 0; u < 16; ++u)
      if (32 * u < K) b[u] = *(const uint4*)(wp + 32 * u);
  }
  if (A_IN_LDS) stage_a_to_lds(st, fa, A_lds);
  if (fa.stamps && blockIdx.x == 0 && threadIdx.x == 0) fa.stamps[128 + fa.dbg_si * 8 + 1] = wall_clock64();
  for (int strip = first; strip < n_strips; strip += G * waves) {
    const int n0 = strip << 4;
    const bf16_t* wp = W + (size_t)(n0 + r) * K + kq * 8;
    f32x4 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    const bf16_t* ap[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if (A_IN_LDS) {
        ap[t] = A_lds + (t * 16 + r) * ld + kq * 8;
      } else {
        int row = t * 16 + r;
        row = row < M ? row : M - 1;
        ap[t] = (const bf16_t*)st.a_src + (size_t)row * K + kq * 8;
      }
    }
    for (int k0 = 0; k0 < K; k0 += 512) {
      if (strip != first || k0 != 0) {
#pragma unroll
        for (int u = 0; u < 16; ++u)
          if (k0 + 32 * u < K) b[u] = *(const uint4*)(wp + k0 + 32 * u);
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        if (k0 + 32 * u < K) {
          const bf16x8 bv = __builtin_bit_cast(bf16x8, b[u]);
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            if (t < mt_used) {
              const uint4 araw = A_IN_LDS ? *(const uint4*)(ap[t] + k0 + 32 * u) : ldg16<true>(ap[t] + k0 + 32 * u);
              const bf16x8 av = __builtin_bit_cast(bf16x8, araw);
              acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bv, acc[t], 0, 0, 0);
            }
          }
        }
      }
    }
    if (fa.stamps && blockIdx.x == 0 && threadIdx.x == 0) fa.stamps[128 + fa.dbg_si * 8 + 2] = wall_clock64();
    strip_epilogue<bf16_t, 4, true>(st.epi, acc, mt_used, 0, n0, M, N, lane);
    if (fa.stamps && blockIdx.x == 0 && threadIdx.x == 0) fa.stamps[128 + fa.dbg_si * 8 + 3] = wall_clock64();
  }
}

// ------------------------------------------------------------------------------------- attention stage
__device__ __forceinline__ void attn_stage(const Stage& st, const FusedArgs& fa, unsigned* lds) {
  const int tasks = fa.B * fa.H;
  const float scale = 1.0f / sqrtf((float)fa.dh);
  for (int task = blockIdx.x; task < tasks; task += gridDim.x) {
    const int b = task / fa.H, h = task - b * fa.H;
    const SeqDesc sd = st.desc[b];
    if (sd.nq <= 0) continue;
    const bf16_t* q = (const bf16_t*)st.q;
    const bf16_t* Kb = (const bf16_t*)st.Kb;
    const bf16_t* Vb = (const bf16_t*)st.Vb;
    bf16_t* out = (bf16_t*)st.att_out;
    switch (fa.dh) {
      case 16: attn_block<bf16_t, 16, true>(q, Kb, Vb, out, sd, 0, sd.nq, h, fa.d, scale, lds, st.nk_cap); break;
      case 32: attn_block<bf16_t, 32, true>(q, Kb, Vb, out, sd, 0, sd.nq, h, fa.d, scale, lds, st.nk_cap); break;
      case 64: attn_block<bf16_t, 64, true>(q, Kb, Vb, out, sd, 0, sd.nq, h, fa.d, scale, lds, st.nk_cap); break;
      default: attn_block<bf16_t, 128, true>(q, Kb, Vb, out, sd, 0, sd.nq, h, fa.d, scale, lds, st.nk_cap); break;
    }
  }
}

// ------------------------------------------------------------------------------------- finish stage
// Workgroup 0: second arg-max stage for every row, then longest-prefix match, acceptance,
// truncation at [EOS] / the output limit and rollback, one thread per sequence (same rules as
// k_accept).
__device__ __forceinline__ void finish_stage(const FusedArgs& fa, int* o_lds) {
  if (blockIdx.x != 0) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, waves = blockDim.x >> 6;
  for (int m = wave; m < fa.M; m += waves) {
    float v;
    int idx;
    argmax_row<true>(fa.part_val + (size_t)m * fa.n_strips, fa.part_idx + (size_t)m * fa.n_strips, fa.n_strips, lane, v, idx);
    if (lane == 0) {
      fa.o_hat[m] = idx;
      fa.o_val[m] = v;
      o_lds[m] = idx;
    }
  }
  __syncthreads();
  if (!fa.do_accept) return;
  for (int b = threadIdx.x; b < fa.B; b += blockDim.x) {
    const int kb = fa.k[b];
    if (kb == 0) { fa.result[2 * b] = 0; fa.result[2 * b + 1] = 0; continue; }
    const int r0 = fa.row_start[b];
    int c = kb;
    for (int i = 0; i < kb; ++i)
      if (fa.draft[b * fa.k_max + i] != o_lds[r0 + i]) { c = i + 1; break; }
    const int L = fa.len[b], lim = fa.max_out[b];
    int n = 0, last = 0;
    for (int i = 0; i < c; ++i) {
      if (L + n >= lim) break;
      last = o_lds[r0 + i];
      fa.out[b * fa.max_len + L + n] = last;
      ++n;
      if (last == fa.eos) break;
    }
    fa.len[b] = L + n;
    if (n > 0) fa.pending[b] = last;
    fa.finished[b] = (n > 0 && last == fa.eos) || (L + n >= lim);
    fa.result[2 * b] = n;
    fa.result[2 * b + 1] = last;
  }
}

// ------------------------------------------------------------------------------------- the kernel
__global__ __launch_bounds__(512) void k_fused_forward(FusedArgs fa) {
  fa.dbg_si = 0;
  extern __shared__ uint4 fused_lds[];
  __shared__ int o_lds[64];
  unsigned long long phase = fa.bar_base;   // barriers completed before this launch
  for (int si = 0; si < fa.n_stages; ++si) {
    const Stage& st = fa.stages[si];
    fa.dbg_si = si;
    if (si > 0) {
      if (fa.stamps && blockIdx.x == 0 && threadIdx.x == 0) fa.stamps[128 + si * 8 + 4] = wall_clock64();
      ++phase;
      if (!grid_barrier(fa.bar, phase)) return;
    }
    if (fa.stamps && blockIdx.x == 0 && threadIdx.x == 0) { fa.stamps[si] = wall_clock64(); fa.stamps[64 + si] = clock64(); }
    if (st.type == ST_GEMM) {
      if (st.a_mode == A_GLOBAL) gemm_stage<false>(st, fa, nullptr);
      else gemm_stage<true>(st, fa, (bf16_t*)fused_lds);
    } else if (st.type == ST_ATTN) {
      attn_stage(st, fa, (unsigned*)fused_lds);
    } else {
      finish_stage(fa, o_lds);
    }
  }
  if (fa.stamps && blockIdx.x == 0 && threadIdx.x == 0) fa.stamps[fa.n_stages] = wall_clock64();
}

int fused_max_blocks_per_cu(size_t lds_bytes) {
  int n = 0;
  if (hipFuncSetAttribute((const void*)k_fused_forward, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) !=
      hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, (const void*)k_fused_forward, 512, lds_bytes) != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  return n;
}

hipError_t launch_fused_forward(const FusedArgs& fa, int grid, size_t lds_bytes, hipStream_t s) {
  FusedArgs a = fa;
  void* params[] = {(void*)&a};
  return hipLaunchCooperativeKernel((const void*)k_fused_forward, dim3(grid), dim3(512), params, (unsigned)lds_bytes, s);
}

}  // namespace ad

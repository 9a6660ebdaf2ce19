// Persistent single-launch verify forward (bf16 mode).
//
// A verify forward is ~50 dependent stages that each move little data; launched one by one they
// are bound by launch and first-access latency, not by bandwidth.  Here ONE cooperative launch
// (one workgroup per compute unit) walks a static stage program.
//
// The chip is eight XCDs, each with its own L2; workgroup i of a launch runs on XCD i % 8.  A
// stage barrier plus the exchange of the stage's output costs ~5 us across XCDs (the data has to
// go through memory) but ~1.7 us among the workgroups of ONE XCD, which share an L2.  So the
// decoder layers run XCD-locally: the workgroups of an XCD form a TEAM, every team takes a
// contiguous share of the call's sequences through all layers on its own (weights are re-read
// per team, from the last-level cache; activations never leave the team's L2), synchronising
// with a team barrier only.  One device-wide barrier later all teams share the output
// projection (each wave owns 16 vocabulary columns whose weights it fetched into registers at
// kernel start, i.e. the largest tensor streams from HBM behind the layer phase), and after a
// second device-wide barrier one workgroup per sequence finishes the arg max and runs prefix
// match / accept / rollback.
//
// Visibility rules: anything another workgroup wrote in this launch is LOADED with the coherent
// policy (misses the compute unit's L1, served by the XCD's L2); data that crosses teams is also
// STORED with it (write-through to memory).  Every value is produced by the device functions of
// ad_device.h in the same order as in the stand-alone kernels, so rows are bit-identical between
// the two launch styles.
#include <hip/hip_runtime.h>

#include "ad_device.h"

namespace ad {

typedef unsigned long long u64;

constexpr int kWaves = kFusedWaves;       // waves of a workgroup: one per SIMD, so that each may use the whole register file
constexpr int kKP = kFusedMaxWidth;       // widest K slice of an A tile
// rows of an A tile: 64 with slices up to 512 wide, 32 with wider ones (same bytes)
__device__ __forceinline__ int tile_rows(int KP) { return KP > 512 ? 32 : 64; }
constexpr unsigned kSpinLimit = 1u << 21;

// Stage descriptors: the whole program is copied into LDS at kernel start (one round trip to
// memory instead of several dependent ones per stage), and a stage's fields are read from there
// into scalar registers (they are the same for every lane).
constexpr int kMaxStages = kFusedMaxStages;
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
template <typename P> __device__ __forceinline__ P* uni(P* p) {
  const unsigned long long u = (unsigned long long)p;
  const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)u);
  const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(u >> 32));
  return (P*)(((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ Stage fetch_stage(const Stage* l) {
  Stage s;
  s.type = uni(l->type); s.a_mode = uni(l->a_mode); s.N = uni(l->N); s.K = uni(l->K);
  s.W = uni(l->W); s.a_src = uni(l->a_src); s.ln_g = uni(l->ln_g); s.ln_b = uni(l->ln_b); s.x_out = uni(l->x_out);
  s.epi.mode = uni(l->epi.mode); s.epi.d = uni(l->epi.d); s.epi.bias = uni(l->epi.bias); s.epi.out0 = uni(l->epi.out0);
  s.epi.out1 = uni(l->epi.out1); s.epi.out2 = uni(l->epi.out2); s.epi.row_dst = uni(l->epi.row_dst);
  s.epi.resid = uni(l->epi.resid); s.epi.part_val = uni(l->epi.part_val); s.epi.part_idx = uni(l->epi.part_idx);
  s.epi.n_strips = uni(l->epi.n_strips); s.epi.logits = uni(l->epi.logits);
  s.q = uni(l->q); s.Kb = uni(l->Kb); s.Vb = uni(l->Vb); s.att_out = uni(l->att_out); s.desc = uni(l->desc);
  s.nk_cap = uni(l->nk_cap); s.pf_stage = uni(l->pf_stage);
  return s;
}

__device__ __forceinline__ int xcc_id() {
  int v;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(v));
  return v & 0xf;
}

// ------------------------------------------------------------------------------------- barriers
// Barrier words (64-bit, 128 bytes apart): see kBar* in ad_internal.h.  All counters are
// monotonic over the life of the context; the host passes how far each has counted.  A waiter
// that exceeds the spin limit raises the abort word; every workgroup leaves the kernel once it
// sees the word, so the grid always drains.
//
// Team barrier, first half: this workgroup's stores have reached the L2.  A wave that stored
// nothing in the stage skips the wait (it may have L2-prefetch touches in flight, which must not
// hold the barrier up).
__device__ __forceinline__ void barrier_stores_done(bool wave_stored = true) {
  if (wave_stored) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
}
// Team barrier, second half: arrive and wait until `target` arrivals.  Read-modify-write
// operations only (performed at the L2 / memory side, never served by an L1).
__device__ __forceinline__ bool team_arrive_wait(u64* bar, u64* ctr, u64 target, u64 zero, int* ok_lds) {
  if (threadIdx.x == 0) {
    int good = 1;
    u64 seen = __hip_atomic_fetch_add(ctr, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1;
    unsigned spins = 0;
    while (seen < target) {
      __builtin_amdgcn_s_sleep(20);
      seen = __hip_atomic_fetch_add(ctr, zero, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if ((++spins & 1023u) == 0) {
        if (__hip_atomic_load(&bar[kBarAbort], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0ull) { good = 0; break; }
        if (spins > kSpinLimit) {
          __hip_atomic_store(&bar[kBarAbort], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          good = 0;
          break;
        }
      }
    }
    *ok_lds = good;
  }
  __syncthreads();
  return *ok_lds != 0;
}

// Device-wide barrier, two levels to keep contention low: 16 workgroups share a group counter,
// the last arriver of a group bumps the top counter, the last of those publishes the phase
// number that everyone else polls.  `phase` = device barriers completed so far + 1.
constexpr int kBarGroup = 16;
// `patient`: poll rarely.  A workgroup that waits for a long time (a team without rows, while the
// others run their layers) must not flood the memory channel that holds the barrier word:
// every poll is a read that goes all the way to memory.
template <bool PATIENT>
__device__ __forceinline__ bool device_barrier(u64* bar, u64 phase, int* ok_lds) {
  barrier_stores_done();
  if (threadIdx.x == 0) {
    const int G = gridDim.x;
    const int grp = blockIdx.x / kBarGroup, ngrp = (G + kBarGroup - 1) / kBarGroup;
    const int gsz = min(kBarGroup, G - grp * kBarGroup);
    int good = 1;
    bool last = false;
    const u64 a = __hip_atomic_fetch_add(&bar[kBarDevGroup + 16 * grp], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (a + 1 == phase * (u64)gsz) {
      const u64 t = __hip_atomic_fetch_add(&bar[kBarDevTop], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      last = t + 1 == phase * (u64)ngrp;
    }
    if (last) {
      __hip_atomic_store(&bar[kBarDevPhase], phase, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      unsigned spins = 0;
      while (__hip_atomic_load(&bar[kBarDevPhase], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < phase) {
        if (PATIENT) { __builtin_amdgcn_s_sleep(127); __builtin_amdgcn_s_sleep(127); }   // ~7 us
        else __builtin_amdgcn_s_sleep(8);
        if ((++spins & 255u) == 0) {
          if (__hip_atomic_load(&bar[kBarAbort], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0ull) { good = 0; break; }
          if (spins > kSpinLimit) {
            __hip_atomic_store(&bar[kBarAbort], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            good = 0;
            break;
          }
        }
      }
    }
    *ok_lds = good;
  }
  __syncthreads();
  return *ok_lds != 0;
}

// ------------------------------------------------------------------------------------- weights
// Weights are stored as B-operand tiles: step u (32 k) of a 16-column strip is 1 KB contiguous,
// lane l's 8 values at + l * 8 elements.  They never change during a launch: ordinary loads.
//
// (1) Into registers, 128 k (four steps) at a time: see mfma_k.
// (2) Ahead of a stage, into the wave's LDS slot, by loads that write LDS directly (no register
// is involved, so nothing waits for them until the stage reads the slot): step u lands at
// slot + u KB with lane l's 16 bytes at + 16 l, exactly as the MFMA reads it back.
__device__ __forceinline__ void w_prefetch(const bf16_t* strip_base, int steps, char* slot) {
  const int lane = threadIdx.x & 63;
  for (int u = 0; u < steps; ++u)
    __builtin_amdgcn_global_load_lds((const AD_GLOBAL void*)(strip_base + 512 * u + lane * 8),
                                     (__attribute__((address_space(3))) void*)(slot + 1024 * u), 16, 0, 0);
}
// How the weight slots are shared out in a GEMM stage: the workgroup's `n_active` waves that own
// a round-0 strip (the lowest wave indices) split the 64 KB evenly, up to four of them; a slot
// holds the first `depth` k of the wave's strip (a multiple of 512, at most K).
struct WSlots { int n_active, n_slots, slot_bytes, depth; };
__device__ __forceinline__ WSlots w_slots(int n_strips, int K, int rank, int T) {
  WSlots w;
  w.n_active = rank < n_strips ? min(kWaves, (n_strips - rank + T - 1) / T) : 0;
  w.n_slots = min(w.n_active, 4);
  // whole KB per slot: every step's 1 KB block (16-byte pieces per lane) stays 16-byte aligned
  w.slot_bytes = w.n_slots ? ((kFusedWSlotBytes / w.n_slots) >> 10) << 10 : 0;
  w.depth = min(K & ~511, (w.slot_bytes >> 14) << 9);   // 16 KB per 512 k
  return w;
}
__device__ __forceinline__ char* w_slot(char* wbase, const WSlots& w, int wave) {
  return wbase + (size_t)wave * w.slot_bytes;
}
__device__ __forceinline__ void gemm_prefetch(const Stage& st, int rank, int T, char* wbase) {
  const int wave = threadIdx.x >> 6;
  const WSlots w = w_slots(st.N >> 4, st.K, rank, T);
  if (wave < w.n_slots && w.depth > 0)
    w_prefetch((const bf16_t*)st.W + (size_t)((rank + T * wave) << 4) * st.K, w.depth >> 5, w_slot(wbase, w, wave));
}

// Touches every 128-byte line of the strip this wave owns in round 0 of GEMM stage `st`, so that
// the lines sit in the XCD's L2 when the stage's real loads come (they stream from HBM / the
// last-level cache under the stages before).  The touches are loads whose destination is a junk
// word in LDS: no register waits for them.
__device__ __forceinline__ void l2_touch(const void* p, unsigned* junk) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)p,
                                   (__attribute__((address_space(3))) void*)junk, 4, 0, 0);
}
// Called by the `n_idle` waves of a workgroup that own no strip in the current stage (`idle_rank`
// = index among them): together they touch the round-0 strips this workgroup's waves will own in
// stage `nx`.  first / stride: strip of wave w = first + stride * w.
__device__ __forceinline__ void l2_prefetch_strips(const void* W, int K, int n_strips, int first, int stride,
                                                   int idle_rank, int n_idle, unsigned* junk) {
  const int lane = threadIdx.x & 63;
  const int lines = (K * 32) >> 7;          // 16 * K * 2 bytes per strip, contiguous
  for (int w = 0; w < kWaves; ++w) {
    const int strip = first + stride * w;
    if (strip >= n_strips) break;
    const char* base = (const char*)W + (size_t)(strip << 4) * K * 2;
    for (int j = idle_rank * 64 + lane; j < lines; j += n_idle * 64) l2_touch(base + (j << 7), junk);
  }
}
__device__ __forceinline__ void l2_prefetch_vectors(const Stage& nx, unsigned* junk) {
  const int lane = threadIdx.x & 63;
  if (nx.epi.bias && lane * 32 < nx.N) l2_touch(nx.epi.bias + lane * 32, junk);
  if (nx.a_mode == A_LN && lane * 32 < nx.K) { l2_touch(nx.ln_g + lane * 32, junk); l2_touch(nx.ln_b + lane * 32, junk); }
}

// ------------------------------------------------------------------------------------- A tiles
// Rows [mc, mc + rows) x columns [kp, kp + KP) of a GEMM's left operand, as bf16 in LDS, row
// stride (KP + 8) so that the 16 lanes of a k-group read 16-byte vectors from different banks.
//
// LayerNorm rows (KP == K): one wave per row, up to four rows per wave in flight so that their load
// and reduction latencies overlap; gain and bias are fetched first, under the rows' loads.
template <int NJ, bool EXACT>
__device__ __forceinline__ void stage_ln(const float* __restrict__ s, const float* __restrict__ ln_g,
                                         const float* __restrict__ ln_b, float* __restrict__ x_out, bf16_t* A, int ld,
                                         int mc, int rows, int K, bool write_x) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float gv[NJ], bv[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int c = lane + 64 * j;
    gv[j] = (EXACT || c < K) ? gload(ln_g + c) : 0.f;
    bv[j] = (EXACT || c < K) ? gload(ln_b + c) : 0.f;
  }
  constexpr int R = NJ <= 8 ? 4 : 2;   // rows per wave in flight
  for (int i0 = wave; i0 < rows; i0 += R * kWaves) {
    float xv[R][NJ];
#pragma unroll
    for (int u = 0; u < R; ++u) {
      const int i = i0 + u * kWaves;
      if (i < rows) ln_load<true, NJ, EXACT>(s + (size_t)(mc + i) * K, K, lane, xv[u]);
    }
#pragma unroll
    for (int u = 0; u < R; ++u) {
      const int i = i0 + u * kWaves;
      if (i < rows) {
        float mean, rstd;
        ln_stats<NJ, EXACT>(xv[u], K, lane, mean, rstd);
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const int c = lane + 64 * j;
          if (EXACT || c < K) {
            const float o = ln_value(xv[u][j], mean, rstd, gv[j], bv[j]);
            A[i * ld + c] = f2bf(o);
            if (write_x) gstore(x_out + (size_t)(mc + i) * K + c, o);
          }
        }
      }
    }
  }
}

// The 16-byte rule (widths 256, 512, 1024): NV = K / 256.
template <int NV>
__device__ __forceinline__ void stage_ln4(const float* __restrict__ s, const float* __restrict__ ln_g,
                                          const float* __restrict__ ln_b, float* __restrict__ x_out, bf16_t* A, int ld,
                                          int mc, int rows, int K, bool write_x) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float4 gv[NV], bv[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    gv[j] = gload((const float4*)(ln_g + 4 * lane + 256 * j));
    bv[j] = gload((const float4*)(ln_b + 4 * lane + 256 * j));
  }
  constexpr int R = NV <= 2 ? 4 : 2;   // rows per wave in flight
  for (int i0 = wave; i0 < rows; i0 += R * kWaves) {
    float4 xv[R][NV];
#pragma unroll
    for (int u = 0; u < R; ++u) {
      const int i = i0 + u * kWaves;
      if (i < rows) ln_load4<true, NV>(s + (size_t)(mc + i) * K, lane, xv[u]);
    }
#pragma unroll
    for (int u = 0; u < R; ++u) {
      const int i = i0 + u * kWaves;
      if (i < rows) {
        float mean, rstd;
        ln_stats4<NV>(xv[u], K, mean, rstd);
#pragma unroll
        for (int j = 0; j < NV; ++j) {
          const int c = 4 * lane + 256 * j;
          const float4 o = float4{ln_value(xv[u][j].x, mean, rstd, gv[j].x, bv[j].x), ln_value(xv[u][j].y, mean, rstd, gv[j].y, bv[j].y),
                                  ln_value(xv[u][j].z, mean, rstd, gv[j].z, bv[j].z), ln_value(xv[u][j].w, mean, rstd, gv[j].w, bv[j].w)};
          *(uint2*)(A + i * ld + c) = uint2{(unsigned)f2bf(o.x) | ((unsigned)f2bf(o.y) << 16), (unsigned)f2bf(o.z) | ((unsigned)f2bf(o.w) << 16)};
          if (write_x) gstore((float4*)(x_out + (size_t)(mc + i) * K + c), o);
        }
      }
    }
  }
}

__device__ __forceinline__ void stage_a(int a_mode, int K, const void* a_src, const float* __restrict__ ln_g,
                                        const float* __restrict__ ln_b, float* __restrict__ x_out,
                                        const FusedArgs& fa, bf16_t* A, int mc, int rows, int kp, int KP,
                                        bool write_x) {
  const int ld = KP + 8;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (a_mode == A_LN) {
    const float* s = (const float*)a_src;
    if (K == 512) stage_ln4<2>(s, ln_g, ln_b, x_out, A, ld, mc, rows, K, write_x);
    else if (K == 1024) stage_ln4<4>(s, ln_g, ln_b, x_out, A, ld, mc, rows, K, write_x);
    else if (K == 256) stage_ln4<1>(s, ln_g, ln_b, x_out, A, ld, mc, rows, K, write_x);
    else if (K < 256) stage_ln<4, false>(s, ln_g, ln_b, x_out, A, ld, mc, rows, K, write_x);
    else stage_ln<16, false>(s, ln_g, ln_b, x_out, A, ld, mc, rows, K, write_x);
  } else if (a_mode == A_EMBED) {
    // one wave per row, four rows per wave in flight; a lane owns 8 consecutive columns
    const bf16_t* emb = (const bf16_t*)a_src;
    for (int i0 = wave; i0 < rows; i0 += 4 * kWaves) {
      int tok[4], pos[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + u * kWaves;
        tok[u] = i < rows ? gload(fa.row_tok + mc + i) : 0;
        pos[u] = i < rows ? gload(fa.row_pos + mc + i) : 0;
      }
      for (int c0 = lane * 8; c0 < K; c0 += 512) {
        uint4 ev[4];
        float4 p0[4], p1[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int i = i0 + u * kWaves;
          if (i < rows) {
            ev[u] = gload((const uint4*)(emb + (size_t)tok[u] * K + c0));
            p0[u] = gload((const float4*)(fa.pe + (size_t)pos[u] * K + c0));
            p1[u] = gload((const float4*)(fa.pe + (size_t)pos[u] * K + c0 + 4));
          }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int i = i0 + u * kWaves;
          if (i < rows) {
            const unsigned w[4] = {ev[u].x, ev[u].y, ev[u].z, ev[u].w};
            const float pe[8] = {p0[u].x, p0[u].y, p0[u].z, p0[u].w, p1[u].x, p1[u].y, p1[u].z, p1[u].w};
            float o[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              o[2 * j] = embed_value(__uint_as_float(w[j] << 16), fa.sqrt_d, pe[2 * j]);
              o[2 * j + 1] = embed_value(__uint_as_float(w[j] & 0xFFFF0000u), fa.sqrt_d, pe[2 * j + 1]);
            }
            uint4 pk;
            pk.x = (unsigned)f2bf(o[0]) | ((unsigned)f2bf(o[1]) << 16);
            pk.y = (unsigned)f2bf(o[2]) | ((unsigned)f2bf(o[3]) << 16);
            pk.z = (unsigned)f2bf(o[4]) | ((unsigned)f2bf(o[5]) << 16);
            pk.w = (unsigned)f2bf(o[6]) | ((unsigned)f2bf(o[7]) << 16);
            *(uint4*)(A + i * ld + c0) = pk;
            if (write_x) {
              gstore((float4*)(x_out + (size_t)(mc + i) * K + c0), float4{o[0], o[1], o[2], o[3]});
              gstore((float4*)(x_out + (size_t)(mc + i) * K + c0 + 4), float4{o[4], o[5], o[6], o[7]});
            }
          }
        }
      }
    }
  } else {   // A_COPY: storage-type rows [*, K]; one wave per row, lanes over its 16-byte vectors
    const bf16_t* src = (const bf16_t*)a_src + (size_t)mc * K + kp;
    const int vpr = KP >> 3;
    if (vpr <= 64) {
      // up to four rows per wave in flight
      for (int i0 = wave; i0 < rows; i0 += 4 * kWaves) {
        uint4 v4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int i = i0 + u * kWaves;
          if (i < rows && lane < vpr) v4[u] = ldg16<true>(src + (size_t)i * K + lane * 8);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int i = i0 + u * kWaves;
          if (i < rows && lane < vpr) *(uint4*)(A + i * ld + lane * 8) = v4[u];
        }
      }
    } else {
      // wide slices (vpr = 128): two vectors per lane per row, two rows in flight
      for (int i0 = wave; i0 < rows; i0 += 2 * kWaves) {
        uint4 v4[2][2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int i = i0 + u * kWaves;
#pragma unroll
          for (int h = 0; h < 2; ++h)
            if (i < rows && lane + 64 * h < vpr) v4[u][h] = ldg16<true>(src + (size_t)i * K + (lane + 64 * h) * 8);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int i = i0 + u * kWaves;
#pragma unroll
          for (int h = 0; h < 2; ++h)
            if (i < rows && lane + 64 * h < vpr) *(uint4*)(A + i * ld + (lane + 64 * h) * 8) = v4[u][h];
        }
      }
    }
  }
}

// MFMA over k for the first MT 16-row tiles, in groups of G steps of 32 k: first every operand
// read of the group is issued (A from the LDS tile, B from the weight slot or from memory), then
// its MFMAs run, so that a wave that has its SIMD to itself pays the read latency once per group.
// `a_lds` = this lane's row and k-group in the A tile.
//
// B from memory into registers (`wp` = strip base + first step * 512 + lane * 8): the path of
// weights that were not fetched ahead.
template <int MT>
__device__ __forceinline__ void mfma_regs(const bf16_t* __restrict__ a_lds, int ld, const bf16_t* __restrict__ wp,
                                          int k_len, f32x4 (&acc)[4]) {
  constexpr int G = MT <= 2 ? 4 : 2;
  const int steps = k_len >> 5;
#pragma unroll 1
  for (int s0 = 0; s0 < steps; s0 += 16) {      // up to 512 k: all their weights are requested at once
    uint4 b[16];
#pragma unroll
    for (int u = 0; u < 16; ++u)
      if (s0 + u < steps) b[u] = gload((const uint4*)(wp + 512 * (s0 + u)));
#pragma unroll
    for (int g0 = 0; g0 < 16; g0 += G) {
      if (s0 + g0 < steps) {
        uint4 a[G][MT];
#pragma unroll
        for (int g = 0; g < G; ++g)
          if (s0 + g0 + g < steps) {
#pragma unroll
            for (int t = 0; t < MT; ++t) a[g][t] = *(const uint4*)(a_lds + t * 16 * ld + 32 * (s0 + g0 + g));
          }
#pragma unroll
        for (int g = 0; g < G; ++g)
          if (s0 + g0 + g < steps) {
            const bf16x8 bv = __builtin_bit_cast(bf16x8, b[g0 + g]);
#pragma unroll
            for (int t = 0; t < MT; ++t)
              acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[g][t]), bv, acc[t], 0, 0, 0);
          }
      }
    }
  }
}
// mt = 16-row tiles in use (1..4)
__device__ __forceinline__ void mfma_k(int mt, const bf16_t* __restrict__ a_lds, int ld, const bf16_t* __restrict__ wp,
                                       int k_len, f32x4 (&acc)[4]) {
  switch (mt) {
    case 1: mfma_regs<1>(a_lds, ld, wp, k_len, acc); break;
    case 2: mfma_regs<2>(a_lds, ld, wp, k_len, acc); break;
    case 3: mfma_regs<3>(a_lds, ld, wp, k_len, acc); break;
    default: mfma_regs<4>(a_lds, ld, wp, k_len, acc); break;
  }
}

// B read back from the wave's weight slot (`w_lds` = slot + first step * 1 KB + lane * 16).
template <int MT>
__device__ __forceinline__ void mfma_lds(const bf16_t* __restrict__ a_lds, int ld, const char* __restrict__ w_lds,
                                         int steps, f32x4 (&acc)[4]) {
  constexpr int G = MT <= 2 ? 4 : 2;
#pragma unroll 1
  for (int u0 = 0; u0 < steps; u0 += G) {
    uint4 b[G], a[G][MT];
#pragma unroll
    for (int g = 0; g < G; ++g)
      if (u0 + g < steps) {
        b[g] = *(const uint4*)(w_lds + 1024 * (u0 + g));
#pragma unroll
        for (int t = 0; t < MT; ++t) a[g][t] = *(const uint4*)(a_lds + t * 16 * ld + 32 * (u0 + g));
      }
#pragma unroll
    for (int g = 0; g < G; ++g)
      if (u0 + g < steps) {
        const bf16x8 bv = __builtin_bit_cast(bf16x8, b[g]);
#pragma unroll
        for (int t = 0; t < MT; ++t)
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[g][t]), bv, acc[t], 0, 0, 0);
      }
  }
}
__device__ __forceinline__ void mfma_k_lds(int mt, const bf16_t* __restrict__ a_lds, int ld, const char* __restrict__ w_lds,
                                           int steps, f32x4 (&acc)[4]) {
  switch (mt) {
    case 1: mfma_lds<1>(a_lds, ld, w_lds, steps, acc); break;
    case 2: mfma_lds<2>(a_lds, ld, w_lds, steps, acc); break;
    case 3: mfma_lds<3>(a_lds, ld, w_lds, steps, acc); break;
    default: mfma_lds<4>(a_lds, ld, w_lds, steps, acc); break;
  }
}

// ------------------------------------------------------------------------------------- GEMM stage (team)
// Strip s of the stage belongs to workgroup s % T of the team, wave (s / T) % 8, round s / (8T).
// The first `depth` k of every round-0 strip sit in the wave's weight slot (fetched during the
// barrier before the stage); everything else comes from memory into registers.
// Returns whether this wave stored anything (i.e. owned a strip).
__device__ __forceinline__ bool gemm_stage(const Stage& st, const Stage* prog, const FusedArgs& fa, int m_lo, int m_hi, int rank, int T,
                                           bf16_t* A, char* wbase, unsigned* junk, u64* stp, int si) {
  const int K = st.K, N = st.N, n_strips = N >> 4;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 15, kq = lane >> 4;
  const int KP = K < kKP ? K : kKP, ld = KP + 8, MC = tile_rows(KP);
  const bf16_t* W = (const bf16_t*)st.W;
  const Epi& epi = st.epi;
  const WSlots ws = w_slots(n_strips, K, rank, T);
  const char* my_slot = w_slot(wbase, ws, wave) + lane * 16;
  bool first = true;
  for (int round = 0; rank + T * kWaves * round < n_strips; ++round) {
    const int strip = rank + T * (wave + kWaves * round);
    const bool active = strip < n_strips;
    const int n0 = strip << 4;
    const bf16_t* wp = W + (size_t)n0 * K + lane * 8;
    const bool write_x = rank == 0 && round == 0;
    const int in_lds = (round == 0 && wave < ws.n_slots) ? ws.depth : 0;   // k below this: weight slot
    for (int mc = m_lo; mc < m_hi; mc += MC) {
      const int rows = min(MC, m_hi - mc);
      const int mt = (rows + 15) >> 4;
      EpiRegs<4> eg;
      eg.bias = 0.f;
#pragma unroll
      for (int q = 0; q < 16; ++q) eg.aux[q] = 0u;
      f32x4 acc[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
      for (int kp = 0; kp < K; kp += KP) {
        if (!first) __syncthreads();            // the previous tile is no longer read
        if (stp && threadIdx.x == 0 && first) fa.stamps[576 + 4 * si + 0] = wall_clock64();
        stage_a(st.a_mode, K, st.a_src, st.ln_g, st.ln_b, st.x_out, fa, A, mc, rows, kp, KP, write_x);
        if (stp && threadIdx.x == 0 && first) fa.stamps[576 + 4 * si + 1] = wall_clock64();
        // the tile's loads, the x rows' stores and the weight slot's fetches are done
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (stp && threadIdx.x == 0 && first) fa.stamps[576 + 4 * si + 2] = wall_clock64();
        __syncthreads();
        if (stp && threadIdx.x == 0) stp[3] = wall_clock64();
        if (first && st.pf_stage != -1 && wave >= ws.n_active) {
          // Waves without a strip in this stage start the weights of a later stage streaming into
          // the XCD's L2 (they have no loads of their own left that could queue up behind these).
          if (st.pf_stage >= 0) {
            const Stage nx = fetch_stage(prog + st.pf_stage);
            l2_prefetch_strips(nx.W, nx.K, nx.N >> 4, rank, T, wave - ws.n_active, kWaves - ws.n_active, junk);
            if (wave == ws.n_active) l2_prefetch_vectors(nx, junk);
          } else {
            l2_prefetch_strips(fa.out_w, fa.d, fa.V >> 4, blockIdx.x, gridDim.x, wave - ws.n_active, kWaves - ws.n_active, junk);
          }
        }
        if (active) {
          // the epilogue's operands: in flight under the last pass's MFMAs
          if (kp + KP >= K) epi_preload<4, true>(epi, mt, mc, n0, m_hi, N, lane, eg);
          const bf16_t* a_lane = A + r * ld + kq * 8;
          // k in [kp, kp + KP): first what sits in the weight slot, then the rest from memory
          const int lds_end = min(max(in_lds, kp), kp + KP);
          if (lds_end > kp) mfma_k_lds(mt, a_lane, ld, my_slot + (size_t)(kp >> 5) * 1024, (lds_end - kp) >> 5, acc);
          if (lds_end < kp + KP) mfma_k(mt, a_lane + (lds_end - kp), ld, wp + (size_t)lds_end * 16, kp + KP - lds_end, acc);
        }
        first = false;
      }
      if (stp && threadIdx.x == 0) stp[4] = wall_clock64();
      if (active) epi_apply<bf16_t, 4, false>(epi, acc, eg, mt, mc, n0, m_hi, N, lane);
      if (stp && threadIdx.x == 0) stp[5] = wall_clock64();
    }
  }
  return rank + T * wave < n_strips;
}

// ------------------------------------------------------------------------------------- attention stage (team)
// Tasks = (sequence of the team, head, chunk of query rows); the rows of a sequence are cut into
// chunks so that every workgroup of the team has one.
__device__ __forceinline__ void attn_stage(const Stage& st, const FusedArgs& fa, int s_lo, int s_hi, int rank, int T,
                                           unsigned* lds) {
  const int nbh = (s_hi - s_lo) * fa.H;
  const int split = nbh < T ? T / nbh : 1;
  const int tasks = nbh * split;
  const float scale = 1.0f / sqrtf((float)fa.dh);
  const bf16_t* q = (const bf16_t*)st.q;
  const bf16_t* Kb = (const bf16_t*)st.Kb;
  const bf16_t* Vb = (const bf16_t*)st.Vb;
  bf16_t* out = (bf16_t*)st.att_out;
  for (int task = rank; task < tasks; task += T) {
    const int c = task % split, bh = task / split;
    const int b = s_lo + bh / fa.H, h = bh % fa.H;
    const SeqDesc sd = gload(st.desc + b);
    if (sd.nq <= 0) continue;
    const int rc = (sd.nq + split - 1) / split;
    const int rb = c * rc, re = min(sd.nq, rb + rc);
    for (int r0 = rb; r0 < re; r0 += 64) {
      const int r1 = min(re, r0 + 64);
      switch (fa.dh) {
        case 16: attn_block<bf16_t, 16, true, false>(q, Kb, Vb, out, sd, r0, r1, h, fa.d, scale, lds, st.nk_cap); break;
        case 32: attn_block<bf16_t, 32, true, false>(q, Kb, Vb, out, sd, r0, r1, h, fa.d, scale, lds, st.nk_cap); break;
        case 64: attn_block<bf16_t, 64, true, false>(q, Kb, Vb, out, sd, r0, r1, h, fa.d, scale, lds, st.nk_cap); break;
        default: break;   // other head widths never reach this kernel (the host keeps them on the staged path)
      }
    }
  }
}

// ------------------------------------------------------------------------------------- LayerNorm stage (team)
// The last LayerNorm: one wave per row, output rows in the storage type, visible device-wide.
template <int NV>
__device__ __forceinline__ void ln_row4_out(const float* __restrict__ sr, const float* __restrict__ g,
                                            const float* __restrict__ b, int K, int lane, bf16_t* __restrict__ outr) {
  float4 xv[NV];
  float mean, rstd;
  ln_load4<true, NV>(sr, lane, xv);
  ln_stats4<NV>(xv, K, mean, rstd);
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int c = 4 * lane + 256 * j;
    const float4 gv = gload((const float4*)(g + c)), bv = gload((const float4*)(b + c));
    const unsigned lo = (unsigned)f2bf(ln_value(xv[j].x, mean, rstd, gv.x, bv.x)) | ((unsigned)f2bf(ln_value(xv[j].y, mean, rstd, gv.y, bv.y)) << 16);
    const unsigned hi = (unsigned)f2bf(ln_value(xv[j].z, mean, rstd, gv.z, bv.z)) | ((unsigned)f2bf(ln_value(xv[j].w, mean, rstd, gv.w, bv.w)) << 16);
    stg<true>((unsigned long long*)(outr + c), (unsigned long long)lo | ((unsigned long long)hi << 32));
  }
}
__device__ __forceinline__ void ln_stage(const Stage& st, int m_lo, int m_hi, int rank, int T) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, K = st.K;
  const float* s = (const float*)st.a_src;
  bf16_t* out = (bf16_t*)st.epi.out0;
  for (int m = m_lo + rank * kWaves + wave; m < m_hi; m += T * kWaves) {
    const float* sr = s + (size_t)m * K;
    bf16_t* outr = out + (size_t)m * K;
    const int nv = ln_vector_width(K);
    if (nv == 2) { ln_row4_out<2>(sr, st.ln_g, st.ln_b, K, lane, outr); continue; }
    if (nv == 4) { ln_row4_out<4>(sr, st.ln_g, st.ln_b, K, lane, outr); continue; }
    if (nv == 1) { ln_row4_out<1>(sr, st.ln_g, st.ln_b, K, lane, outr); continue; }
    float xv[16], mean, rstd;
    ln_load<true, 16>(sr, K, lane, xv);
    ln_stats<16>(xv, K, lane, mean, rstd);
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int c = lane + 64 * j;
      if (c < K) stg<true>(outr + c, f2bf(ln_value(xv[j], mean, rstd, gload(st.ln_g + c), gload(st.ln_b + c))));
    }
  }
}

// ------------------------------------------------------------------------------------- output projection (all teams)
// Strip s belongs to workgroup s % G, wave (s / G) % 8, round s / (8G).  Per chunk of rows the
// workgroup's waves merge their strips' (value, index) maxima through LDS into ONE partial per
// (row, workgroup).  The first kVocabDepth k of every round-0 strip sit in the wave's weight slot
// (16 KB each), fetched by vocab_prefetch; the rest of the strip was touched into the L2 then.
constexpr int kVocabDepth = 512;
__device__ __forceinline__ void vocab_prefetch(const FusedArgs& fa, char* wbase, unsigned* junk) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int strip = blockIdx.x + gridDim.x * wave;
  if (strip >= (fa.V >> 4)) return;
  const bf16_t* base = (const bf16_t*)fa.out_w + (size_t)(strip << 4) * fa.d;
  const int depth = min(kVocabDepth, fa.d);
  w_prefetch(base, depth >> 5, wbase + wave * (kFusedWSlotBytes / kWaves));
  const int lines = (fa.d * 32) >> 7;
  for (int j = ((depth * 32) >> 7) + lane; j < lines; j += 64) l2_touch((const char*)base + (j << 7), junk);
  // the strips of later rounds come from memory during the stage: touch them whole
  for (int s2 = strip + gridDim.x * kWaves; s2 < (fa.V >> 4); s2 += gridDim.x * kWaves) {
    const char* b2 = (const char*)fa.out_w + (size_t)(s2 << 4) * fa.d * 2;
    for (int j = lane; j < lines; j += 64) l2_touch(b2 + (j << 7), junk);
  }
}
__device__ __forceinline__ void vocab_tile(const FusedArgs& fa, const bf16_t* A, const char* wbase, float* red_val,
                                           int* red_idx, int mc, int mt, int MC) {
  const int K = fa.d, N = fa.V, n_strips = N >> 4, M = fa.M, G = gridDim.x;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 15, kq = lane >> 4;
  const int ld = K + 8;
  const bf16_t* W = (const bf16_t*)fa.out_w;
  const bf16_t* a_lane = A + r * ld + kq * 8;
  const int depth = min(kVocabDepth, K);
  for (int round = 0; blockIdx.x + G * kWaves * round < n_strips; ++round) {
    const int strip = blockIdx.x + G * (wave + kWaves * round);
    if (strip >= n_strips) continue;
    const int n0 = strip << 4;
    const bf16_t* wp = W + (size_t)n0 * K + lane * 8;
    f32x4 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    int k0 = 0;
    if (round == 0) {
      mfma_k_lds(mt, a_lane, ld, wbase + wave * (kFusedWSlotBytes / kWaves) + lane * 16, depth >> 5, acc);
      k0 = depth;
    }
    if (k0 < K) mfma_k(mt, a_lane + k0, ld, wp + (size_t)k0 * 16, K - k0, acc);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if (t >= mt) break;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int ml = t * 16 + kq * 4 + i, m = mc + ml;
        float v = acc[t][i];
        int idx = n0 + r;
        if (fa.logits && m < M) gstore(fa.logits + (size_t)m * N + n0 + r, v);
        argmax_row16(v, idx);
        if (r == 0) {
          float cv = red_val[wave * 64 + ml];
          int ci = red_idx[wave * 64 + ml];
          argmax_merge(cv, ci, v, idx);
          red_val[wave * 64 + ml] = cv;
          red_idx[wave * 64 + ml] = ci;
        }
      }
    }
  }
}

__device__ __forceinline__ void vocab_stage(const FusedArgs& fa, bf16_t* A, const char* wbase, float* red_val,
                                            int* red_idx) {
  const int K = fa.d, M = fa.M, MC = tile_rows(K);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if ((int)blockIdx.x >= (fa.V >> 4)) return;
  for (int mc = 0; mc < M; mc += MC) {
    const int rows = min(MC, M - mc);
    if (mc > 0) __syncthreads();
    stage_a(A_COPY, K, fa.xa, nullptr, nullptr, nullptr, fa, A, mc, rows, 0, K, false);
    // this wave's running maxima start empty (slot [wave][row])
    red_val[wave * 64 + lane] = -INFINITY;
    red_idx[wave * 64 + lane] = 0x7fffffff;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the tile's loads and the weight slot's fetches are done
    __syncthreads();
    vocab_tile(fa, A, wbase, red_val, red_idx, mc, (rows + 15) >> 4, MC);
    __syncthreads();
    if ((int)threadIdx.x < rows) {
      float v = red_val[threadIdx.x];
      int idx = red_idx[threadIdx.x];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) argmax_merge(v, idx, red_val[w * 64 + threadIdx.x], red_idx[w * 64 + threadIdx.x]);
      const size_t o = (size_t)(mc + threadIdx.x) * fa.part_stride + blockIdx.x;
      stg<true>(fa.part_val + o, v);
      stg<true>(fa.part_idx + o, idx);
    }
  }
}

// ------------------------------------------------------------------------------------- finish stage
// Workgroup b % G takes sequence b: second arg-max stage for its rows, then longest-prefix
// match, acceptance, truncation at [EOS] / the output limit and rollback (same rules as k_accept).
__device__ __forceinline__ void finish_stage(const FusedArgs& fa, int* o_lds) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, G = gridDim.x;
  const int n_part = min(G, fa.V >> 4);
  for (int b = blockIdx.x; b < fa.B; b += G) {
    const int kb = gload(fa.k + b), r0 = gload(fa.row_start + b);
    __syncthreads();
    // second arg-max stage: one wave per row, four rows per wave in flight (up to 256 partials
    // per row are held four per lane; more go through the general routine)
    for (int i0 = wave; i0 < kb; i0 += 4 * kWaves) {
      float pv[4][4];
      int pi[4][4];
      if (n_part <= 256) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int i = i0 + u * kWaves;
          const size_t o = (size_t)(r0 + i) * fa.part_stride;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int t = lane + 64 * j;
            const bool live = i < kb && t < n_part;
            pv[u][j] = live ? ldg<true>(fa.part_val + o + t) : -INFINITY;
            pi[u][j] = live ? ldg<true>(fa.part_idx + o + t) : 0x7fffffff;
          }
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + u * kWaves;
        if (i >= kb) break;
        float v;
        int idx;
        if (n_part <= 256) {
          v = pv[u][0]; idx = pi[u][0];
#pragma unroll
          for (int j = 1; j < 4; ++j) argmax_merge(v, idx, pv[u][j], pi[u][j]);
          argmax_wave(v, idx);
        } else {
          const size_t o = (size_t)(r0 + i) * fa.part_stride;
          argmax_row<true>(fa.part_val + o, fa.part_idx + o, n_part, lane, v, idx);
        }
        if (lane == 0) {
          stg<true>(fa.o_hat + r0 + i, idx);
          stg<true>(fa.o_val + r0 + i, v);
          o_lds[i] = idx;
        }
      }
    }
    __syncthreads();
    if (wave != 0 || !fa.do_accept) continue;
    // wave 0: c = first position whose draft token differs from the arg max (else k); the block
    // o_hat_1..o_hat_c is cut after the first [EOS] and at the output limit
    if (kb == 0) {
      if (lane == 0) { stg<true>(fa.result + 2 * b, 0); stg<true>(fa.result + 2 * b + 1, 0); }
      continue;
    }
    const int L = gload(fa.len + b), lim = gload(fa.max_out + b);
    int c = kb, e = kb;                     // first mismatch (1-based length), first [EOS] position (0-based)
    for (int i0 = 0; i0 < kb && c == kb && e == kb; i0 += 64) {
      const int i = i0 + lane;
      const int oh = i < kb ? o_lds[i] : 0;
      const bool mis = i < kb && gload(fa.draft + b * fa.k_max + i) != oh;
      const bool eos = i < kb && oh == fa.eos;
      const unsigned long long mm = __ballot(mis), me = __ballot(eos);
      if (mm) c = i0 + __builtin_ctzll(mm) + 1;
      if (me) e = i0 + __builtin_ctzll(me);
    }
    int n = min(c, max(lim - L, 0));
    if (e < n) n = e + 1;                   // keep the [EOS] itself
    for (int i = lane; i < n; i += 64) stg<true>(fa.out + b * fa.max_len + L + i, o_lds[i]);
    if (lane == 0) {
      const int last = n > 0 ? o_lds[n - 1] : 0;
      stg<true>(fa.len + b, L + n);
      if (n > 0) stg<true>(fa.pending + b, last);
      stg<true>(fa.finished + b, (int)((n > 0 && last == fa.eos) || (L + n >= lim)));
      stg<true>(fa.result + 2 * b, n);
      stg<true>(fa.result + 2 * b + 1, last);
    }
  }
}

// ------------------------------------------------------------------------------------- the kernel
__global__ __launch_bounds__(kWaves * 64) void k_fused_forward(FusedArgs fa) {
  extern __shared__ uint4 fused_lds[];
  __shared__ int ok_lds;
  __shared__ unsigned junk_lds[64];   // destination of the L2-prefetch touches
  __shared__ Stage prog[kMaxStages];  // the layer-phase program
  for (int i = threadIdx.x; i < fa.n_stages * (int)(sizeof(Stage) / 4); i += blockDim.x)
    ((unsigned*)prog)[i] = gload((const unsigned*)fa.stages + i);
  __syncthreads();
  bf16_t* A = (bf16_t*)fused_lds;
  char* wbase = (char*)fused_lds + kFusedATileBytes;                       // weight slots
  char* tail = (char*)fused_lds + kFusedATileBytes + kFusedWSlotBytes;     // arg-max merge slots
  float* red_val = (float*)tail;
  int* red_idx = (int*)(tail + kWaves * 64 * 4);
  const int G = gridDim.x, nt = fa.n_teams;
  const int team = blockIdx.x % nt, rank = blockIdx.x / nt, T = (G - team + nt - 1) / nt;
  // Workgroups go to the XCDs round-robin, starting at an XCD that differs from launch to launch:
  // workgroup i sits on XCD (i + off) % n_teams.  Every workgroup votes its `off` into this
  // launch's placement word; one set bit = every team sits on one XCD.
  u64* place = &fa.bar[kBarPlacement + (int)((fa.dev_base >> 1) & 1)];
  if (threadIdx.x == 0) {
    const int off = (xcc_id() - team + 2 * nt) % nt;
    __hip_atomic_fetch_or(place, 1ull << off, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // A team without rows fetches its output-projection strips right away: the largest tensor
  // then streams from HBM behind the other teams' layer phase.  A team with rows does so after
  // its layers (the weight slots are in use until then).
  const int m_lo = fa.team_row[team], m_hi = fa.team_row[team + 1];
  if (m_hi <= m_lo) {
    vocab_prefetch(fa, wbase, junk_lds);
  } else {
    // ---- layer phase of this team
    const int s_lo = fa.team_seq[team], s_hi = fa.team_seq[team + 1];
    u64* ctr = &fa.bar[kBarTeam + 16 * team];
    u64 target = fa.team_base[team];
    bool wave_stored = true;
    {
      const Stage s0 = fetch_stage(prog);
      if (s0.type == ST_GEMM) gemm_prefetch(s0, rank, T, wbase);
    }
    for (int si = 0; si < fa.n_stages; ++si) {
      const Stage st = fetch_stage(prog + si);
      u64* stp = (fa.stamps && rank == 0) ? fa.stamps + 64 + 8 * si : nullptr;
      if (si > 0) {
        if (stp && threadIdx.x == 0) stp[0] = wall_clock64();
        barrier_stores_done(wave_stored);
        if (stp && threadIdx.x == 0) stp[1] = wall_clock64();
        if (st.type == ST_GEMM) gemm_prefetch(st, rank, T, wbase);
        if (stp) {   // diagnostic: how long this wave's weight fetch takes when nothing else is in flight
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          if (threadIdx.x == 0) stp[6] = wall_clock64();
        }
        target += (u64)T;
        if (!team_arrive_wait(fa.bar, ctr, target, fa.zero, &ok_lds)) return;
        if (stp && threadIdx.x == 0) stp[2] = wall_clock64();
      }
      if (fa.stamps && rank == 0 && threadIdx.x == 0) { fa.stamps[si] = wall_clock64(); }
      wave_stored = true;
      if (st.type == ST_GEMM) wave_stored = gemm_stage(st, prog, fa, m_lo, m_hi, rank, T, A, wbase, junk_lds, stp, si);
      else if (st.type == ST_ATTN) attn_stage(st, fa, s_lo, s_hi, rank, T, (unsigned*)fused_lds);
      else ln_stage(st, m_lo, m_hi, rank, T);
    }
    __syncthreads();   // the last stage no longer reads the weight slots
    vocab_prefetch(fa, wbase, junk_lds);
  }
  if (fa.stamps && rank == 0 && m_hi > m_lo && threadIdx.x == 0) fa.stamps[fa.n_stages] = wall_clock64();
  // ---- output projection over all rows, shared by all teams
  if (m_hi <= m_lo) {
    if (!device_barrier<true>(fa.bar, fa.dev_base + 1, &ok_lds)) return;
  } else {
    if (!device_barrier<false>(fa.bar, fa.dev_base + 1, &ok_lds)) return;
  }
  if (fa.stamps && blockIdx.x == 0 && threadIdx.x == 0) fa.stamps[fa.n_stages + 1] = wall_clock64();
  vocab_stage(fa, A, wbase, red_val, red_idx);
  if (fa.stamps && blockIdx.x == 0 && threadIdx.x == 0) fa.stamps[fa.n_stages + 2] = wall_clock64();
  if (!device_barrier<false>(fa.bar, fa.dev_base + 2, &ok_lds)) return;
  if (fa.stamps && blockIdx.x == 0 && threadIdx.x == 0) fa.stamps[fa.n_stages + 3] = wall_clock64();
  // A team spread over several XCDs may have read stale rows: then leave the decode state
  // untouched (the host sees the word and repeats the call with one launch per stage).
  {
    const u64 votes = __hip_atomic_load(place, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((votes & (votes - 1)) != 0ull) return;
    // the next launch votes into the other word: clear it (nobody touches it during this launch)
    if (blockIdx.x == 0 && threadIdx.x == 0)
      __hip_atomic_store(&fa.bar[kBarPlacement + (int)(((fa.dev_base >> 1) + 1) & 1)], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  finish_stage(fa, (int*)fused_lds);
  if (fa.stamps && blockIdx.x == 0 && threadIdx.x == 0) fa.stamps[fa.n_stages + 4] = wall_clock64();
}

// Records the XCD of every workgroup of a launch shaped like the persistent one.
__global__ __launch_bounds__(kWaves * 64) void k_probe_placement(int* xcc) {
  extern __shared__ uint4 fused_lds[];
  if (threadIdx.x == 0) {
    xcc[blockIdx.x] = xcc_id();
    ((volatile int*)fused_lds)[0] = 0;
  }
}

int fused_max_blocks_per_cu(size_t lds_bytes) {
  int n = 0;
  if (hipFuncSetAttribute((const void*)k_fused_forward, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) !=
          hipSuccess ||
      hipFuncSetAttribute((const void*)k_probe_placement, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) !=
          hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, (const void*)k_fused_forward, kWaves * 64, lds_bytes) != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  return n;
}

hipError_t launch_probe_placement(int* xcc_dev, int grid, size_t lds_bytes, hipStream_t s) {
  k_probe_placement<<<grid, kWaves * 64, lds_bytes, s>>>(xcc_dev);
  return hipGetLastError();
}

hipError_t launch_fused_forward(const FusedArgs& fa, int grid, size_t lds_bytes, hipStream_t s) {
  FusedArgs a = fa;
  void* params[] = {(void*)&a};
  return hipLaunchCooperativeKernel((const void*)k_fused_forward, dim3(grid), dim3(kWaves * 64), params, (unsigned)lds_bytes, s);
}

}  // namespace ad

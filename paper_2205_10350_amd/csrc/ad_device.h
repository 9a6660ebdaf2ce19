// Device functions shared by the stand-alone kernels and the persistent fused forward.
// Everything that decides a value's bits (reduction orders, rounding points, fused
// multiply-adds) lives here exactly once, so that both launch styles give bit-identical rows.
#pragma once

#include <hip/hip_runtime.h>

#include "ad_internal.h"

namespace ad {

typedef unsigned short bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((unsigned)v) << 16); }
__device__ __forceinline__ bf16_t f2bf(float f) {   // round to nearest, ties to even
  unsigned u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
// Memory access policy.  COH = false: ordinary cached accesses (data produced by an earlier
// launch).  COH = true: device-coherent accesses that bypass the per-XCD L2 (volatile accesses:
// ordinary coalesced vector loads/stores carrying the system-coherence cache policy).  The
// persistent kernel uses them for everything one workgroup writes and another reads in a later
// stage, so that its stage barrier needs no cache write-back or invalidate.
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
template <bool COH, typename V> __device__ __forceinline__ V ldg(const V* p) {
  if constexpr (COH) return *(const volatile V*)p;
  else return *p;
}
template <bool COH, typename V> __device__ __forceinline__ void stg(V* p, V v) {
  if constexpr (COH) *(volatile V*)p = v;
  else *p = v;
}
template <bool COH> __device__ __forceinline__ uint4 ldg16(const void* p) {
  if constexpr (COH) {
    const u32x4_t v = *(const volatile u32x4_t*)p;
    return uint4{v[0], v[1], v[2], v[3]};
  } else {
    return *(const uint4*)p;
  }
}

template <typename T> struct Store;
template <> struct Store<float> {
  template <bool COH = false> static __device__ __forceinline__ float load(const float* p) { return ldg<COH>(p); }
  template <bool COH = false> static __device__ __forceinline__ void store(float* p, float v) { stg<COH>(p, v); }
  static __device__ __forceinline__ float round(float v) { return v; }
};
template <> struct Store<bf16_t> {
  template <bool COH = false> static __device__ __forceinline__ float load(const bf16_t* p) { return bf2f(ldg<COH>(p)); }
  template <bool COH = false> static __device__ __forceinline__ void store(bf16_t* p, float v) { stg<COH>(p, f2bf(v)); }
  static __device__ __forceinline__ float round(float v) { return bf2f(f2bf(v)); }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
// (value, index) maximum with the lowest index winning ties: a total order, so the result does
// not depend on the shape of the reduction tree.
__device__ __forceinline__ void argmax_merge(float& v, int& i, float ov, int oi) {
  if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
}

// x = E[tok] * sqrt(d) + PE[pos], one element
__device__ __forceinline__ float embed_value(float e, float sqrt_d, float pe) { return fmaf(e, sqrt_d, pe); }

// LayerNorm statistics of one row by one wave: lane l owns elements l, l+64, ... (kept in
// registers, at most 32 per lane: d <= 2048); mean, then the biased variance of the centred
// values; eps = 1e-5.
template <bool COH = false>
__device__ __forceinline__ void ln_load(const float* __restrict__ xr, int d, int lane, float (&xv)[32]) {
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const int c = lane + 64 * j;
    xv[j] = c < d ? ldg<COH>(xr + c) : 0.f;
  }
}
__device__ __forceinline__ void ln_stats(const float (&xv)[32], int d, int lane, float& mean, float& rstd) {
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 32; ++j)
    if (lane + 64 * j < d) s += xv[j];
  mean = wave_sum(s) / (float)d;
  float v = 0.f;
#pragma unroll
  for (int j = 0; j < 32; ++j)
    if (lane + 64 * j < d) {
      const float t = xv[j] - mean;
      v = fmaf(t, t, v);
    }
  rstd = 1.0f / sqrtf(wave_sum(v) / (float)d + 1e-5f);
}
template <bool COH = false>
__device__ __forceinline__ void ln_load_stats(const float* __restrict__ xr, int d, int lane, float (&xv)[32],
                                              float& mean, float& rstd) {
  ln_load<COH>(xr, d, lane, xv);
  ln_stats(xv, d, lane, mean, rstd);
}
__device__ __forceinline__ float ln_value(float x, float mean, float rstd, float g, float b) {
  const float t = (x - mean) * rstd;
  return fmaf(t, g, b);
}

// ------------------------------------------------------------------------------------- GEMM epilogue
// Epilogue of one 16-column strip held in MFMA C layout (lane l: column n0 + l%16, rows
// m0 + 4*(l/16) + i of tile t).  Everything the stores depend on (bias, destination rows,
// residual values) is loaded first, in one batch, so that no store waits behind a load.
// For EPI_ARGMAX the 16 lanes of a row reduce to one (value, index) partial.
template <typename T, int MT, bool COH = false>
__device__ __forceinline__ void strip_epilogue(const Epi& e, const f32x4 (&acc)[MT], int mt_used, int m0, int n0,
                                               int M, int N, int lane) {
  const int r = lane & 15, kq = lane >> 4, n = n0 + r;
  if (e.mode == EPI_ARGMAX) {
    const int strip = n0 >> 4;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      if (t >= mt_used) break;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int m = m0 + t * 16 + kq * 4 + i;
        float v = acc[t][i];
        int idx = n;
        if (e.logits && m < M) e.logits[(size_t)m * N + n] = v;
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) {
          float ov = __shfl_xor(v, o, 64);
          int oi = __shfl_xor(idx, o, 64);
          argmax_merge(v, idx, ov, oi);
        }
        if (r == 0 && m < M) {
          stg<COH>(e.part_val + (size_t)m * e.n_strips + strip, v);
          stg<COH>(e.part_idx + (size_t)m * e.n_strips + strip, idx);
        }
      }
    }
    return;
  }
  const float bias = e.bias ? e.bias[n] : 0.f;
  const int mode = e.mode, d = e.d;
  int dst[MT * 4];
  float res[MT * 4];
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = m0 + t * 16 + kq * 4 + i;
      const bool live = t < mt_used && m < M;
      dst[t * 4 + i] = (live && (mode == EPI_QKV || mode == EPI_KV)) ? e.row_dst[m] : 0;
      res[t * 4 + i] = (live && mode == EPI_RESID) ? ldg<COH>(e.resid + (size_t)m * N + n) : 0.f;
    }
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = m0 + t * 16 + kq * 4 + i;
      if (t >= mt_used || m >= M) continue;
      float v = acc[t][i];
      if (e.bias) v += bias;
      switch (mode) {
        case EPI_QKV:
          if (n < d) Store<T>::template store<COH>((T*)e.out0 + (size_t)m * d + n, v);
          else if (n < 2 * d) Store<T>::template store<COH>((T*)e.out1 + (size_t)dst[t * 4 + i] * d + (n - d), v);
          else Store<T>::template store<COH>((T*)e.out2 + (size_t)dst[t * 4 + i] * d + (n - 2 * d), v);
          break;
        case EPI_KV:
          if (n < d) Store<T>::template store<COH>((T*)e.out1 + (size_t)dst[t * 4 + i] * d + n, v);
          else Store<T>::template store<COH>((T*)e.out2 + (size_t)dst[t * 4 + i] * d + (n - d), v);
          break;
        case EPI_STORE: Store<T>::template store<COH>((T*)e.out0 + (size_t)m * N + n, v); break;
        case EPI_RELU: Store<T>::template store<COH>((T*)e.out0 + (size_t)m * N + n, fmaxf(v, 0.f)); break;
        case EPI_RESID: stg<COH>((float*)e.out0 + (size_t)m * N + n, v + res[t * 4 + i]); break;
        default: break;
      }
    }
}

// Epilogue of a single element (fp32 GEMM path).
template <typename T>
__device__ __forceinline__ void epi_store(const Epi& e, int m, int n, int N, float acc) {
  if (e.bias) acc += e.bias[n];
  switch (e.mode) {
    case EPI_QKV: {
      const int d = e.d;
      if (n < d) Store<T>::store((T*)e.out0 + (size_t)m * d + n, acc);
      else if (n < 2 * d) Store<T>::store((T*)e.out1 + (size_t)e.row_dst[m] * d + (n - d), acc);
      else Store<T>::store((T*)e.out2 + (size_t)e.row_dst[m] * d + (n - 2 * d), acc);
      break;
    }
    case EPI_KV: {
      const int d = e.d;
      if (n < d) Store<T>::store((T*)e.out1 + (size_t)e.row_dst[m] * d + n, acc);
      else Store<T>::store((T*)e.out2 + (size_t)e.row_dst[m] * d + (n - d), acc);
      break;
    }
    case EPI_STORE: Store<T>::store((T*)e.out0 + (size_t)m * N + n, acc); break;
    case EPI_RELU: Store<T>::store((T*)e.out0 + (size_t)m * N + n, fmaxf(acc, 0.f)); break;
    case EPI_RESID: ((float*)e.out0)[(size_t)m * N + n] = acc + e.resid[(size_t)m * N + n]; break;
    default: break;
  }
}

// Second stage of the arg max for one row by one wave; partials are loaded eight at a time.
template <bool COH = false>
__device__ __forceinline__ void argmax_row(const float* __restrict__ pv, const int* __restrict__ pi, int n_strips,
                                           int lane, float& v, int& idx) {
  v = -INFINITY;
  idx = 0x7fffffff;
  for (int t0 = lane; t0 < n_strips; t0 += 64 * 8) {
    float pvv[8];
    int pii[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int t = t0 + 64 * u;
      pvv[u] = t < n_strips ? ldg<COH>(pv + t) : -INFINITY;
      pii[u] = t < n_strips ? ldg<COH>(pi + t) : 0x7fffffff;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) argmax_merge(v, idx, pvv[u], pii[u]);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(v, o, 64);
    int oi = __shfl_xor(idx, o, 64);
    argmax_merge(v, idx, ov, oi);
  }
}

// ------------------------------------------------------------------------------------- attention
// Block-level attention of one (sequence, head) over query rows [row_begin, row_end) of the
// sequence.  The head's keys and values are staged in LDS once (rows padded by one dword so that
// lanes reading different keys hit different banks); then one wave per query row:
//   pass 1  lane t scores keys t, t+64, ..: dot product with c ascending, times `scale`;
//           exact row maximum
//   pass 2  p = exp(s - max); the denominator sums the unrounded p; numerators are rounded to
//           the storage type
//   pass 3  lane c accumulates output channel c over the keys in ascending order
// LDS bytes needed: attn_lds_bytes().
template <typename T> struct LdsRow;
template <> struct LdsRow<bf16_t> {
  static constexpr int kPerDword = 2;
  static __device__ __forceinline__ void unpack(unsigned w, float& lo, float& hi) {
    lo = __uint_as_float(w << 16);
    hi = __uint_as_float(w & 0xFFFF0000u);
  }
};
template <> struct LdsRow<float> {
  static constexpr int kPerDword = 1;
};

__host__ __device__ inline size_t attn_lds_bytes(int nk_cap, int dh, int esz, int waves) {
  const size_t row_dwords = (size_t)dh * esz / 4 + 1;
  return 2 * (size_t)nk_cap * row_dwords * 4 + 64 * (size_t)dh * 4 + (size_t)waves * nk_cap * 4;
}

template <typename T, int DH, bool COH = false>
__device__ void attn_block(const T* __restrict__ q, const T* __restrict__ Kb, const T* __restrict__ Vb,
                           T* __restrict__ out, const SeqDesc sd, int row_begin, int row_end, int h, int d,
                           float scale, unsigned* lds, int nk_cap) {
  constexpr int RD = DH * (int)sizeof(T) / 4;   // dwords per key row
  constexpr int RS = RD + 1;                    // padded row stride
  const int waves = blockDim.x >> 6, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  unsigned* Ks = lds;
  unsigned* Vs = lds + (size_t)nk_cap * RS;
  float* Qs = (float*)(lds + 2 * (size_t)nk_cap * RS);            // [<= 64 query rows][DH]
  float* sc = Qs + 64 * DH + (size_t)wave * nk_cap;                // this wave's score row
  const int nk_all = sd.causal ? sd.nk_base + row_end : sd.nk_base;   // keys the last row of this call sees
  {
    // stage keys, values and the query rows; loads are issued four deep so that their latencies overlap
    const unsigned* kg = (const unsigned*)(Kb + (size_t)sd.kv_row0 * d + h * DH);
    const unsigned* vg = (const unsigned*)(Vb + (size_t)sd.kv_row0 * d + h * DH);
    const size_t gs = (size_t)d * sizeof(T) / 4;   // global row stride in dwords
    const int n = nk_all * RD, nt = blockDim.x;
    for (int base = threadIdx.x; base < n; base += 4 * nt) {
      unsigned kv[4], vv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = base + u * nt;
        if (i < n) {
          const int t = i / RD, w = i - t * RD;
          kv[u] = ldg<COH>(kg + t * gs + w);
          vv[u] = ldg<COH>(vg + t * gs + w);
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = base + u * nt;
        if (i < n) {
          const int t = i / RD, w = i - t * RD;
          Ks[t * RS + w] = kv[u];
          Vs[t * RS + w] = vv[u];
        }
      }
    }
    const int nq = (row_end - row_begin) * DH;
    for (int base = threadIdx.x; base < nq; base += 4 * nt) {
      float qv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = base + u * nt;
        if (i < nq) {
          const int rr = i / DH, c = i - rr * DH;
          qv[u] = Store<T>::template load<COH>(q + (size_t)(sd.q_row0 + row_begin + rr) * d + h * DH + c);
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = base + u * nt;
        if (i < nq) Qs[i] = qv[u];
      }
    }
  }
  __syncthreads();
  for (int i = row_begin + wave; i < row_end; i += waves) {
    const int m = sd.q_row0 + i;
    const int nk = sd.causal ? sd.nk_base + i + 1 : sd.nk_base;
    const float* qs = Qs + (i - row_begin) * DH;
    float mx = -INFINITY;
    for (int t = lane; t < nk; t += 64) {
      const unsigned* kr = Ks + t * RS;
      float a = 0.f;
      if constexpr (sizeof(T) == 2) {
#pragma unroll 8
        for (int w = 0; w < RD; ++w) {
          float lo, hi;
          LdsRow<bf16_t>::unpack(kr[w], lo, hi);
          a = fmaf(qs[2 * w], lo, a);
          a = fmaf(qs[2 * w + 1], hi, a);
        }
      } else {
#pragma unroll 8
        for (int w = 0; w < RD; ++w) a = fmaf(qs[w], __uint_as_float(kr[w]), a);
      }
      a *= scale;
      sc[t] = a;
      mx = fmaxf(mx, a);
    }
    mx = wave_max(mx);
    float l = 0.f;
    for (int t = lane; t < nk; t += 64) {
      const float p = expf(sc[t] - mx);
      l += p;
      sc[t] = Store<T>::round(p);
    }
    l = wave_sum(l);
    __builtin_amdgcn_wave_barrier();
    for (int c = lane; c < DH; c += 64) {
      float a = 0.f;
      if constexpr (sizeof(T) == 2) {
        const bf16_t* vcol = (const bf16_t*)Vs + c;
        for (int t = 0; t < nk; ++t) a = fmaf(sc[t], bf2f(vcol[(size_t)t * RS * 2]), a);
      } else {
        const float* vcol = (const float*)Vs + c;
        for (int t = 0; t < nk; ++t) a = fmaf(sc[t], vcol[(size_t)t * RS], a);
      }
      Store<T>::template store<COH>(out + (size_t)m * d + h * DH + c, a / l);
    }
    __builtin_amdgcn_wave_barrier();
  }
  __syncthreads();
}

}  // namespace ad

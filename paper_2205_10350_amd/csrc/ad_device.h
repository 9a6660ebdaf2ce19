// Device functions shared by the kernels.  Everything that decides a value's bits (reduction
// orders, rounding points, fused multiply-adds) lives here exactly once, so that a row's result does
// not depend on which kernel computes it.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>

#include "ad_internal.h"

namespace ad {

typedef unsigned short bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((unsigned)v) << 16); }
__device__ __forceinline__ bf16_t f2bf(float f) {   // round to nearest, ties to even (the hardware conversion)
  return __builtin_bit_cast(bf16_t, (__bf16)f);
}
// Memory accesses name the global address space explicitly: that keeps the compiler from falling
// back to the slower flat instructions when it cannot see where a pointer came from.
#define AD_GLOBAL __attribute__((address_space(1)))
// (class types are moved as raw 16-, 8-, 4- or 2-byte pieces: their copy constructors take
// generic references, which would undo the address space)
template <int BYTES> struct RawPiece;
template <> struct RawPiece<16> { typedef unsigned type __attribute__((ext_vector_type(4))); };
template <> struct RawPiece<8> { typedef unsigned type __attribute__((ext_vector_type(2))); };
template <> struct RawPiece<4> { typedef unsigned type; };
template <> struct RawPiece<2> { typedef unsigned short type; };
template <typename V> struct RawOf {
  static constexpr int kPiece = sizeof(V) % 16 == 0 ? 16 : (sizeof(V) % 8 == 0 ? 8 : (sizeof(V) % 4 == 0 ? 4 : 2));
  typedef typename RawPiece<kPiece>::type piece;
  static constexpr int kCount = sizeof(V) / kPiece;
  struct Raw { piece v[kCount]; };
};
template <typename V> __device__ __forceinline__ V gload(const V* p) {
  typedef RawOf<V> R;
  typename R::Raw raw;
  const AD_GLOBAL typename R::piece* gp = (const AD_GLOBAL typename R::piece*)p;
#pragma unroll
  for (int i = 0; i < R::kCount; ++i) raw.v[i] = gp[i];
  return __builtin_bit_cast(V, raw);
}
template <typename V> __device__ __forceinline__ void gstore(V* p, V v) {
  typedef RawOf<V> R;
  const typename R::Raw raw = __builtin_bit_cast(typename R::Raw, v);
  AD_GLOBAL typename R::piece* gp = (AD_GLOBAL typename R::piece*)p;
#pragma unroll
  for (int i = 0; i < R::kCount; ++i) gp[i] = raw.v[i];
}
// 16 bytes (16-byte aligned)
__device__ __forceinline__ uint4 ldg16(const void* p) { return gload((const uint4*)p); }

template <typename T> struct Store;
template <> struct Store<float> {
  static __device__ __forceinline__ float load(const float* p) { return gload(p); }
  static __device__ __forceinline__ void store(float* p, float v) { gstore(p, v); }
  static __device__ __forceinline__ float round(float v) { return v; }
};
template <> struct Store<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf2f(gload(p)); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { gstore(p, f2bf(v)); }
  static __device__ __forceinline__ float round(float v) { return bf2f(f2bf(v)); }
};

// Wave-wide sum / maximum, all 64 lanes active, the same value in every lane.  Data-parallel
// lane moves (no LDS traffic): xor 1, xor 2 inside quads, mirror inside half rows, mirror inside
// rows of 16 lanes (every lane of a row then holds the row's total, built from commutative
// pairs, hence identical across the row), then the four rows: (r0 + r1) + (r2 + r3).
template <int CTRL> __device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);   // row_half_mirror
  v += dpp_move<0x140>(v);   // row_mirror
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
  const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
  const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
  return (r0 + r1) + (r2 + r3);
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_move<0xB1>(v));
  v = fmaxf(v, dpp_move<0x4E>(v));
  v = fmaxf(v, dpp_move<0x141>(v));
  v = fmaxf(v, dpp_move<0x140>(v));
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
  const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
  const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
  return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}
// (value, index) maximum with the lowest index winning ties: a total order, so the result does
// not depend on the shape of the reduction tree.
__device__ __forceinline__ void argmax_merge(float& v, int& i, float ov, int oi) {
  if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
}
// (value, index) maximum over each row of 16 lanes (every lane of the row gets it), and over the
// whole wave; lane moves as in wave_sum.  All 64 lanes active.
template <int CTRL> __device__ __forceinline__ int dpp_move_i(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
__device__ __forceinline__ void argmax_row16(float& v, int& i) {
  argmax_merge(v, i, dpp_move<0xB1>(v), dpp_move_i<0xB1>(i));
  argmax_merge(v, i, dpp_move<0x4E>(v), dpp_move_i<0x4E>(i));
  argmax_merge(v, i, dpp_move<0x141>(v), dpp_move_i<0x141>(i));
  argmax_merge(v, i, dpp_move<0x140>(v), dpp_move_i<0x140>(i));
}
// integer sum over each row of 16 lanes (every lane of the row gets it)
__device__ __forceinline__ int row16_sum_i(int v) {
  v += dpp_move_i<0xB1>(v);
  v += dpp_move_i<0x4E>(v);
  v += dpp_move_i<0x141>(v);
  v += dpp_move_i<0x140>(v);
  return v;
}
__device__ __forceinline__ void argmax_wave(float& v, int& i) {
  argmax_row16(v, i);
  float rv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
  int ri = __builtin_amdgcn_readlane(i, 0);
#pragma unroll
  for (int r = 1; r < 4; ++r)
    argmax_merge(rv, ri, __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16 * r)), __builtin_amdgcn_readlane(i, 16 * r));
  v = rv; i = ri;
}

// x = E[tok] * sqrt(d) + PE[pos], one element
__device__ __forceinline__ float embed_value(float e, float sqrt_d, float pe) { return fmaf(e, sqrt_d, pe); }

// LayerNorm statistics of one row by one wave: lane l owns elements l, l+64, ... (kept in
// registers, NJ per lane: d <= 64*NJ); mean, then the biased variance of the centred values;
// eps = 1e-5.  NJ only bounds the register array: the arithmetic depends on d alone.
template <int NJ = 32, bool EXACT = false>   // EXACT: d == 64 * NJ, no bounds tests
__device__ __forceinline__ void ln_load(const float* __restrict__ xr, int d, int lane, float (&xv)[NJ]) {
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int c = lane + 64 * j;
    xv[j] = (EXACT || c < d) ? gload(xr + c) : 0.f;
  }
}
template <int NJ = 32, bool EXACT = false>
__device__ __forceinline__ void ln_stats(const float (&xv)[NJ], int d, int lane, float& mean, float& rstd) {
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < NJ; ++j)
    if (EXACT || lane + 64 * j < d) s += xv[j];
  mean = wave_sum(s) / (float)d;
  float v = 0.f;
#pragma unroll
  for (int j = 0; j < NJ; ++j)
    if (EXACT || lane + 64 * j < d) {
      const float t = xv[j] - mean;
      v = fmaf(t, t, v);
    }
  rstd = 1.0f / sqrtf(wave_sum(v) / (float)d + 1e-5f);
}
// Rows whose width is 256, 512, 1024 or 2048 use 16-byte accesses instead: lane l owns the four
// consecutive elements at 4*l + 256*j, j < NV = d / 256 (ln_vector_width says which rule a width
// takes; every kernel follows it, so a row's statistics never depend on the kernel).
__host__ __device__ inline int ln_vector_width(int d) { return (d == 256 || d == 512 || d == 1024 || d == 2048) ? d / 256 : 0; }
template <int NV>
__device__ __forceinline__ void ln_load4(const float* __restrict__ xr, int lane, float4 (&xv)[NV]) {
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const uint4 u = ldg16(xr + 4 * lane + 256 * j);
    xv[j] = float4{__uint_as_float(u.x), __uint_as_float(u.y), __uint_as_float(u.z), __uint_as_float(u.w)};
  }
}
template <int NV>
__device__ __forceinline__ void ln_stats4(const float4 (&xv)[NV], int d, float& mean, float& rstd) {
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < NV; ++j) { s += xv[j].x; s += xv[j].y; s += xv[j].z; s += xv[j].w; }
  // d is a power of two here: multiplying by 1/d is the division, exactly
  const float inv_d = 1.0f / (float)d;
  mean = wave_sum(s) * inv_d;
  float v = 0.f;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    float t = xv[j].x - mean; v = fmaf(t, t, v);
    t = xv[j].y - mean; v = fmaf(t, t, v);
    t = xv[j].z - mean; v = fmaf(t, t, v);
    t = xv[j].w - mean; v = fmaf(t, t, v);
  }
  rstd = __builtin_amdgcn_rsqf(fmaf(wave_sum(v), inv_d, 1e-5f));   // hardware reciprocal square root (1 ulp)
}
__device__ __forceinline__ void ln_load_stats(const float* __restrict__ xr, int d, int lane, float (&xv)[32],
                                              float& mean, float& rstd) {
  ln_load<32>(xr, d, lane, xv);
  ln_stats<32>(xv, d, lane, mean, rstd);
}
__device__ __forceinline__ float ln_value(float x, float mean, float rstd, float g, float b) {
  const float t = (x - mean) * rstd;
  return fmaf(t, g, b);
}

// ------------------------------------------------------------------------------------- GEMM epilogue
// Operands of a strip's epilogue that do not depend on the accumulators: bias, destination rows
// (key/value rows of the cache), residual values.  Loaded in one batch, possibly long before the
// accumulators are ready, so that no store waits behind a load.
template <int MT> struct EpiRegs {
  float bias;
  unsigned aux[MT * 4];   // destination row (QKV / KV) or the residual value's bits (RESID): never both
};
// EM: the epilogue mode where the caller knows it at compile time (the mode's branches then fold
// away), -1: e.mode decides at run time.
template <int MT, int EM = -1>
__device__ __forceinline__ void epi_preload(const Epi& e, int mt_used, int m0, int n0, int M, int N, int lane,
                                            EpiRegs<MT>& g) {
  const int r = lane & 15, kq = lane >> 4, n = n0 + r;
  g.bias = e.bias ? gload(e.bias + n) : 0.f;
  const int mode = EM < 0 ? e.mode : EM;
  const bool want_dst = (mode == EPI_QKV && n0 >= e.d) || mode == EPI_KV, want_res = mode == EPI_RESID;
  // all MT tiles inside the matrix: no per-row tests (the common case away from the last rows)
  const bool full = mt_used == MT && m0 + MT * 16 <= M;
#pragma unroll
  for (int x = 0; x < MT * 4; ++x) g.aux[x] = 0u;
  if (want_dst) {
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int m = m0 + t * 16 + kq * 4 + i;
        if (full || (t < mt_used && m < M)) g.aux[t * 4 + i] = (unsigned)gload(e.row_dst + m);
      }
  } else if (want_res) {
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int m = m0 + t * 16 + kq * 4 + i;
        if (full || (t < mt_used && m < M)) g.aux[t * 4 + i] = __float_as_uint(gload(e.resid + (size_t)m * N + n));
      }
  }
}
// value = acc + bias, then the mode's operation.  A strip of 16 columns lies inside one of the
// q / k / v column ranges (d is a multiple of 16), so the destination is uniform over the wave.
template <typename T, int MT, int EM = -1>
__device__ __forceinline__ void epi_apply(const Epi& e, const f32x4 (&acc)[MT], const EpiRegs<MT>& g, int mt_used,
                                          int m0, int n0, int M, int N, int lane) {
  const int r = lane & 15, kq = lane >> 4, n = n0 + r;
  const int mode = EM < 0 ? e.mode : EM, d = e.d;
  const bool has_bias = e.bias != nullptr;
  const bool full = mt_used == MT && m0 + MT * 16 <= M;
  if (mode == EPI_RESID) {
    float* out = (float*)e.out0 + n;
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int m = m0 + t * 16 + kq * 4 + i;
        float v = acc[t][i];
        if (has_bias) v += g.bias;
        if (full || (t < mt_used && m < M)) gstore(out + (size_t)m * N, v + __uint_as_float(g.aux[t * 4 + i]));
      }
    return;
  }
  // destination of (row m, this lane's column) for the row-indexed modes
  T* base = nullptr;
  int ld = N, col = n;
  bool by_dst = false;
  if (mode == EPI_QKV) {
    ld = d;
    if (n0 < d) base = (T*)e.out0;
    else if (n0 < 2 * d) { base = (T*)e.out1; col = n - d; by_dst = true; }
    else { base = (T*)e.out2; col = n - 2 * d; by_dst = true; }
  } else if (mode == EPI_KV) {
    // columns [layer][key d | value d]: one product serves every layer's memory keys and values
    ld = d; by_dst = true;
    const int layer = n0 / (2 * d), c0 = n0 - layer * 2 * d;
    if (c0 < d) { base = (T*)((char*)e.out1 + layer * e.layer_stride); col = n - layer * 2 * d; }
    else { base = (T*)((char*)e.out2 + layer * e.layer_stride); col = n - layer * 2 * d - d; }
  } else if (mode == EPI_STORE || mode == EPI_RELU) {
    base = (T*)e.out0;
  }
  base += col;
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = m0 + t * 16 + kq * 4 + i;
      float v = acc[t][i];
      if (has_bias) v += g.bias;
      if (mode == EPI_RELU) v = fmaxf(v, 0.f);
      const size_t row = by_dst ? (size_t)g.aux[t * 4 + i] : (size_t)m;
      if (full || (t < mt_used && m < M)) Store<T>::store(base + row * ld, v);
    }
}

// Epilogue of one 16-column strip held in MFMA C layout (lane l: column n0 + l%16, rows
// m0 + 4*(l/16) + i of tile t).  For EPI_ARGMAX the 16 lanes of a row reduce to one
// (value, index) partial.
template <typename T, int MT>
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
        if (e.logits && m < M) gstore(e.logits + (size_t)m * N + n, v);
        argmax_row16(v, idx);
        if (r == 0 && m < M) {
          gstore(e.part_val + (size_t)m * e.n_strips + strip, v);
          gstore(e.part_idx + (size_t)m * e.n_strips + strip, idx);
        }
      }
    }
    return;
  }
  if (e.mode == EPI_COUNT) {
    const int strip = n0 >> 4;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      if (t >= mt_used) break;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int m = m0 + t * 16 + kq * 4 + i;
        const float th = e.thr[m < M ? m : M - 1];
        const int cnt = row16_sum_i(acc[t][i] > th ? 1 : 0);
        if (r == 0 && m < M) gstore(e.part_idx + (size_t)m * e.n_strips + strip, cnt);
      }
    }
    return;
  }
  EpiRegs<MT> g;
  epi_preload<MT>(e, mt_used, m0, n0, M, N, lane, g);
  epi_apply<T, MT>(e, acc, g, mt_used, m0, n0, M, N, lane);
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
      const int d = e.d, layer = n / (2 * d), c = n - layer * 2 * d;
      T* kb = (T*)((char*)e.out1 + layer * e.layer_stride);
      T* vb = (T*)((char*)e.out2 + layer * e.layer_stride);
      if (c < d) Store<T>::store(kb + (size_t)e.row_dst[m] * d + c, acc);
      else Store<T>::store(vb + (size_t)e.row_dst[m] * d + (c - d), acc);
      break;
    }
    case EPI_STORE: Store<T>::store((T*)e.out0 + (size_t)m * N + n, acc); break;
    case EPI_RELU: Store<T>::store((T*)e.out0 + (size_t)m * N + n, fmaxf(acc, 0.f)); break;
    case EPI_RESID: ((float*)e.out0)[(size_t)m * N + n] = acc + e.resid[(size_t)m * N + n]; break;
    default: break;
  }
}

// Second stage of the arg max for one row by one wave; partials are loaded eight at a time.
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
      pvv[u] = t < n_strips ? gload(pv + t) : -INFINITY;
      pii[u] = t < n_strips ? gload(pi + t) : 0x7fffffff;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) argmax_merge(v, idx, pvv[u], pii[u]);
  }
  argmax_wave(v, idx);
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
  const size_t scalar_path = 2 * (size_t)nk_cap * row_dwords * 4 + 64 * (size_t)dh * 4 + (size_t)waves * nk_cap * 4;
  // matrix-core path: transposed values [dh][keys + 16] and one 16-row probability tile per wave
  // (row stride = 32 bytes past a multiple of 64: the 16-byte fragment reads meet no bank twice)
  const size_t ldv = (size_t)((nk_cap + 31) & ~31) + 16;
  const size_t mfma_path = ((size_t)dh + 16 * (size_t)waves) * ldv * 2;
  return scalar_path > mfma_path ? scalar_path : mfma_path;
}

// Maximum / sum over each row of 16 lanes (every lane of the row gets it); lane moves as in
// wave_sum, so the pairing depends on the lane's position in the row only.
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_move<0xB1>(v));
  v = fmaxf(v, dpp_move<0x4E>(v));
  v = fmaxf(v, dpp_move<0x141>(v));
  v = fmaxf(v, dpp_move<0x140>(v));
  return v;
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_move<0xB1>(v);
  v += dpp_move<0x4E>(v);
  v += dpp_move<0x141>(v);
  v += dpp_move<0x140>(v);
  return v;
}

// Attention of one (sequence, head) on the matrix cores, bf16 storage, head width a multiple of
// 32; the keys are walked NT tiles of 16 at a time.  The workgroup stages the head's values transposed in LDS (keys past
// the last needed one as zeros); then each wave takes 16 query rows at a time:
//   scores   S = Q K^T by MFMA, Q and K fragments straight from memory (k = head channel, 32 at
//            a time, ascending); times `scale`; keys a row must not see become -inf
//   softmax  exact row maximum; p = exp(s - max) (hardware 2^x of (s - max) log2 e); the denominator sums the unrounded p: each of
//            the 16 lanes of a row adds its keys (key % 16 = lane) in ascending order, then the
//            lanes combine by row16_sum; numerators are rounded to bf16 and go through LDS to
//            become the left operand of
//   output   O = P V by MFMA (k = key, 32 at a time, ascending), divided by the denominator.
// Every step treats a query row independently of the other rows of its tile and of how many
// tiles or keys the call covers (keys a row does not see contribute exact zeros), so a row's
// result does not depend on the shape of the block it is verified in.
template <int DH, int NT>
__device__ __forceinline__ void attn_tiles_mfma(const bf16_t* __restrict__ q, const bf16_t* __restrict__ Kb, bf16_t* __restrict__ out,
                                const SeqDesc sd, int row_begin, int row_end, int h, int d, float scale,
                                const bf16_t* Vt, bf16_t* Pw, int ldv, int nk_all,
                                const uint4 (&qf_pre)[DH / 32], const uint4 (&kf_pre)[4][DH / 32],
                                const float* Sbuf, int lds_s) {
  constexpr int KS = DH / 32, CT = DH / 16;
  const int waves = blockDim.x >> 6, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 15, kq = lane >> 4;
  const int n_tiles = (row_end - row_begin + 15) >> 4;
  // pre_c: the wave's first tile, whose query fragments and first four key tiles were requested
  // before the values were staged (attn_preload)
  auto tile = [&](auto pre_c, int rt) {
    constexpr bool PRE = decltype(pre_c)::value;
    const int row0 = row_begin + rt * 16;
    const int tile_end = min(row0 + 16, row_end);
    const int nk_tile = sd.causal ? sd.nk_base + tile_end : sd.nk_base;   // keys the tile's last row sees
    const int nt = (nk_tile + 15) >> 4, nb = (nk_tile + 31) >> 5;
    const int nch = (nt + NT - 1) / NT;   // the key tiles are walked NT at a time
    uint4 qf[KS];
    if constexpr (PRE) {
#pragma unroll
      for (int s = 0; s < KS; ++s) qf[s] = qf_pre[s];
    } else {
      const bf16_t* qp = q + (size_t)(sd.q_row0 + min(row0 + r, row_end - 1)) * d + h * DH + kq * 8;
#pragma unroll
      for (int s = 0; s < KS; ++s) qf[s] = ldg16(qp + 32 * s);
    }
    // this lane: rows row0 + 4*kq + i, key 16*(tile) + r
    int nkr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) nkr[i] = sd.causal ? sd.nk_base + row0 + 4 * kq + i + 1 : sd.nk_base;
    // scores of key tiles ch*NT .. ch*NT + NT - 1, scaled, -inf where the row must not see the key
    auto scores = [&](int ch, f32x4 (&S)[NT]) {
      // Loads are unconditional inside a group of four key tiles (indices clamped to the last tile
      // that exists; what lies past it is masked below): a load under its own branch would be
      // waited for on its own.
      if (Sbuf) {
        // the raw products were left in LDS by all waves together (attn_coop_scores)
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          const int jc = min(ch * NT + j, nt - 1);
#pragma unroll
          for (int i = 0; i < 4; ++i) S[j][i] = Sbuf[(4 * kq + i) * lds_s + 16 * jc + r];
        }
      } else {
        uint4 kf[NT][KS];
#pragma unroll
        for (int j0 = 0; j0 < NT; j0 += 4) {
          if (ch * NT + j0 < nt) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
              const int j = j0 + jj, jc = min(ch * NT + j, nt - 1);
              if (PRE && j0 == 0 && ch == 0 && jc == j) {
#pragma unroll
                for (int s = 0; s < KS; ++s) kf[j][s] = kf_pre[jj][s];
              } else {
                const bf16_t* kp = Kb + (size_t)(sd.kv_row0 + min(16 * jc + r, nk_all - 1)) * d + h * DH + kq * 8;
#pragma unroll
                for (int s = 0; s < KS; ++s) kf[j][s] = ldg16(kp + 32 * s);
              }
            }
          }
        }
#pragma unroll
        for (int j0 = 0; j0 < NT; j0 += 4) {
          if (ch * NT + j0 < nt) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
              const int j = j0 + jj;
              S[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
              for (int s = 0; s < KS; ++s)
                S[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qf[s]), __builtin_bit_cast(bf16x8, kf[j][s]), S[j], 0, 0, 0);
            }
          } else {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) S[j0 + jj] = f32x4{0.f, 0.f, 0.f, 0.f};
          }
        }
      }
      // (a key tile that does not exist needs no test of its own: its keys' indices are at least
      // 16 nt, which no row of the tile sees)
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int key = 16 * (ch * NT + j) + r;
#pragma unroll
        for (int i = 0; i < 4; ++i) S[j][i] = key < nkr[i] ? S[j][i] * scale : -INFINITY;
      }
    };
    f32x4 S[NT];
    float mx[4], sum[4], l[4];
    // exact row maximum: one pass over all key tiles (more than NT of them: the scores are
    // computed again, tile group by tile group, in the pass below)
    {
      float m[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
      for (int ch = 0; ch < max(nch, 1); ++ch) {
        scores(ch, S);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < NT; ++j) m[i] = fmaxf(m[i], S[j][i]);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) { mx[i] = row16_max(m[i]); sum[i] = 0.f; }
    }
    f32x4 O[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) O[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int ch = 0; ch < max(nch, 1); ++ch) {
      if (nch > 1) scores(ch, S);
      const int tiles_here = 2 * nb - ch * NT;   // tiles of this group the output product reads (an odd count is padded with zeros)
      // Slot i of a lane holds row row0 + 4*kq + i.  All four slots are computed, tile by tile, as
      // independent chains (a slot whose rows do not exist computes on the clamped query rows, lands
      // in the wave's own probability tile and is never stored; skipping such slots under a branch
      // each made the four chains run one after the other: 0.3 us per slot).
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        if (j < tiles_here) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            // e^x as 2^(x log2 e) on the hardware exponential; 2^(-inf) = 0 for the keys the row does not see
            const float pv = __builtin_amdgcn_exp2f((S[j][i] - mx[i]) * 1.44269504088896340736f);
            sum[i] += pv;
            Pw[(4 * kq + i) * ldv + r + 16 * j] = f2bf(pv);
          }
        }
      }
      __builtin_amdgcn_wave_barrier();
      const int kb_end = min(nb, (ch + 1) * (NT / 2));
      for (int kb = ch * (NT / 2); kb < kb_end; ++kb) {
        const uint4 pa = *(const uint4*)(Pw + r * ldv + 32 * (kb - ch * (NT / 2)) + 8 * kq);
        uint4 vb[CT];
#pragma unroll
        for (int c = 0; c < CT; ++c) vb[c] = *(const uint4*)(Vt + (16 * c + r) * ldv + 32 * kb + 8 * kq);
#pragma unroll
        for (int c = 0; c < CT; ++c)
          O[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pa), __builtin_bit_cast(bf16x8, vb[c]), O[c], 0, 0, 0);
      }
      __builtin_amdgcn_wave_barrier();   // the probability tile is reused by the next group and the wave's next rows
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) l[i] = row16_sum(sum[i]);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = row0 + 4 * kq + i;
      if (row < row_end) {
        bf16_t* op = out + (size_t)(sd.q_row0 + row) * d + h * DH + r;
#pragma unroll
        for (int c = 0; c < CT; ++c) Store<bf16_t>::store(op + 16 * c, O[c][i] / l[i]);
      }
    }
  };
  if (wave < n_tiles) tile(std::true_type{}, wave);
  for (int rt = wave + waves; rt < n_tiles; rt += waves) tile(std::false_type{}, rt);
}
// Query fragments and the first four key tiles of the wave's first 16-row tile (what
// attn_tiles_mfma takes as qf_pre / kf_pre): same addresses, same clamping.
template <int DH>
__device__ __forceinline__ void attn_preload(const bf16_t* __restrict__ q, const bf16_t* __restrict__ Kb, const SeqDesc sd,
                                             int row_begin, int row_end, int h, int d, int nk_all,
                                             uint4 (&qf)[DH / 32], uint4 (&kf)[4][DH / 32]) {
  constexpr int KS = DH / 32;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 15, kq = lane >> 4;
  const int n_tiles = (row_end - row_begin + 15) >> 4;
  if (wave >= n_tiles) return;
  const int row0 = row_begin + wave * 16;
  const int tile_end = min(row0 + 16, row_end);
  const int nk_tile = sd.causal ? sd.nk_base + tile_end : sd.nk_base;
  const int nt = (nk_tile + 15) >> 4;
  const bf16_t* qp = q + (size_t)(sd.q_row0 + min(row0 + r, row_end - 1)) * d + h * DH + kq * 8;
#pragma unroll
  for (int s = 0; s < KS; ++s) qf[s] = ldg16(qp + 32 * s);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (j < nt) {
      const bf16_t* kp = Kb + (size_t)(sd.kv_row0 + min(16 * j + r, nk_all - 1)) * d + h * DH + kq * 8;
#pragma unroll
      for (int s = 0; s < KS; ++s) kf[j][s] = ldg16(kp + 32 * s);
    }
  }
}
// The key half of attn_preload alone (the queries come from somewhere else).
template <int DH>
__device__ __forceinline__ void attn_preload_k(const bf16_t* __restrict__ Kb, const SeqDesc sd, int row_begin, int row_end,
                                               int h, int d, int nk_all, uint4 (&kf)[4][DH / 32]) {
  constexpr int KS = DH / 32;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 15, kq = lane >> 4;
  const int n_tiles = (row_end - row_begin + 15) >> 4;
  if (wave >= n_tiles) return;
  const int tile_end = min(row_begin + wave * 16 + 16, row_end);
  const int nk_tile = sd.causal ? sd.nk_base + tile_end : sd.nk_base;
  const int nt = (nk_tile + 15) >> 4;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (j < nt) {
      const bf16_t* kp = Kb + (size_t)(sd.kv_row0 + min(16 * j + r, nk_all - 1)) * d + h * DH + kq * 8;
#pragma unroll
      for (int s = 0; s < KS; ++s) kf[j][s] = ldg16(kp + 32 * s);
    }
  }
}
template <int DH>
__device__ __forceinline__ void attn_coop_scores_q(const uint4 (&qf)[DH / 32], const bf16_t* __restrict__ Kb, const SeqDesc sd,
                                                   int h, int d, int nk_all, int nt, float* Sbuf, int lds_s);
// One 16-row tile, many keys: the score products Q K^T are independent per key tile, so all waves
// of the workgroup compute them together (wave w: key tiles w, w + waves, ..; one fetch latency
// instead of one per group of tiles on a single wave) and leave the raw fp32 products in LDS,
// [16 rows][lds_s]; the tile's wave then goes on exactly as if it had computed them itself.
template <int DH>
__device__ __forceinline__ void attn_coop_scores(const bf16_t* __restrict__ q, const bf16_t* __restrict__ Kb, const SeqDesc sd,
                                                 int row_begin, int row_end, int h, int d, int nk_all, int nt,
                                                 float* Sbuf, int lds_s) {
  constexpr int KS = DH / 32;
  const int lane = threadIdx.x & 63;
  const int r = lane & 15, kq = lane >> 4;
  uint4 qf[KS];
  {
    const bf16_t* qp = q + (size_t)(sd.q_row0 + min(row_begin + r, row_end - 1)) * d + h * DH + kq * 8;
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = ldg16(qp + 32 * s);
  }
  attn_coop_scores_q<DH>(qf, Kb, sd, h, d, nk_all, nt, Sbuf, lds_s);
}
// (the same with the tile's query fragments given)
template <int DH>
__device__ __forceinline__ void attn_coop_scores_q(const uint4 (&qf)[DH / 32], const bf16_t* __restrict__ Kb, const SeqDesc sd,
                                                   int h, int d, int nk_all, int nt, float* Sbuf, int lds_s) {
  constexpr int KS = DH / 32, TB = 8;   // key tiles per batch of loads
  const int waves = blockDim.x >> 6, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 15, kq = lane >> 4;
  for (int b0 = wave; b0 < nt; b0 += waves * TB) {
    uint4 kf[TB][KS];
#pragma unroll
    for (int jj = 0; jj < TB; ++jj) {
      // unconditional (clamped to the last tile): a load under its own branch is waited for on its own
      const int jc = min(b0 + jj * waves, nt - 1);
      const bf16_t* kp = Kb + (size_t)(sd.kv_row0 + min(16 * jc + r, nk_all - 1)) * d + h * DH + kq * 8;
#pragma unroll
      for (int s = 0; s < KS; ++s) kf[jj][s] = ldg16(kp + 32 * s);
    }
#pragma unroll
    for (int jj = 0; jj < TB; ++jj) {
      const int jg = b0 + jj * waves;
      if (jg < nt) {
        f32x4 S = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s)
          S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qf[s]), __builtin_bit_cast(bf16x8, kf[jj][s]), S, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) Sbuf[(4 * kq + i) * lds_s + 16 * jg + r] = S[i];
      }
    }
  }
}
// Values of one (sequence, head) transposed into LDS: Vt[c][t] = V[t][c], keys nk_all .. nkp - 1 as zeros.
template <int DH>
__device__ __forceinline__ void attn_stage_values(const bf16_t* __restrict__ Vb, const SeqDesc sd, int h, int d, bf16_t* Vt,
                                                  int ldv, int nkp, int nk_all) {
  // Values transposed into LDS.  Many keys: 8 keys x 8 channels per step and thread: eight 16-byte loads
  // (one key row piece each), an 8 x 8 transpose of 16-bit values in registers (byte permutes),
  // eight 16-byte LDS stores (one channel row piece each).  Keys past the last needed one: zeros.
  constexpr int G = DH / 8;   // 16-byte pieces per key row
  const bf16_t* vg = Vb + (size_t)sd.kv_row0 * d + h * DH;
  // few keys: one 16-byte piece per thread and step, eight 2-byte LDS stores (more threads in
  // flight, which is what counts there); many keys: the transposing path below
  if (nkp <= 128)
  for (int i = threadIdx.x; i < nkp * G; i += blockDim.x) {
    const int g = i / nkp, t = i - g * nkp;
    uint4 v = uint4{0u, 0u, 0u, 0u};
    if (t < nk_all) v = ldg16(vg + (size_t)t * d + g * 8);
    bf16_t* dst = Vt + (size_t)(g * 8) * ldv + t;
    dst[0] = (bf16_t)(v.x & 0xffffu); dst[ldv] = (bf16_t)(v.x >> 16);
    dst[2 * ldv] = (bf16_t)(v.y & 0xffffu); dst[3 * ldv] = (bf16_t)(v.y >> 16);
    dst[4 * ldv] = (bf16_t)(v.z & 0xffffu); dst[5 * ldv] = (bf16_t)(v.z >> 16);
    dst[6 * ldv] = (bf16_t)(v.w & 0xffffu); dst[7 * ldv] = (bf16_t)(v.w >> 16);
  }
  const int n_items = nkp <= 128 ? 0 : (nkp >> 3) * G;
  for (int it = threadIdx.x; it < n_items; it += blockDim.x) {
    const int g = it % G, t0 = (it / G) << 3;
    unsigned in[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      uint4 v = uint4{0u, 0u, 0u, 0u};
      if (t0 + i < nk_all) v = ldg16(vg + (size_t)(t0 + i) * d + g * 8);
      in[i][0] = v.x; in[i][1] = v.y; in[i][2] = v.z; in[i][3] = v.w;
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      // channel c of keys t0 .. t0+7: the low (c even) or high (c odd) half of dword c/2 of every key
      unsigned o[4];
#pragma unroll
      for (int pr = 0; pr < 4; ++pr) {
        const unsigned lo = in[2 * pr][c >> 1], hi = in[2 * pr + 1][c >> 1];
        o[pr] = (c & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
      }
      *(uint4*)(Vt + (size_t)(g * 8 + c) * ldv + t0) = uint4{o[0], o[1], o[2], o[3]};
    }
  }
}
template <int DH>
__device__ __forceinline__ void attn_block_mfma(const bf16_t* __restrict__ q, const bf16_t* __restrict__ Kb,
                                const bf16_t* __restrict__ Vb, bf16_t* __restrict__ out, const SeqDesc sd,
                                int row_begin, int row_end, int h, int d, float scale, unsigned* lds, int nk_all) {
  const int wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
  const int nkp = (nk_all + 31) & ~31, ldv = nkp + 16;
  bf16_t* Vt = (bf16_t*)lds;                      // [DH][ldv]: Vt[c][t] = V[t][c]
  bf16_t* Pw = Vt + DH * ldv + wave * 16 * ldv;   // this wave's probability tile [16][ldv]
  // the first tile's operands of the score product are requested before the values are staged:
  // the two fetch latencies overlap
  uint4 qf_pre[DH / 32], kf_pre[4][DH / 32];
  attn_preload<DH>(q, Kb, sd, row_begin, row_end, h, d, nk_all, qf_pre, kf_pre);
  // a single row tile against more than 128 keys: the waves share the score products; the buffer
  // lies over the probability tiles of the waves that have no rows
  const int nt_all = (nk_all + 15) >> 4;
  const bool coop = row_end - row_begin <= 16 && nt_all > 8 && waves >= 3;
  float* Sbuf = coop ? (float*)(Vt + DH * ldv + 16 * ldv) : nullptr;
  if (coop) attn_coop_scores<DH>(q, Kb, sd, row_begin, row_end, h, d, nk_all, nt_all, Sbuf, nkp);
  attn_stage_values<DH>(Vb, sd, h, d, Vt, ldv, nkp, nk_all);
  __syncthreads();
  if (nkp <= 64) attn_tiles_mfma<DH, 4>(q, Kb, out, sd, row_begin, row_end, h, d, scale, Vt, Pw, ldv, nk_all, qf_pre, kf_pre, Sbuf, nkp);
  else if (nkp <= 128) attn_tiles_mfma<DH, 8>(q, Kb, out, sd, row_begin, row_end, h, d, scale, Vt, Pw, ldv, nk_all, qf_pre, kf_pre, Sbuf, nkp);
  else attn_tiles_mfma<DH, 16>(q, Kb, out, sd, row_begin, row_end, h, d, scale, Vt, Pw, ldv, nk_all, qf_pre, kf_pre, Sbuf, nkp);
  __syncthreads();   // LDS is free for the next call
}

template <typename T, int DH>
__device__ __forceinline__ void attn_block(const T* __restrict__ q, const T* __restrict__ Kb, const T* __restrict__ Vb,
                           T* __restrict__ out, const SeqDesc sd, int row_begin, int row_end, int h, int d,
                           float scale, unsigned* lds, int nk_cap) {
  if constexpr (sizeof(T) == 2 && DH % 32 == 0) {
    const int nk_need = sd.causal ? sd.nk_base + row_end : sd.nk_base;
    attn_block_mfma<DH>(q, Kb, Vb, out, sd, row_begin, row_end, h, d, scale, lds, nk_need);
    return;
  }
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
          kv[u] = gload(kg + t * gs + w);
          vv[u] = gload(vg + t * gs + w);
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
          qv[u] = Store<T>::load(q + (size_t)(sd.q_row0 + row_begin + rr) * d + h * DH + c);
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
    // Operands are read in batches (the whole query row once, a key row at a time, eight
    // value rows at a time) before the arithmetic that uses them, so that a wave that has its
    // SIMD to itself waits for LDS once per batch; the arithmetic order is the one stated above.
    float qv[DH];
    {
      const float* qs = Qs + (i - row_begin) * DH;
#pragma unroll
      for (int c = 0; c < DH; ++c) qv[c] = qs[c];
    }
    float mx = -INFINITY;
    for (int t = lane; t < nk; t += 64) {
      const unsigned* kr = Ks + t * RS;
      unsigned kw[RD];
#pragma unroll
      for (int w = 0; w < RD; ++w) kw[w] = kr[w];
      float a = 0.f;
      if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int w = 0; w < RD; ++w) {
          float lo, hi;
          LdsRow<bf16_t>::unpack(kw[w], lo, hi);
          a = fmaf(qv[2 * w], lo, a);
          a = fmaf(qv[2 * w + 1], hi, a);
        }
      } else {
#pragma unroll
        for (int w = 0; w < RD; ++w) a = fmaf(qv[w], __uint_as_float(kw[w]), a);
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
      for (int t0 = 0; t0 < nk; t0 += 8) {
        float pt[8], vt[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int t = t0 + j < nk ? t0 + j : nk - 1;    // (past the end: re-read the last key, not used)
          pt[j] = sc[t];
          if constexpr (sizeof(T) == 2) vt[j] = bf2f(((const bf16_t*)Vs)[(size_t)t * RS * 2 + c]);
          else vt[j] = ((const float*)Vs)[(size_t)t * RS + c];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (t0 + j < nk) a = fmaf(pt[j], vt[j], a);
      }
      Store<T>::store(out + (size_t)m * d + h * DH + c, a / l);
    }
    __builtin_amdgcn_wave_barrier();
  }
  __syncthreads();
}

}  // namespace ad

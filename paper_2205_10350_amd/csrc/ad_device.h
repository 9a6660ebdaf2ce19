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

// (the key-split paths, attn_split_keys / attn_split_tiles: per wave a [64][kSplitLd] value tile and a [16][kSplitLd]
// probability tile)
constexpr int kSplitLd = 128 + 16;                                   // row stride (elements): 32 bytes past a multiple of 64
constexpr int kSplitWaveElems = (64 + 16) * kSplitLd;                // bf16 elements of a wave's two tiles
constexpr int kSplitXchBytes = 4 * 16 * 4 + 4 * 64 * 16 + 4 * 4 * 64 * 16;   // attn_split_keys: maxima, denominators, partial outputs
constexpr int kLongKeys = 256;   // key capacity from which the generic attention launch is the kernel that can split the keys
constexpr int kSplitTilesBytes = 4 * kSplitWaveElems * 2 + 4 * 64 * 4;      // attn_split_tiles: the waves' tiles and the row maxima
__host__ __device__ inline size_t attn_lds_bytes(int nk_cap, int dh, int esz, int waves) {
  const size_t row_dwords = (size_t)dh * esz / 4 + 1;
  const size_t scalar_path = 2 * (size_t)nk_cap * row_dwords * 4 + 64 * (size_t)dh * 4 + (size_t)waves * nk_cap * 4;
  // matrix-core path: transposed values [dh][keys + 16] and one 16-row probability tile per wave
  // (row stride = 32 bytes past a multiple of 64: the 16-byte fragment reads meet no bank twice)
  const size_t ldv = (size_t)((nk_cap + 31) & ~31) + 16;
  size_t mfma_path = ((size_t)dh + 16 * (size_t)waves) * ldv * 2;
  if (dh == 64 && esz == 2 && nk_cap >= kLongKeys && mfma_path < (size_t)kSplitTilesBytes) mfma_path = kSplitTilesBytes;
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
template <int DH, int NT, bool LONGK = false>
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
    float mx[4], l[4];
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
      for (int i = 0; i < 4; ++i) mx[i] = row16_max(m[i]);
    }
    // LONGK (the launches of configurations whose key capacity is kLongKeys or more; head width up to 64), more than
    // 128 keys (NT = 16): the keys are taken in super-blocks of 128, super-block sb adds into accumulator sb % 4 (output
    // sums and denominators alike, ascending inside an accumulator), and the four are combined as (a0 + a1) + (a2 + a3)
    // at the end.  The order depends on the key index alone, so the kernels that give the four accumulators to four
    // waves (attn_split_keys, attn_split_tiles) produce the same bits; with at most 128 keys there is one chain.
    // Otherwise one chain for any key count: no kernel of such a configuration splits the keys, and the short-range
    // kernels, the batch-1 path, stay as small as they were (the four accumulator sets alone cost their launches
    // 0.3 us each, forward at 25 rows 186.6 -> 188.4 us, although that code never ran).
    constexpr int NA = LONGK && NT == 16 && DH <= 64 ? 4 : 1;
    f32x4 O[NA][CT];
    float psum[NA][4];
#pragma unroll
    for (int a = 0; a < NA; ++a) {
#pragma unroll
      for (int c = 0; c < CT; ++c) O[a][c] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < 4; ++i) psum[a][i] = 0.f;
    }
    // group ch of NT key tiles; PAR = ch % 2 at compile time (a group of 16 tiles is the two super-blocks 2 ch, 2 ch + 1)
    auto group = [&](auto par_c, int ch) {
      constexpr int PAR = decltype(par_c)::value;
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
            psum[NA == 1 ? 0 : (2 * PAR + (j >> 3)) & 3][i] += pv;
            Pw[(4 * kq + i) * ldv + r + 16 * j] = f2bf(pv);
          }
        }
      }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int half = 0; half < (NA == 1 ? 1 : 2); ++half) {
        const int kb_begin = ch * (NT / 2) + (NA == 1 ? 0 : 4 * half);
        const int kb_end = min(nb, NA == 1 ? (ch + 1) * (NT / 2) : kb_begin + 4);
        f32x4 (&Oa)[CT] = O[NA == 1 ? 0 : (2 * PAR + half) & 3];
        for (int kb = kb_begin; kb < kb_end; ++kb) {
          const uint4 pa = *(const uint4*)(Pw + r * ldv + 32 * (kb - ch * (NT / 2)) + 8 * kq);
          uint4 vb[CT];
#pragma unroll
          for (int c = 0; c < CT; ++c) vb[c] = *(const uint4*)(Vt + (16 * c + r) * ldv + 32 * kb + 8 * kq);
#pragma unroll
          for (int c = 0; c < CT; ++c)
            Oa[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pa), __builtin_bit_cast(bf16x8, vb[c]), Oa[c], 0, 0, 0);
        }
      }
      __builtin_amdgcn_wave_barrier();   // the probability tile is reused by the next group and the wave's next rows
    };
    if constexpr (NA == 1) {
      for (int ch = 0; ch < max(nch, 1); ++ch) group(std::integral_constant<int, 0>{}, ch);
    } else {
      for (int ch = 0; ch < max(nch, 1); ch += 2) {
        group(std::integral_constant<int, 0>{}, ch);
        if (ch + 1 < nch) group(std::integral_constant<int, 1>{}, ch + 1);
      }
    }
    if constexpr (NA == 4) {
#pragma unroll
      for (int c = 0; c < CT; ++c) O[0][c] = (O[0][c] + O[1][c]) + (O[2][c] + O[3][c]);
#pragma unroll
      for (int i = 0; i < 4; ++i) psum[0][i] = (psum[0][i] + psum[1][i]) + (psum[2][i] + psum[3][i]);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) l[i] = row16_sum(psum[0][i]);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = row0 + 4 * kq + i;
      if (row < row_end) {
        bf16_t* op = out + (size_t)(sd.q_row0 + row) * d + h * DH + r;
#pragma unroll
        for (int c = 0; c < CT; ++c) Store<bf16_t>::store(op + 16 * c, O[0][c][i] / l[i]);
      }
    }
  };
  // (Every caller hands a chunk of at most 64 rows to a workgroup of four waves: a wave has at most one tile, the one
  // whose operands were requested ahead.  A loop over further tiles, with its own copy of the tile body, was never
  // entered, and the attention kernels ran slower for carrying it.)
  if (wave < n_tiles) tile(std::true_type{}, wave);
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
// One 16-row tile against many keys (head width 64, four waves): wave w owns the key super-blocks (128 keys each)
// w, w + 4, ... from the scores to the output product, i.e. accumulator w of the order attn_tiles_mfma<64, 16>
// states, so the bits are the same whichever of the two serves a row.  Per wave: scores of its keys (key fragments
// straight from memory), row maxima exchanged through LDS (exact, so their order cannot matter), exponentials,
// probabilities into the wave's own LDS tile, its 128 values transposed into its own LDS tile (no other wave
// touches either: no workgroup barrier), output product; then the four partial outputs and per-lane denominators
// go through LDS and wave c combines and stores channel block c.
// LDS per wave: values [64][kSplitLd] then probabilities [16][kSplitLd]; exchange area: see attn_split_lds_bytes.
__host__ __device__ inline size_t attn_split_lds_bytes() { return 4 * (size_t)kSplitWaveElems * 2 + kSplitXchBytes; }
// the key fragments of the eight tiles of super-block sb (indices clamped to the last key)
__device__ __forceinline__ void split_request_keys(const bf16_t* __restrict__ Kb, const SeqDesc sd, int h, int d, int nk_all,
                                                   int sb, uint4 (&kf)[8][2]) {
  const int lane = threadIdx.x & 63, r = lane & 15, kq = lane >> 4;
  const bf16_t* kbase = Kb + (size_t)sd.kv_row0 * d + h * 64 + kq * 8;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const bf16_t* kp = kbase + (size_t)min(128 * sb + 16 * j + r, nk_all - 1) * d;
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) kf[j][s2] = ldg16(kp + 32 * s2);
  }
}
// the raw values of super-block sb: two 8-key x 8-channel items per lane (transposed later)
__device__ __forceinline__ void split_request_values(const bf16_t* __restrict__ Vb, const SeqDesc sd, int h, int d, int nk_all,
                                                     int sb, uint4 (&vraw)[2][8]) {
  const int lane = threadIdx.x & 63;
  const bf16_t* vbase = Vb + (size_t)sd.kv_row0 * d + h * 64;
#pragma unroll
  for (int b2 = 0; b2 < 2; ++b2) {
    const int it = lane + 64 * b2, g = it & 7, t0 = 128 * sb + ((it >> 3) << 3);
#pragma unroll
    for (int i = 0; i < 8; ++i) vraw[b2][i] = ldg16(vbase + (size_t)min(t0 + i, nk_all - 1) * d + g * 8);
  }
}
// the raw values of super-block sb into the wave's tile Vw[c][t] = V[128 sb + t][c]: 8 x 8 transposes in registers,
// 16-byte stores; keys past the last one as zeros
__device__ __forceinline__ void split_stage_values(const uint4 (&vraw)[2][8], bf16_t* Vw, int sb, int nk_all) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int b2 = 0; b2 < 2; ++b2) {
    const int it = lane + 64 * b2, g = it & 7, tl = (it >> 3) << 3, t0 = 128 * sb + tl;
    unsigned in[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bool there = t0 + i < nk_all;
      in[i][0] = there ? vraw[b2][i].x : 0u; in[i][1] = there ? vraw[b2][i].y : 0u;
      in[i][2] = there ? vraw[b2][i].z : 0u; in[i][3] = there ? vraw[b2][i].w : 0u;
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      unsigned o[4];
#pragma unroll
      for (int pr = 0; pr < 4; ++pr) {
        const unsigned lo = in[2 * pr][c >> 1], hi = in[2 * pr + 1][c >> 1];
        o[pr] = (c & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
      }
      *(uint4*)(Vw + (size_t)(g * 8 + c) * kSplitLd + tl) = uint4{o[0], o[1], o[2], o[3]};
    }
  }
}
// kf0, vraw: the key fragments and raw values of the wave's first super-block (sb = wave), requested by the caller
__device__ __forceinline__ void attn_split_keys(const uint4 (&qf)[2], const uint4 (&kf0)[8][2], uint4 (&vraw)[2][8],
                                                const bf16_t* __restrict__ Kb, const bf16_t* __restrict__ Vb,
                                                bf16_t* __restrict__ out, const SeqDesc sd, int row_begin, int row_end, int h,
                                                int d, float scale, int nk_all, bf16_t* lds_waves, float* xch) {
  constexpr int DH = 64, KS = 2, CT = 4, LD = kSplitLd;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 15, kq = lane >> 4;
  bf16_t* Vw = lds_waves + wave * kSplitWaveElems;   // [64][LD]: Vw[c][t] = V[128 sb + t][c]
  bf16_t* Pw = Vw + 64 * LD;                          // [16][LD]
  float* xmax = xch;                                  // [4 waves][16 rows]
  float* xsum = xch + 64;                             // [4 waves][64 lanes][4]
  f32x4* xout = (f32x4*)(xch + 64 + 1024);            // [4 waves][4 channel blocks][64 lanes]
  const int n_sb = (nk_all + 127) >> 7;
  int nkr[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) nkr[i] = sd.causal ? sd.nk_base + row_begin + 4 * kq + i + 1 : sd.nk_base;
  // the eight score tiles of super-block sb from its key fragments: S[j][i] = row 4 kq + i, key 128 sb + 16 j + r
  auto scores = [&](int sb, const uint4 (&kf)[8][2], f32x4 (&S)[8]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      S[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s2 = 0; s2 < KS; ++s2)
        S[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qf[s2]), __builtin_bit_cast(bf16x8, kf[j][s2]), S[j], 0, 0, 0);
      const int key = 128 * sb + 16 * j + r;
#pragma unroll
      for (int i = 0; i < 4; ++i) S[j][i] = key < nkr[i] ? S[j][i] * scale : -INFINITY;
    }
  };
  f32x4 S[8];
  const bool mine = wave < n_sb;
  const bool single = wave + 4 >= n_sb;   // at most one super-block: its scores stay in registers
  float m[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
  if (mine) {
    scores(wave, kf0, S);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) m[i] = fmaxf(m[i], S[j][i]);
    for (int sb = wave + 4; sb < n_sb; sb += 4) {
      uint4 kf[8][2];
      f32x4 S2[8];
      split_request_keys(Kb, sd, h, d, nk_all, sb, kf);
      scores(sb, kf, S2);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) m[i] = fmaxf(m[i], S2[j][i]);
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) m[i] = row16_max(m[i]);
  if (r == 0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) xmax[wave * 16 + 4 * kq + i] = m[i];
  }
  __syncthreads();
  float mx[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    mx[i] = fmaxf(fmaxf(xmax[4 * kq + i], xmax[16 + 4 * kq + i]), fmaxf(xmax[32 + 4 * kq + i], xmax[48 + 4 * kq + i]));
  f32x4 O[CT];
  float psum[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < CT; ++c) O[c] = f32x4{0.f, 0.f, 0.f, 0.f};
  if (mine) {
    for (int sb = wave; sb < n_sb; sb += 4) {
      if (sb != wave) {
        uint4 kf[8][2];
        split_request_keys(Kb, sd, h, d, nk_all, sb, kf);
        split_request_values(Vb, sd, h, d, nk_all, sb, vraw);
        scores(sb, kf, S);
      } else if (!single) {
        scores(sb, kf0, S);
      }
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float pv = __builtin_amdgcn_exp2f((S[j][i] - mx[i]) * 1.44269504088896340736f);
          psum[i] += pv;
          Pw[(4 * kq + i) * LD + r + 16 * j] = f2bf(pv);
        }
      split_stage_values(vraw, Vw, sb, nk_all);
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int kb = 0; kb < 4; ++kb) {
        const uint4 pa = *(const uint4*)(Pw + r * LD + 32 * kb + 8 * kq);
        uint4 vb[CT];
#pragma unroll
        for (int c = 0; c < CT; ++c) vb[c] = *(const uint4*)(Vw + (16 * c + r) * LD + 32 * kb + 8 * kq);
#pragma unroll
        for (int c = 0; c < CT; ++c)
          O[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pa), __builtin_bit_cast(bf16x8, vb[c]), O[c], 0, 0, 0);
      }
      __builtin_amdgcn_wave_barrier();   // the tiles are reused by the wave's next super-block
    }
  }
#pragma unroll
  for (int c = 0; c < CT; ++c) xout[(wave * 4 + c) * 64 + lane] = O[c];
  *(f32x4*)(xsum + (wave * 64 + lane) * 4) = f32x4{psum[0], psum[1], psum[2], psum[3]};
  __syncthreads();
  // wave c: channel block c of the tile
  const f32x4 o = (xout[(0 * 4 + wave) * 64 + lane] + xout[(1 * 4 + wave) * 64 + lane]) +
                  (xout[(2 * 4 + wave) * 64 + lane] + xout[(3 * 4 + wave) * 64 + lane]);
  const f32x4 sm = (*(const f32x4*)(xsum + (0 * 64 + lane) * 4) + *(const f32x4*)(xsum + (1 * 64 + lane) * 4)) +
                   (*(const f32x4*)(xsum + (2 * 64 + lane) * 4) + *(const f32x4*)(xsum + (3 * 64 + lane) * 4));
  float l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) l[i] = row16_sum(sm[i]);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = row_begin + 4 * kq + i;
    if (row < row_end) Store<bf16_t>::store(out + (size_t)(sd.q_row0 + row) * d + h * DH + 16 * wave + r, o[i] / l[i]);
  }
}
// Up to four 16-row tiles (one per wave in the other kernels) against 129..512 keys, head width 64, four waves: the split
// of attn_split_keys for every row tile of the chunk.  Wave w owns super-block w: its key fragments are fetched once
// and multiply the queries of all tiles; the row maxima of all tiles cross LDS behind one barrier; then, tile by tile,
// exponentials, probabilities (the wave's own LDS tile), output product against the wave's own transposed values.
// Behind a second barrier the partial outputs and denominators go through LDS (over the tiles, which nobody reads any
// more) and wave c combines and stores channel block c of every tile.  Keys and values cross from memory once per
// workgroup instead of once (values) and twice (keys) per wave.  Same bits as attn_tiles_mfma<64, 16>.
__device__ __forceinline__ void attn_split_tiles(const bf16_t* __restrict__ q, const bf16_t* __restrict__ Kb,
                                                 const bf16_t* __restrict__ Vb, bf16_t* __restrict__ out, const SeqDesc sd,
                                                 int row_begin, int row_end, int h, int d, float scale, int nk_all,
                                                 bf16_t* lds) {
  constexpr int DH = 64, CT = 4, LD = kSplitLd;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 15, kq = lane >> 4;
  const int nt = (row_end - row_begin + 15) >> 4;     // 1..4 row tiles
  bf16_t* Vw = lds + wave * kSplitWaveElems;          // [64][LD]
  bf16_t* Pw = Vw + 64 * LD;                          // [16][LD]
  float* xmax = (float*)(lds + 4 * kSplitWaveElems);  // [4 waves][64 rows]
  f32x4* xout = (f32x4*)lds;                          // [(wave * 4 + tile) * 4 + channel block][64 lanes], over the tiles
  f32x4* xsum = xout + 4 * 4 * 4 * 64;                // [wave * 4 + tile][64 lanes]
  const int n_sb = (nk_all + 127) >> 7;
  const bool mine = wave < n_sb;
  uint4 kf[8][2];
  split_request_keys(Kb, sd, h, d, nk_all, wave, kf);
  uint4 qf[4][2];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int row = min(row_begin + 16 * min(t, nt - 1) + r, row_end - 1);
    const bf16_t* qp = q + (size_t)(sd.q_row0 + row) * d + h * DH + kq * 8;
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) qf[t][s2] = ldg16(qp + 32 * s2);
  }
  f32x4 S[4][8];
  float m[4][4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
#pragma unroll
    for (int i = 0; i < 4; ++i) m[t][i] = -INFINITY;
    if (mine && t < nt) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        S[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
          S[t][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qf[t][s2]), __builtin_bit_cast(bf16x8, kf[j][s2]), S[t][j], 0, 0, 0);
        const int key = 128 * wave + 16 * j + r;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int nkr = sd.causal ? sd.nk_base + row_begin + 16 * t + 4 * kq + i + 1 : sd.nk_base;
          S[t][j][i] = key < nkr ? S[t][j][i] * scale : -INFINITY;
          m[t][i] = fmaxf(m[t][i], S[t][j][i]);
        }
      }
    }
  }
  uint4 vraw[2][8];
  split_request_values(Vb, sd, h, d, nk_all, wave, vraw);
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) m[t][i] = row16_max(m[t][i]);
  if (r == 0) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) xmax[wave * 64 + 16 * t + 4 * kq + i] = m[t][i];
  }
  __syncthreads();
  f32x4 O[4][CT];
  f32x4 psum[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    psum[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < CT; ++c) O[t][c] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  if (mine) {
    split_stage_values(vraw, Vw, wave, nk_all);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if (t < nt) {
        float mx[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = 16 * t + 4 * kq + i;
          mx[i] = fmaxf(fmaxf(xmax[row], xmax[64 + row]), fmaxf(xmax[128 + row], xmax[192 + row]));
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float pv = __builtin_amdgcn_exp2f((S[t][j][i] - mx[i]) * 1.44269504088896340736f);
            psum[t][i] += pv;
            Pw[(4 * kq + i) * LD + r + 16 * j] = f2bf(pv);
          }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
          const uint4 pa = *(const uint4*)(Pw + r * LD + 32 * kb + 8 * kq);
          uint4 vb[CT];
#pragma unroll
          for (int c = 0; c < CT; ++c) vb[c] = *(const uint4*)(Vw + (16 * c + r) * LD + 32 * kb + 8 * kq);
#pragma unroll
          for (int c = 0; c < CT; ++c)
            O[t][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pa), __builtin_bit_cast(bf16x8, vb[c]), O[t][c], 0, 0, 0);
        }
        __builtin_amdgcn_wave_barrier();   // the probability tile is reused by the next row tile
      }
    }
  }
  __syncthreads();   // every wave is done with its tiles: the exchange area lies over them
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    if (t < nt) {
#pragma unroll
      for (int c = 0; c < CT; ++c) xout[((wave * 4 + t) * 4 + c) * 64 + lane] = O[t][c];
      xsum[(wave * 4 + t) * 64 + lane] = psum[t];
    }
  }
  __syncthreads();
  // wave c: channel block c of every tile
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    if (t < nt) {
      const f32x4 o = (xout[((0 * 4 + t) * 4 + wave) * 64 + lane] + xout[((1 * 4 + t) * 4 + wave) * 64 + lane]) +
                      (xout[((2 * 4 + t) * 4 + wave) * 64 + lane] + xout[((3 * 4 + t) * 4 + wave) * 64 + lane]);
      const f32x4 sm = (xsum[(0 * 4 + t) * 64 + lane] + xsum[(1 * 4 + t) * 64 + lane]) +
                       (xsum[(2 * 4 + t) * 64 + lane] + xsum[(3 * 4 + t) * 64 + lane]);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float l = row16_sum(sm[i]);
        const int row = row_begin + 16 * t + 4 * kq + i;
        if (row < row_end) Store<bf16_t>::store(out + (size_t)(sd.q_row0 + row) * d + h * DH + 16 * wave + r, o[i] / l);
      }
    }
  }
}
template <int DH, bool LONGK = false>
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
  else attn_tiles_mfma<DH, 16, LONGK>(q, Kb, out, sd, row_begin, row_end, h, d, scale, Vt, Pw, ldv, nk_all, qf_pre, kf_pre, Sbuf, nkp);
  __syncthreads();   // LDS is free for the next call
}

template <typename T, int DH, bool LONGK = false>
__device__ __forceinline__ void attn_block(const T* __restrict__ q, const T* __restrict__ Kb, const T* __restrict__ Vb,
                           T* __restrict__ out, const SeqDesc sd, int row_begin, int row_end, int h, int d,
                           float scale, unsigned* lds, int nk_cap) {
  if constexpr (sizeof(T) == 2 && DH % 32 == 0) {
    const int nk_need = sd.causal ? sd.nk_base + row_end : sd.nk_base;
    attn_block_mfma<DH, LONGK>(q, Kb, Vb, out, sd, row_begin, row_end, h, d, scale, lds, nk_need);
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

// ------------------------------------------------- operand staging through LayerNorm (GEMM and cross-attention kernels)
// A tile rows [row0, row0 + NR) of a workgroup from fp32 rows through LayerNorm (width
// 256 * NV, the 16-byte rule of ln_load4 / ln_stats4), in rounds of RB rows.
// after_first_loads(): called once, when the wave's first batch of row loads has been issued:
// whatever the caller wants in flight behind them.  Loads return in issue order, so what is
// needed first (the rows: everything waits for the tile) is requested first.
struct NoOp { __device__ __forceinline__ void operator()() const {} };
template <int NV, int RB, int NR, typename F = NoOp>
__device__ __forceinline__ void astat_stage_ln(const LnA& ln, bf16_t* At, int ld, int row0, int m0, int M,
                                               int lane, bool store_y, const F& after_first_loads = F{}) {
  constexpr int K = 256 * NV, ROUNDS = (NR + RB - 1) / RB;
  constexpr bool PIPE = ROUNDS > 1 && NV == 2;   // (the 1024-wide rows of four in a second register set would spill)
  float4 gv[NV], bv[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    gv[j] = *(const float4*)(ln.g + 4 * lane + 256 * j);
    bv[j] = *(const float4*)(ln.b + 4 * lane + 256 * j);
  }
  // NR rows in rounds of RB; with PIPE a round's rows are requested before the round before it is worked on (two
  // register sets), so that a wave with several rounds waits for memory once
  float4 xv[PIPE ? 2 : 1][RB][NV];
  auto request = [&](int rd) {
#pragma unroll
    for (int i = 0; i < RB; ++i)
      if (rd * RB + i < NR) ln_load4<NV>(ln.x + (size_t)min(m0 + row0 + rd * RB + i, M - 1) * K, lane, xv[PIPE ? rd & 1 : 0][i]);
  };
  request(0);
  after_first_loads();
#pragma unroll
  for (int rd = 0; rd < ROUNDS; ++rd) {
    const int i0 = rd * RB;
    float4 (&xr)[RB][NV] = xv[PIPE ? rd & 1 : 0];
    if (PIPE && rd + 1 < ROUNDS) request(rd + 1);
    if (!PIPE && rd > 0) request(rd);
    // statistics of all rows of the round first (independent reduction chains the scheduler can
    // interleave), then the values, then, in the workgroups that keep them, the fp32 rows
    float mean[RB], rstd[RB];
#pragma unroll
    for (int i = 0; i < RB; ++i) ln_stats4<NV>(xr[i0 + i < NR ? i : 0], K, mean[i], rstd[i]);
#pragma unroll
    for (int i = 0; i < RB; ++i) {
      if (i0 + i >= NR) break;
      const int row = row0 + i0 + i;
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const int c = 4 * lane + 256 * j;
        const float4 o = float4{ln_value(xr[i][j].x, mean[i], rstd[i], gv[j].x, bv[j].x), ln_value(xr[i][j].y, mean[i], rstd[i], gv[j].y, bv[j].y),
                                ln_value(xr[i][j].z, mean[i], rstd[i], gv[j].z, bv[j].z), ln_value(xr[i][j].w, mean[i], rstd[i], gv[j].w, bv[j].w)};
        const unsigned lo = (unsigned)f2bf(o.x) | ((unsigned)f2bf(o.y) << 16), hi = (unsigned)f2bf(o.z) | ((unsigned)f2bf(o.w) << 16);
        *(uint2*)(At + row * ld + c) = uint2{lo, hi};
        xr[i][j] = o;
      }
    }
    if (store_y) {
#pragma unroll
      for (int i = 0; i < RB; ++i) {
        const int m = m0 + row0 + i0 + i;
        if (i0 + i < NR && m < M) {
#pragma unroll
          for (int j = 0; j < NV; ++j) *(float4*)(ln.y + (size_t)m * K + 4 * lane + 256 * j) = xr[i][j];
        }
      }
    }
  }
}


// ------------------------------------------------- cross-attention with its query projection (kernels; launched from
// ad_kernels.hip, and from ad_attention_long.hip for configurations with long sources)
constexpr int kCrossqQld = 64 + 16;   // query tile row stride (elements): 32 bytes past a multiple of 64
inline size_t crossq_lds_bytes(int nk_cap, int mt, int d) {
  const size_t ldv = (size_t)((nk_cap + 31) & ~31) + 16;
  return (64 * ldv + ((size_t)64 * ldv > (size_t)mt * 16 * (d + 16) ? (size_t)64 * ldv : (size_t)mt * 16 * (d + 16)) + 64 * (size_t)kCrossqQld) * 2;
}
// The query projection of k_crossq_attention for MT row tiles: stage the chunk's rows in LDS (through
// the pending LayerNorm, or as they are), multiply by the wave's strip `b` of the query matrix,
// leave the queries (bias added, rounded) in the LDS tile Qt.  (A function with the arrays as
// reference parameters, not a lambda that captures them: captured arrays end up in scratch memory.)
// (LNMODE 1: the caller knows at compile time that a LayerNorm is pending; -1: ln.x decides)
template <int NV, int MT, int LNMODE = -1>
__device__ __forceinline__ void crossq_stage(const LnA& ln, const bf16_t* __restrict__ A, bf16_t* At, int m0, int m_end,
                                             bool keep_rows) {
  constexpr int K = 256 * NV, ld = K + 16, per_wave = MT * 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (LNMODE == 1 || ln.x) {
    astat_stage_ln<NV, (NV == 2 && per_wave <= 8 ? 8 : 4), per_wave>(ln, At, ld, wave * per_wave, m0, m_end, lane, keep_rows);
  } else {
    uint4 av[per_wave][K / 512];
#pragma unroll
    for (int i = 0; i < per_wave; ++i)
#pragma unroll
      for (int j = 0; j < K / 512; ++j)
        av[i][j] = *(const uint4*)(A + (size_t)min(m0 + wave * per_wave + i, m_end - 1) * K + j * 512 + lane * 8);
#pragma unroll
    for (int i = 0; i < per_wave; ++i)
#pragma unroll
      for (int j = 0; j < K / 512; ++j) *(uint4*)(At + (wave * per_wave + i) * ld + j * 512 + lane * 8) = av[i][j];
  }
  __syncthreads();
}
template <int NV, int MT>
__device__ __forceinline__ void crossq_multiply(const bf16_t* At, bf16_t* Qt, const uint4 (&b)[8 * NV], bool has_bias, float bn) {
  constexpr int K = 256 * NV, KS = K / 32, ld = K + 16, QLD = kCrossqQld;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, kq = lane >> 4;
  const bf16_t* a_lane = At + r * ld + kq * 8;
  f32x4 acc[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int u = 0; u < KS; ++u) {
    uint4 af[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) af[t] = *(const uint4*)(a_lane + t * 16 * ld + 32 * u);
#pragma unroll
    for (int t = 0; t < MT; ++t)
      acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, af[t]), __builtin_bit_cast(bf16x8, b[u]), acc[t], 0, 0, 0);
  }
  // this lane: rows 16 t + 4 kq + i of the chunk, column 16 wave + r of the head
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float v = acc[t][i];
      if (has_bias) v += bn;
      Qt[(t * 16 + 4 * kq + i) * QLD + wave * 16 + r] = f2bf(v);
    }
}
template <int NV, int MT, int LNMODE = -1>
__device__ __forceinline__ void crossq_project(const LnA& ln, const bf16_t* __restrict__ A, bf16_t* At, bf16_t* Qt,
                                               const uint4 (&b)[8 * NV], bool has_bias, float bn, int m0, int m_end,
                                               bool keep_rows) {
  crossq_stage<NV, MT, LNMODE>(ln, A, At, m0, m_end, keep_rows);
  crossq_multiply<NV, MT>(At, Qt, b, has_bias, bn);
}
// LONGK: the configuration's source capacity is kLongKeys or more (the summation order beyond 128 keys, attn_tiles_mfma)
// SMALL: what the launch bounds promise: 1 = one row tile per workgroup and at most 64 keys, 2 = at most 64 keys, 0 = nothing
template <int NV, int SMALL, bool LONGK = false, int LNMODE = -1>
__global__ __launch_bounds__(256) void k_crossq_attention(const SeqDesc* __restrict__ desc, int chunk_rows, float scale,
                                                          const bf16_t* __restrict__ W, const bf16_t* __restrict__ Kb,
                                                          const bf16_t* __restrict__ Vb, const float* __restrict__ ln_x,
                                                          const float* __restrict__ ln_g, const float* __restrict__ ln_b,
                                                          float* __restrict__ ln_y, const bf16_t* __restrict__ A,
                                                          const float* __restrict__ bias, bf16_t* __restrict__ out) {
  LnA ln;
  ln.x = ln_x; ln.g = ln_g; ln.b = ln_b; ln.y = ln_y;
  constexpr int K = 256 * NV, KS = K / 32, DH = 64, ld = K + 16, QLD = kCrossqQld, G = DH / 8;
  extern __shared__ uint4 cq_lds[];
  const SeqDesc sd = desc[blockIdx.x];
  const int row_begin = blockIdx.z * chunk_rows;
  if (row_begin >= sd.nq) return;
  const int row_end = min(sd.nq, row_begin + chunk_rows);
  const int h = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, kq = lane >> 4;
  const int mt = (row_end - row_begin + 15) >> 4;
  const int m0 = sd.q_row0 + row_begin, m_end = sd.q_row0 + row_end;   // packed rows of the chunk
  const int n0 = h * DH + wave * 16;
  const int nk_all = sd.causal ? sd.nk_base + row_end : sd.nk_base;
  const int nkp = (nk_all + 31) & ~31, ldv = nkp + 16;
  bf16_t* Vt = (bf16_t*)cq_lds;          // [DH][ldv]
  bf16_t* Pall = Vt + DH * ldv;          // [4 waves][16][ldv]
  bf16_t* At = Pall;                     // [16 * mt][K + 16]
  bf16_t* Qt = Pall + max(64 * ldv, mt * 16 * ld);   // [64][QLD]
  // the wave's strip of the query matrix
  uint4 b[KS];
  {
    const bf16_t* wp = W + (size_t)n0 * K + lane * 8;
#pragma unroll
    for (int u = 0; u < KS; ++u) b[u] = *(const uint4*)(wp + u * 512);
  }
  const float bn = bias ? bias[n0 + r] : 0.f;
  uint4 kf_pre[4][DH / 32];
  attn_preload_k<DH>(Kb, sd, row_begin, row_end, h, K, nk_all, kf_pre);
  // up to 128 keys: the values (piece i = 8 channels of one key; addresses clamped, never under a
  // branch of their own) wait in registers until the row tile is staged
  const bool v_small = SMALL || nkp <= 128;
  uint4 vreg[4];
  if (v_small) {
    const bf16_t* vg = Vb + (size_t)sd.kv_row0 * K + h * DH;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int i = min((int)threadIdx.x + 256 * it, nkp * G - 1);
      const int g = i / nkp, t = min(i - g * nkp, nk_all - 1);
      vreg[it] = *(const uint4*)(vg + (size_t)t * K + g * 8);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  // the number of row tiles as a constant (staging and product fully unrolled, as in the GEMM kernel)
  if (SMALL == 1 || mt == 1) crossq_project<NV, 1, LNMODE>(ln, A, At, Qt, b, bias != nullptr, bn, m0, m_end, h == 0);
  else if (mt == 2) crossq_project<NV, 2, LNMODE>(ln, A, At, Qt, b, bias != nullptr, bn, m0, m_end, h == 0);
  else if (mt == 3) crossq_project<NV, 3, LNMODE>(ln, A, At, Qt, b, bias != nullptr, bn, m0, m_end, h == 0);
  else crossq_project<NV, 4, LNMODE>(ln, A, At, Qt, b, bias != nullptr, bn, m0, m_end, h == 0);
  // values into LDS, transposed (keys nk_all .. nkp - 1 as zeros)
  if (v_small) {
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int i = threadIdx.x + 256 * it;
      if (i < nkp * G) {
        const int g = i / nkp, t = i - g * nkp;
        const uint4 v = t < nk_all ? vreg[it] : uint4{0u, 0u, 0u, 0u};
        bf16_t* dst = Vt + (size_t)(g * 8) * ldv + t;
        dst[0] = (bf16_t)(v.x & 0xffffu); dst[ldv] = (bf16_t)(v.x >> 16);
        dst[2 * ldv] = (bf16_t)(v.y & 0xffffu); dst[3 * ldv] = (bf16_t)(v.y >> 16);
        dst[4 * ldv] = (bf16_t)(v.z & 0xffffu); dst[5 * ldv] = (bf16_t)(v.z >> 16);
        dst[6 * ldv] = (bf16_t)(v.w & 0xffffu); dst[7 * ldv] = (bf16_t)(v.w >> 16);
      }
    }
  } else {
    attn_stage_values<DH>(Vb, sd, h, K, Vt, ldv, nkp, nk_all);
  }
  __syncthreads();   // queries and values are in LDS; the row tile is no longer needed
  // the rest is attn_block_mfma with the query fragments read from the LDS tile
  const int n_tiles = mt;
  uint4 qf_pre[DH / 32];
  {
    const int row = min(min(wave, n_tiles - 1) * 16 + r, row_end - row_begin - 1);
#pragma unroll
    for (int s2 = 0; s2 < DH / 32; ++s2) qf_pre[s2] = *(const uint4*)(Qt + row * QLD + kq * 8 + 32 * s2);
  }
  const int nt_all = (nk_all + 15) >> 4;
  const bool coop = !SMALL && row_end - row_begin <= 16 && nt_all > 8;
  float* Sbuf = coop ? (float*)(Pall + 16 * ldv) : nullptr;
  if (coop) {
    attn_coop_scores_q<DH>(qf_pre, Kb, sd, h, K, nk_all, nt_all, Sbuf, nkp);
    __syncthreads();
  }
  bf16_t* Pw = Pall + wave * 16 * ldv;
  const bf16_t* qnone = nullptr;   // every wave has at most one tile: its fragments are qf_pre
  if (SMALL || nkp <= 64) attn_tiles_mfma<DH, 4>(qnone, Kb, out, sd, row_begin, row_end, h, K, scale, Vt, Pw, ldv, nk_all, qf_pre, kf_pre, Sbuf, nkp);
  else if (nkp <= 128) attn_tiles_mfma<DH, 8>(qnone, Kb, out, sd, row_begin, row_end, h, K, scale, Vt, Pw, ldv, nk_all, qf_pre, kf_pre, Sbuf, nkp);
  else attn_tiles_mfma<DH, 16, LONGK>(qnone, Kb, out, sd, row_begin, row_end, h, K, scale, Vt, Pw, ldv, nk_all, qf_pre, kf_pre, Sbuf, nkp);
}
// The same for one row tile per workgroup against many keys (long sources): after the projection the four waves
// split the keys (attn_split_keys: wave w owns the 128-key super-blocks w, w + 4, ...), instead of one wave walking
// all of them behind a workgroup-wide staging of the values.  LDS: [4 waves: values, probabilities | row tile (until
// the queries are there)][exchange area][queries].
template <int NV>
__global__ __launch_bounds__(256) void k_crossq_attention_split(const SeqDesc* __restrict__ desc, float scale,
                                                                const bf16_t* __restrict__ W, const bf16_t* __restrict__ Kb,
                                                                const bf16_t* __restrict__ Vb, const float* __restrict__ ln_x,
                                                                const float* __restrict__ ln_g, const float* __restrict__ ln_b,
                                                                float* __restrict__ ln_y, const bf16_t* __restrict__ A,
                                                                const float* __restrict__ bias, bf16_t* __restrict__ out) {
  LnA ln;
  ln.x = ln_x; ln.g = ln_g; ln.b = ln_b; ln.y = ln_y;
  constexpr int K = 256 * NV, KS = K / 32, DH = 64, QLD = kCrossqQld;
  extern __shared__ uint4 cqs_lds[];
  const int h = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, kq = lane >> 4;
  const int n0 = h * DH + wave * 16;
  // the wave's strip of the query matrix first: its address depends on the head alone, not on the
  // sequence's descriptor, which is a trip to memory of its own
  uint4 b[KS];
  {
    const bf16_t* wp = W + (size_t)n0 * K + lane * 8;
#pragma unroll
    for (int u = 0; u < KS; ++u) b[u] = *(const uint4*)(wp + u * 512);
  }
  const float bn = bias ? bias[n0 + r] : 0.f;
  __builtin_amdgcn_sched_barrier(0);
  const SeqDesc sd = desc[blockIdx.x];
  const int row_begin = blockIdx.z * 16;
  if (row_begin >= sd.nq) return;
  const int row_end = min(sd.nq, row_begin + 16);
  const int m0 = sd.q_row0 + row_begin, m_end = sd.q_row0 + row_end;
  bf16_t* lds_waves = (bf16_t*)cqs_lds;
  bf16_t* At = lds_waves;                                          // [16][K + 16]
  float* xch = (float*)(lds_waves + 4 * kSplitWaveElems);
  bf16_t* Qt = (bf16_t*)((char*)xch + kSplitXchBytes);             // [16][QLD]
  const int nk_all = sd.causal ? sd.nk_base + row_end : sd.nk_base;
  // the wave's first keys are requested once the rows are staged (the staging's registers are free
  // again), its first values once the product has used up the weights
  crossq_stage<NV, 1>(ln, A, At, m0, m_end, h == 0);
  uint4 kf0[8][2], vraw0[2][8];
  split_request_keys(Kb, sd, h, K, nk_all, wave, kf0);
  crossq_multiply<NV, 1>(At, Qt, b, bias != nullptr, bn);
  split_request_values(Vb, sd, h, K, nk_all, wave, vraw0);
  __syncthreads();   // the queries are in LDS; the row tile is no longer needed
  uint4 qf[2];
  {
    const int row = min(r, row_end - row_begin - 1);
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) qf[s2] = *(const uint4*)(Qt + row * QLD + kq * 8 + 32 * s2);
  }
  attn_split_keys(qf, kf0, vraw0, Kb, Vb, out, sd, row_begin, row_end, h, K, scale, nk_all, lds_waves, xch);
}
inline size_t crossq_split_lds_bytes() { return attn_split_lds_bytes() + 16 * (size_t)kCrossqQld * 2; }

}  // namespace ad

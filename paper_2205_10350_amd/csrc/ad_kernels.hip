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
#pragma unroll 4
  for (int k0 = 0; k0 < K; k0 += 32) {
    const bf16x8 b = __builtin_bit_cast(bf16x8, *(const uint4*)(wp + k0 * 16));
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const bf16x8 a = __builtin_bit_cast(bf16x8, *(const uint4*)(ap[t] + k0));
      acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[t], 0, 0, 0);
    }
  }
  strip_epilogue<bf16_t, MT>(e, acc, MT, m0, n0, M, N, lane);
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
  if (m < M && n < N) epi_store<float>(e, m, n, N, acc);
}

void launch_gemm(int dtype, const void* A, const void* W, int M, int N, int K, const Epi& e, hipStream_t s) {
  if (M <= 0) return;
  if (dtype == AD_BF16) {
    const int nb = (N / 16 + 3) / 4;
    if (M <= 16)
      k_gemm_bf16<1><<<dim3(nb, 1), 256, 0, s>>>((const bf16_t*)A, (const bf16_t*)W, M, N, K, e);
    else if (M <= 32)
      k_gemm_bf16<2><<<dim3(nb, 1), 256, 0, s>>>((const bf16_t*)A, (const bf16_t*)W, M, N, K, e);
    else
      k_gemm_bf16<4><<<dim3(nb, (M + 63) / 64), 256, 0, s>>>((const bf16_t*)A, (const bf16_t*)W, M, N, K, e);
  } else {
    k_gemm_f32<<<dim3(N / 16, (M + 15) / 16), 256, 0, s>>>((const float*)A, (const float*)W, M, N, K, e);
  }
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

// ------------------------------------------------------------------------------------- LayerNorm
// One wave per row; mean, then biased variance of the centred values, eps = 1e-5.
template <typename T, int NV>
__device__ __forceinline__ void layernorm_row4(const float* __restrict__ xr, const float* __restrict__ g,
                                               const float* __restrict__ b, int d, int lane, float* __restrict__ yr,
                                               T* __restrict__ yar) {
  float4 xv[NV];
  float mean, rstd;
  ln_load4<false, NV>(xr, lane, xv);
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

// ------------------------------------------------------------------------------------- arg max, second stage
__global__ __launch_bounds__(256) void k_argmax_finish(const float* __restrict__ pv, const int* __restrict__ pi,
                                                       int M, int n_strips, int* __restrict__ o_hat,
                                                       float* __restrict__ o_val) {
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (m >= M) return;
  float v;
  int idx;
  argmax_row(pv + (size_t)m * n_strips, pi + (size_t)m * n_strips, n_strips, lane, v, idx);
  if (lane == 0) {
    o_hat[m] = idx;
    if (o_val) o_val[m] = v;
  }
}
void launch_argmax_finish(const float* pv, const int* pi, int M, int n_strips, int* o_hat, float* o_val,
                          hipStream_t s) {
  if (M <= 0) return;
  k_argmax_finish<<<(M + 3) / 4, 256, 0, s>>>(pv, pi, M, n_strips, o_hat, o_val);
}

template <typename T>
__global__ void k_gather_rows(const T* __restrict__ src, const int* __restrict__ rows, int d, T* __restrict__ dst) {
  const int r = blockIdx.x;
  const T* sp = src + (size_t)rows[r] * d;
  for (int c = threadIdx.x; c < d; c += blockDim.x) dst[(size_t)r * d + c] = sp[c];
}
void launch_gather_rows(int dtype, const void* src, const int* rows, int n, int d, void* dst, hipStream_t s) {
  if (n <= 0) return;
  if (dtype == AD_BF16) k_gather_rows<bf16_t><<<n, 128, 0, s>>>((const bf16_t*)src, rows, d, (bf16_t*)dst);
  else k_gather_rows<float><<<n, 128, 0, s>>>((const float*)src, rows, d, (float*)dst);
}

// ------------------------------------------------------------------------------------- row assembly
// Verify call: sequence b feeds (pending_b, draft_b[0..k_b-2]) at positions len_b .. len_b+k_b-1
// (Section 3.2, the verifier equation conditions row i on the accepted prefix and the first
// i-1 drafted tokens).  One block; thread 0 scans, all threads fill.
__global__ void k_assemble_verify(const int* __restrict__ k, const int* __restrict__ draft, int k_max,
                                  const int* __restrict__ len, const int* __restrict__ pending,
                                  const int* __restrict__ src_len, int B, int l_cap, int s_max, VerifyTables t) {
  if (threadIdx.x == 0) {
    int acc = 0;
    for (int b = 0; b < B; ++b) { t.row_start[b] = acc; acc += k[b]; }
    t.row_start[B] = acc;
  }
  __syncthreads();
  for (int b = threadIdx.x; b < B; b += blockDim.x) {
    SeqDesc s;
    s.q_row0 = t.row_start[b]; s.nq = k[b]; s.kv_row0 = b * l_cap; s.nk_base = len[b]; s.causal = 1;
    s.pad0 = s.pad1 = s.pad2 = 0;
    t.self_desc[b] = s;
    s.kv_row0 = b * s_max; s.nk_base = src_len[b]; s.causal = 0;
    t.cross_desc[b] = s;
  }
  for (int b = 0; b < B; ++b) {
    const int r0 = t.row_start[b], kb = k[b], L = len[b];
    for (int i = threadIdx.x; i < kb; i += blockDim.x) {
      t.row_tok[r0 + i] = i == 0 ? pending[b] : draft[b * k_max + i - 1];
      t.row_pos[r0 + i] = L + i;
      t.row_seq[r0 + i] = b;
      t.row_dst[r0 + i] = b * l_cap + L + i;
    }
  }
}
void launch_assemble_verify(const int* k, const int* draft, int k_max, const int* len, const int* pending,
                            const int* src_len, int B, int l_cap, int s_max, VerifyTables t, hipStream_t s) {
  k_assemble_verify<<<1, 256, 0, s>>>(k, draft, k_max, len, pending, src_len, B, l_cap, s_max, t);
}

// Encoder: rows = x_1..x_n of every sentence at positions 0..n-1, full self-attention over the
// sentence's own rows (keys live in the packed temporary buffers, row_dst = identity); the
// cross_desc slot describes where the memory keys/values of each sentence go.
__global__ void k_assemble_encoder(const int* __restrict__ src, int max_src, const int* __restrict__ src_len, int B,
                                   int s_max, VerifyTables t) {
  if (threadIdx.x == 0) {
    int acc = 0;
    for (int b = 0; b < B; ++b) { t.row_start[b] = acc; acc += src_len[b]; }
    t.row_start[B] = acc;
  }
  __syncthreads();
  for (int b = threadIdx.x; b < B; b += blockDim.x) {
    SeqDesc s;
    s.q_row0 = t.row_start[b]; s.nq = src_len[b]; s.kv_row0 = t.row_start[b]; s.nk_base = src_len[b]; s.causal = 0;
    s.pad0 = s.pad1 = s.pad2 = 0;
    t.self_desc[b] = s;
  }
  for (int b = 0; b < B; ++b) {
    const int r0 = t.row_start[b], n = src_len[b];
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
      t.row_tok[r0 + i] = src[b * max_src + i];
      t.row_pos[r0 + i] = i;
      t.row_seq[r0 + i] = b;
      t.row_dst[r0 + i] = r0 + i;            // own keys/values: packed temporaries
      t.row_dst2[r0 + i] = b * s_max + i;    // where this row's memory key/value goes
    }
  }
}
void launch_assemble_encoder(const int* src, int max_src, const int* src_len, int B, int s_max, VerifyTables t,
                             hipStream_t s) {
  k_assemble_encoder<<<1, 256, 0, s>>>(src, max_src, src_len, B, s_max, t);
}

// Drafter: rows = (o_0..o_j, [MASK] x k) at positions 0..j+k for every unfinished sequence
// (Section 3.2, draft paragraph), bidirectional self-attention over the sequence's own rows.
__global__ void k_assemble_drafter(const int* __restrict__ out, int max_len, const int* __restrict__ len,
                                   const int* __restrict__ finished, const int* __restrict__ src_len, int B, int k,
                                   int bos, int mask, int s_max, VerifyTables t, int* __restrict__ mask_rows) {
  if (threadIdx.x == 0) {
    int acc = 0;
    for (int b = 0; b < B; ++b) { t.row_start[b] = acc; acc += finished[b] ? 0 : len[b] + 1 + k; }
    t.row_start[B] = acc;
  }
  __syncthreads();
  for (int b = threadIdx.x; b < B; b += blockDim.x) {
    const int n = finished[b] ? 0 : len[b] + 1 + k;
    SeqDesc s;
    s.q_row0 = t.row_start[b]; s.nq = n; s.kv_row0 = t.row_start[b]; s.nk_base = n; s.causal = 0;
    s.pad0 = s.pad1 = s.pad2 = 0;
    t.self_desc[b] = s;
    s.kv_row0 = b * s_max; s.nk_base = src_len[b];
    t.cross_desc[b] = s;
  }
  int live = 0;   // index of sequence b among the unfinished ones: its mask rows are [live*k, live*k+k)
  for (int b = 0; b < B; ++b) {
    if (finished[b]) continue;
    const int r0 = t.row_start[b], L = len[b], n = L + 1 + k;
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
      t.row_tok[r0 + i] = i == 0 ? bos : (i <= L ? out[b * max_len + i - 1] : mask);
      t.row_pos[r0 + i] = i;
      t.row_seq[r0 + i] = b;
      t.row_dst[r0 + i] = r0 + i;
      if (i > L) mask_rows[live * k + (i - L - 1)] = r0 + i;
    }
    ++live;
  }
}
void launch_assemble_drafter(const int* out, int max_len, const int* len, const int* finished, const int* src_len,
                             int B, int k, int bos, int mask, int s_max, VerifyTables t, int* mask_rows,
                             hipStream_t s) {
  k_assemble_drafter<<<1, 256, 0, s>>>(out, max_len, len, finished, src_len, B, k, bos, mask, s_max, t, mask_rows);
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
__global__ void k_accept(const int* __restrict__ k, const int* __restrict__ draft, int k_max,
                         const int* __restrict__ o_hat, const int* __restrict__ row_start, int B, int eos,
                         int max_len, const int* __restrict__ max_out, int* __restrict__ len,
                         int* __restrict__ pending, int* __restrict__ finished, int* __restrict__ out,
                         int* __restrict__ result) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const int kb = k[b];
  if (kb == 0) { result[2 * b] = 0; result[2 * b + 1] = 0; return; }
  const int r0 = row_start[b];
  int c = kb;
  for (int i = 0; i < kb; ++i)
    if (draft[b * k_max + i] != o_hat[r0 + i]) { c = i + 1; break; }
  const int L = len[b], lim = max_out[b];
  int n = 0, last = 0;
  for (int i = 0; i < c; ++i) {
    if (L + n >= lim) break;
    last = o_hat[r0 + i];
    out[b * max_len + L + n] = last;
    ++n;
    if (last == eos) break;
  }
  len[b] = L + n;
  if (n > 0) pending[b] = last;
  finished[b] = (n > 0 && last == eos) || (L + n >= lim);
  result[2 * b] = n;
  result[2 * b + 1] = last;
}
void launch_accept(const int* k, const int* draft, int k_max, const int* o_hat, const int* row_start, int B, int eos,
                   int max_len, const int* max_out, int* len, int* pending, int* finished, int* out, int* result,
                   hipStream_t s) {
  k_accept<<<(B + 63) / 64, 64, 0, s>>>(k, draft, k_max, o_hat, row_start, B, eos, max_len, max_out, len, pending,
                                        finished, out, result);
}

__global__ void k_reset_state(int* len, int* pending, int* finished, int B, int bos) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  len[b] = 0; pending[b] = bos; finished[b] = 0;
}
void launch_reset_state(int* len, int* pending, int* finished, int B, int bos, hipStream_t s) {
  k_reset_state<<<(B + 63) / 64, 64, 0, s>>>(len, pending, finished, B, bos);
}

}  // namespace ad

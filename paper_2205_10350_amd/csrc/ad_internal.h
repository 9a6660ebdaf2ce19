// Internal declarations shared by the host side (ad_api.cpp, ad_hostlogic.cpp) and the
// kernels (ad_kernels.hip).  Nothing here is part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/ad.h"

namespace ad {

// ---- weight layout ---------------------------------------------------------------------
struct WEntry {
  std::string name;
  size_t offset;
  int rows, cols;     // vectors: rows = 1
  int elem_bytes;
  int tiled;          // 1: stored as 16 x 32 MFMA B-operand tiles (bf16 GEMM matrices)
};
// Ordered layout of one model's blob.  q,k,v of an attention block are contiguous so
// that they form one [3d, d] matrix (cross-attention: k,v form one [2d, d] matrix).
std::vector<WEntry> weight_layout(const ad_config& c, size_t* total_bytes);

struct AttnW { const void *wqkv, *wo; const float *bqkv, *bo; };          // wqkv = [wq;wk;wv]
struct LnW { const float *g, *b; };
struct FfnW { const void *w1, *w2; const float *b1, *b2; };
struct EncLayerW { AttnW self; LnW ln1; FfnW ffn; LnW ln2; };
struct DecLayerW { AttnW self; LnW ln1; AttnW cross; LnW ln2; FfnW ffn; LnW ln3; };
struct ModelW {
  const void* emb = nullptr;
  const void* out_w = nullptr;
  std::vector<EncLayerW> enc;
  std::vector<DecLayerW> dec;
};
ModelW bind_weights(const ad_config& c, const void* blob);

// ---- per-call row tables (device) -----------------------------------------------------------
// One attention problem per sequence: query rows [q_row0, q_row0+nq) of the packed
// activation matrix; keys/values are rows kv_row0.. of a [*, d] buffer.  Query row i
// (0-based inside the sequence) sees keys [0, causal ? nk_base + i + 1 : nk_base).
struct SeqDesc { int q_row0, nq, kv_row0, nk_base, causal, pad0, pad1, pad2; };

// ---- GEMM left operand given as rows still to be normalised -------------------------------------
// A = LayerNorm(x) * g + b over fp32 rows x [M, K]; the fp32 result also goes to y [M, K] (the
// residual input of a later sublayer).  x == nullptr: A is given as is.
struct LnA {
  const float* x = nullptr;
  const float* g = nullptr;
  const float* b = nullptr;
  float* y = nullptr;
};

// ---- GEMM epilogues ----------------------------------------------------------------------------
// EPI_COUNT (output projection only): per row, how many columns score strictly above the row's
// threshold `thr`; integer partials go where EPI_ARGMAX puts its index partials.
enum EpiMode { EPI_QKV = 0, EPI_KV = 1, EPI_STORE = 2, EPI_RELU = 3, EPI_RESID = 4, EPI_ARGMAX = 5, EPI_COUNT = 6 };
struct Epi {
  int mode;
  int d;                  // model width (column split of QKV / KV)
  const float* bias;      // [N] or null
  void* out0;             // QKV: q [M,d];  STORE/RELU: out [M,N] (storage type);  RESID: fp32 [M,N]
  void* out1;             // QKV/KV: key rows buffer [*, d]
  void* out2;             // QKV/KV: value rows buffer [*, d]
  const int* row_dst;     // QKV/KV: destination row of packed row m in out1/out2
  const float* resid;     // RESID: fp32 [M,N]
  float* part_val;        // ARGMAX: [M, n_strips]
  int* part_idx;          // ARGMAX: [M, n_strips]
  int n_strips;
  float* logits;          // ARGMAX: optional full logits [M,N]
  const float* thr;       // COUNT: [M] thresholds
  size_t layer_stride;    // KV with N = layers * 2d: bytes from one layer's key (value) buffer to the next
};

// ---- launchers (ad_kernels.hip).  dtype: AD_F32 / AD_BF16 selects storage + arithmetic ---------
void launch_embed(int dtype, const void* emb, const float* pe, const int* tok, const int* pos, int M,
                  int d, float sqrt_d, float* x, void* xa, hipStream_t s);
// C[M,N] = A[M,K] . W[N,K]^T with epilogue.  A, W in the storage type.
// returns the number of arg-max partials per row an EPI_ARGMAX launch wrote (row stride e.n_strips)
// With `ln` set, A is LayerNorm(ln.x): kernels that can, normalise the rows while staging them
// (then the storage-type rows `A` are NOT written); otherwise a LayerNorm launch fills ln.y and A
// first.  Same values either way.
int launch_gemm(int dtype, const void* A, const void* W, int M, int N, int K, const Epi& e, hipStream_t s,
                const LnA& ln = LnA{}, bool* a_written = nullptr);
// one attention problem per descriptor (n_seq of them, at most max_rows query rows each)
void launch_attention(int dtype, const void* q, const void* K, const void* V, void* out, const SeqDesc* desc,
                      int n_seq, int max_rows, int H, int dh, int max_keys, hipStream_t s);
// the same launch for long key ranges (ad_attention_long.hip; bf16, head width 64, grid and LDS bytes as launch_attention computes them)
void launch_attention_long(const void* q, const void* K, const void* V, void* out, const SeqDesc* desc, dim3 grid, int d,
                           float scale, int max_keys, size_t lds_bytes, hipStream_t s);
bool launch_crossq_attention_long(const LnA& ln, const void* A, const void* W, const float* bias, const void* K, const void* V,
                                  void* out, const SeqDesc* desc, int n_seq, int max_rows, int H, int chunk, int max_keys,
                                  hipStream_t s);
// Cross-attention of a decoder layer with its query projection (and the pending LayerNorm of the
// rows, `ln`, or the rows `A` as they are) in one launch; false = shape not covered (nothing
// launched: use launch_gemm + launch_attention).
bool launch_crossq_attention(int dtype, const LnA& ln, const void* A, const void* W, const float* bias, const void* K,
                             const void* V, void* out, const SeqDesc* desc, int n_seq, int max_rows, int H, int dh,
                             int max_keys, hipStream_t s);
// y = LayerNorm(x) * g + b -> y (fp32) and ya (storage type)
void launch_layernorm(int dtype, const float* x, const float* g, const float* b, int M, int d, float* y,
                      void* ya, hipStream_t s);
hipError_t launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t s);
// workgroups x 4 waves x iters x 8 bf16 MFMAs (16x16x32) on fixed register operands; out: workgroups x 256 floats
hipError_t launch_calibration_mfma(float* out, int workgroups, int iters, hipStream_t s);
// second stage of the arg max: n_part partials per row, rows `stride` entries apart
void launch_argmax_finish(const float* part_val, const int* part_idx, int M, int stride, int n_part, int* o_hat,
                          float* o_val, hipStream_t s);
// GAD++ (Section 3.2.3).  Score of every row's drafted token, by the same dot-product chain the
// output projection uses (bit-identical to the logit it computes for that column): lp[m], and the
// drafted token col[m] (negative: the never-matching id).
void launch_draft_logit(int dtype, const void* A, const void* W, int M, int N, int K, const int* row_seq,
                        const int* row_start, const int* draft, int k_max, float* lp, int* col, hipStream_t s);
// second stage of the arg max over the drafter's M = live * k mask rows; token i of the l-th unfinished
// sequence b goes to the 8-byte slot [b * k_max + i] of `slots` (host-visible) as (*ticket_in << 32 | token)
void launch_argmax_draft(const float* part_val, const int* part_idx, int M, int stride, int n_part, int* o_hat,
                         const int* finished, int B, int k, int k_max, const int* ticket_in, unsigned long long* slots,
                         hipStream_t s);

// Row assembly of a verify call: from k[B], draft[B,k_max], len[B], pending[B] builds the
// packed row tables and both attention descriptors.
struct VerifyTables {
  int *row_tok, *row_pos, *row_seq, *row_dst, *row_start;   // [M], [M], [M], [M], [B+1]
  int* row_dst2;   // [M] encoder only: row of the memory key/value buffers
  SeqDesc *self_desc, *cross_desc;                          // [B]
};
// those tables and the embedding of the M rows (x, xa) in one launch
void launch_assemble_embed_verify(int dtype, const int* k, const int* draft, const int* rows, int rows_stride, int k_max, const int* len,
                                  const int* pending, const int* src_len, int B, int l_cap, int s_max, VerifyTables t,
                                  int M, const void* emb, const float* pe, int d, float sqrt_d, float* x, void* xa,
                                  hipStream_t s);
// GAD++ inputs of the acceptance kernel (Section 3.2.3; part_cnt == nullptr: plain verification):
// a row's drafted token `col` (score `lp`) replaces its arg max where fewer than `beta` columns
// score above it (the counting pass's partials, n_part per row at `stride`) and the top score is
// at most `tau` above it.
struct GadppIn {
  const int* part_cnt = nullptr;
  int stride = 0, n_part = 0;
  const float* lp = nullptr;
  const int* col = nullptr;
  int beta = 1;
  float tau = 0.f;
};
// Longest-prefix match, acceptance, truncation and rollback for every sequence.
// second stage of the arg max (as launch_argmax_finish) and acceptance in one launch; with
// ticket_out set (host-visible memory), sequence b's 8-byte slot receives *ticket_in (18 bits), the accepted
// length (14) and the next token (32) in one store
void launch_argmax_accept(const float* part_val, const int* part_idx, int stride, int n_part, int* o_hat, float* o_val,
                          const int* k, const int* draft, int k_max, const int* row_start, int B, int eos, int max_len,
                          const int* max_out, int* len, int* pending, int* finished, int* out, int* result,
                          const int* ticket_in, unsigned long long* ticket_out, int max_rows, int M /* sum of k */,
                          hipStream_t s, const GadppIn& gp = GadppIn{});
// Row tables for the encoder (rows = source tokens) and for the drafter (prefix + masks).
// the encoder's row tables, the embedding of the M rows, the copy of src_len (and, with len set, of
// max_out and the start state of a decode) in one launch; the three inputs may be host memory
void launch_assemble_embed_encoder(int dtype, const int* src, int max_src, const int* src_len, const int* max_out_in,
                                   int B, int s_max, VerifyTables t, int* src_len_out, int* max_out, int* len,
                                   int* pending, int* finished, int bos, int M, const void* emb, const float* pe, int d,
                                   float sqrt_d, float* x, void* xa, hipStream_t s);
// Drafter rows: the k mask rows of every unfinished sequence first (l-th unfinished sequence at
// [l*k, l*k + k)), then the prefix rows; descriptors [0, live) = mask rows as queries,
// [live, 2 live) = prefix rows (self_desc and cross_desc hold 2 B entries).
// (with the embedding of the M packed rows in the same launch: x, xa as launch_embed writes them)
void launch_assemble_embed_drafter(int dtype, const int* out, int max_len, const int* len, const int* finished,
                                   const int* src_len, int B, int k, int bos, int mask, int s_max, VerifyTables t,
                                   int M, const void* emb, const float* pe, int d, float sqrt_d, float* x, void* xa,
                                   hipStream_t s);
void launch_draft_scatter(const int* o_hat, const int* finished, int B, int k, int k_max, int* draft_out,
                          hipStream_t s);

// ---- host-only decode loops (ad_hostlogic.cpp) ------------------------------------------------------
struct Backend {
  virtual ~Backend() {}
  // same contract as ad_verify, minus `verified`
  virtual int verify(const int32_t* draft, const int32_t* k, int32_t* n_accept, int32_t* next) = 0;
  virtual int draft(int k, int32_t* draft_out) { (void)k; (void)draft_out; return AD_ESTATE; }
};
struct LoopIO {
  int B, k_max, eos, bos;
  std::vector<int> max_out;            // [B]
  std::vector<std::vector<int32_t>> o; // per sequence: o_0 = bos, then output
  std::vector<std::vector<int>> accepted;  // per iteration, summed over the batch handled by caller
  ad_stats stats{};
};
int suffix_match(const int32_t* o, int o_len, const int32_t* x, int x_len, int* i_out);
int loop_iad(Backend& be, LoopIO& io, const std::vector<std::vector<int32_t>>& guide);
int loop_gad(Backend& be, LoopIO& io, int k, bool use_drafter,
             const std::vector<std::vector<int32_t>>* override_draft);
int loop_greedy(Backend& be, LoopIO& io);

void set_global_error(const char* msg);

}  // namespace ad

// Context, workspace plan and the forward passes (encode, verify, draft) behind the C ABI.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <chrono>
#include <string>
#include <map>
#include <utility>
#include <vector>

#include "ad_internal.h"

namespace ad {
const char* global_error();

static size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// LDS bytes of the block attention (the device code's attn_lds_bytes): the larger of the scalar
// path's need (two padded [nk, dh] tiles plus per-wave query and score rows) and the matrix-core
// path's (transposed values [dh][keys + 8] and one 16-row probability tile per wave)
static size_t attn_lds_host(int nk_cap, int dh, int esz, int waves) {
  const size_t row_dwords = (size_t)dh * esz / 4 + 1;
  const size_t scalar_path = 2 * (size_t)nk_cap * row_dwords * 4 + 64 * (size_t)dh * 4 + (size_t)waves * nk_cap * 4;
  const size_t ldv = (size_t)((nk_cap + 31) & ~31) + 16;
  const size_t mfma_path = ((size_t)dh + 16 * (size_t)waves) * ldv * 2;
  return std::max(scalar_path, mfma_path);
}

// ---------------------------------------------------------------------------------------------
// Workspace plan: one pass computes offsets; used both for sizing and for binding.
struct Plan {
  size_t total = 0;
  int esz = 4;          // storage element size of activations / caches
  int m_cap = 0;        // packed rows of any forward
  int mv_cap = 0;       // rows that reach the output projection
  int l_cap = 0;        // rows of a sequence's self-attention cache
  int n_strips = 0;
  int max_pos = 0;
  size_t kv_w[2], kv_b[2];   // per model: cross-attention [wk; wv] of every decoder layer as one matrix, and its bias
  // [act_begin, act_end): what one forward pass works in (rows, row tables, descriptors); with a
  // drafter a second block of the same layout lies act2_shift bytes further on, for the drafter's
  // encoder running beside the verifier's on a stream of its own
  size_t act_begin = 0, act_end = 0, act2_shift = 0;
  size_t pe, x, s, xa, q, att, tk, tv, f, part_val, part_idx, o_hat, o_val, logits, draft_lp, draft_col;
  size_t cache_k, cache_v, cache_layer_stride;          // [NL][B*l_cap, d]
  size_t mem_k[2], mem_v[2], mem_layer_stride;          // per model: [NL][B*max_src, d]
  size_t row_tok, row_pos, row_seq, row_dst, row_dst2, row_start, self_desc, cross_desc;
  size_t len, pending, finished, max_out, src_len[2], out, result, k_dev, draft_dev, src_dev, draft_out;
};

static Plan make_plan(const ad_config& c, bool with_drafter) {
  Plan p;
  p.esz = c.dtype == AD_BF16 ? 2 : 4;
  const size_t B = c.max_batch, d = c.d_model;
  p.l_cap = c.max_len + c.k_max;
  p.mv_cap = (int)(B * c.k_max);
  size_t m = std::max(B * c.k_max, B * c.max_src);
  if (with_drafter) m = std::max(m, B * (size_t)(c.max_len + c.k_max));
  p.m_cap = (int)m;
  p.n_strips = c.vocab / 16;
  p.max_pos = std::max(c.max_src, c.max_len + c.k_max);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  p.pe = take((size_t)p.max_pos * d * 4);
  p.act_begin = off;
  p.x = take(m * d * 4);
  p.s = take(m * d * 4);
  p.xa = take(m * d * p.esz);
  p.q = take(m * d * p.esz);
  p.att = take(m * d * p.esz);
  p.tk = take(m * d * p.esz);
  p.tv = take(m * d * p.esz);
  p.f = take(m * (size_t)c.d_ffn * p.esz);
  p.row_tok = take(m * 4); p.row_pos = take(m * 4); p.row_seq = take(m * 4); p.row_dst = take(m * 4); p.row_dst2 = take(m * 4);
  p.row_start = take((B + 1) * 4);
  p.self_desc = take(2 * B * sizeof(SeqDesc));    // the drafter has two per sequence (mask rows, prefix rows)
  p.cross_desc = take(2 * B * sizeof(SeqDesc));
  p.act_end = off;
  if (with_drafter) {
    // the second block needs room for an encoder forward only: the same layout scaled would do, the
    // same size is simpler
    p.act2_shift = p.act_end - p.act_begin;
    off += p.act2_shift;
  }
  p.part_val = take((size_t)p.mv_cap * p.n_strips * 4);
  p.part_idx = take((size_t)p.mv_cap * p.n_strips * 4);
  p.o_hat = take((size_t)p.mv_cap * 4);
  p.o_val = take((size_t)p.mv_cap * 4);
  p.draft_lp = take((size_t)p.mv_cap * 4);
  p.draft_col = take((size_t)p.mv_cap * 4);
  p.logits = take(c.debug_logits ? (size_t)p.mv_cap * c.vocab * 4 : 0);
  p.cache_layer_stride = align_up(B * p.l_cap * d * p.esz);
  p.cache_k = take(p.cache_layer_stride * c.dec_layers);
  p.cache_v = take(p.cache_layer_stride * c.dec_layers);
  p.mem_layer_stride = align_up(B * c.max_src * d * p.esz);
  for (int i = 0; i < 2; ++i) {
    const bool on = i == 0 || with_drafter;
    p.mem_k[i] = take(on ? p.mem_layer_stride * c.dec_layers : 0);
    p.mem_v[i] = take(on ? p.mem_layer_stride * c.dec_layers : 0);
    p.src_len[i] = take(B * 4);
    p.kv_w[i] = take(on ? (size_t)c.dec_layers * 2 * d * d * p.esz : 0);
    p.kv_b[i] = take(on ? (size_t)c.dec_layers * 2 * d * 4 : 0);
  }
  p.len = take(B * 4); p.pending = take(B * 4); p.finished = take(B * 4); p.max_out = take(B * 4);
  p.out = take(B * c.max_len * 4);
  p.result = take(B * 2 * 4);   // [B,2] results
  p.k_dev = take(B * 4 + B * c.k_max * 4);   // k[B] followed by draft[B, k_max]: one upload
  p.draft_dev = p.k_dev + B * 4;
  p.src_dev = take(B * 4 * 2 + B * c.max_src * 4);   // src_len[B], max_out[B], src[B, max_src]: one upload
  p.draft_out = take(B * c.k_max * 4);
  p.total = off;
  return p;
}

// Layout (in ints) of the pinned, device-mapped host staging buffer.  Every part has a place of
// its own for the whole life of the context, sized for max_batch: what one call leaves behind
// never lies where another call's words are watched.
struct PinLayout {
  size_t k, draft, result, o_hat;     // ad_verify: k[B], draft[B, k_max] in; result[B, 2], o_hat[mv_cap] out
  size_t rows;                        // ad_verify: the packed rows, (sequence << 14 | index)[mv_cap] then the fed token (or -1: the pending one)[mv_cap]
  size_t v_ticket, v_slots;           // ad_verify: the call's ticket (in), one 8-byte result word per sequence (out)
  size_t d_ticket, d_slots;           // ad_draft_nat: ticket (in), one 8-byte (ticket, token) word per drafted token (out)
  size_t d_copy;                      // ad_draft_nat without the watch: draft_out[B, k_max]
  size_t enc[2];                      // ad_encode per model: src_len[B], max_out[B], src[B, max_src]
  size_t out;                         // ad_output: out[B, max_len]
  size_t total;
};
static PinLayout make_pin_layout(const ad_config& c, const Plan& p) {
  PinLayout l{};
  const size_t B = c.max_batch;
  size_t off = 0;
  auto take = [&](size_t ints) { size_t o = off; off = (off + ints + 3) & ~(size_t)3; return o; };   // 16-byte steps
  l.k = take(B); l.draft = take(B * c.k_max); l.result = take(2 * B); l.o_hat = take(p.mv_cap);
  l.rows = take(2 * p.mv_cap);
  l.v_ticket = take(4); l.v_slots = take(2 * B);
  l.d_ticket = take(4); l.d_slots = take(2 * B * c.k_max);
  l.d_copy = take(B * c.k_max);
  for (int i = 0; i < 2; ++i) l.enc[i] = take(B * (2 + (size_t)c.max_src));
  l.out = take(B * c.max_len);
  l.total = off;
  return l;
}

// where the output projection leaves its arg-max partials: [rows, stride] values and indices
struct PartialBuf { float* val; int* idx; int stride; };

// The static scratch array of ad_verify_static (arg-max partials: values in the first half, indices
// in the second).  Every GPU the library runs on holds its own copy at its own address; the name
// below is a host-side stand-in, so host code only ever uses the address hipGetSymbolAddress
// reports for the current device (looked up once per device in ad_create).
constexpr size_t kStaticScratchBytes = 4u << 20;
static __device__ __align__(256) unsigned char ad_static_scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {};
static void* static_scratch_for_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return nullptr; }
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(ad_static_scratch)) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace ad

using namespace ad;

struct ad_ctx {
  ad_config cfg;
  Plan plan;
  ModelW w[2];
  bool has_drafter = false;
  char* ws = nullptr;
  hipStream_t stream = nullptr;
  hipEvent_t ev0 = nullptr, ev1 = nullptr, ev2 = nullptr, ev3 = nullptr;
  hipEvent_t ev_up[2] = {nullptr, nullptr};   // per model: the last ad_encode's inputs have been read from the staging buffer
  bool up_pending[2] = {false, false};
  int32_t* pin = nullptr;       // pinned staging, ints
  int32_t* pin_dev = nullptr;   // the same buffer as the device addresses it (null: not mapped, use copies)
  PinLayout pl{};
  void* scratch_dev = nullptr;  // this device's address of the static scratch array (ad_verify_static)
  char err[320] = "";
  // host mirror of the decode state
  int B = 0;
  bool encoded[2] = {false, false};
  std::vector<int> h_len, h_finished, h_max_out, h_src_len[2];
  // last verify call, for ad_time_verify_forward / ad_debug_logits
  int last_M = 0;
  int last_logit_rows = 0;
  // shape of the forward being launched: attention problems and the most query rows in one
  int fw_nseq = 0, fw_max_rows = 0;
  int last_nseq = 0, last_max_rows = 0;
  // the keys the longest self-attention problem of the current / last verify forward sees (prefix + block, from the host's
  // mirror of the lengths); 0: unknown, the cache capacity bounds them
  int fw_self_keys = 0, last_self_keys = 0;
  // the same for the cross-attention: the longest source of the batch the forward runs on
  int fw_cross_keys = 0, last_cross_keys = 0;
  // LayerNorm deferred into the next GEMM's operand staging: s -> (x, xa) with these parameters
  const LnW* ln_pending = nullptr;
  const LnW* ln_vocab = nullptr;  // the one the last verify forward's output projection applied (timing)
  int ticket = 0;                 // number of the last ad_verify call that waited by watching memory
  bool spin_wait = true;
  bool fuse_crossq = true;   // cross-attention: query projection + attention as one launch (AD_OPT_FUSE_CROSSQ)
  int gadpp_beta = 1;             // GAD++ (Section 3.2.3): 1 = plain top-1 verification
  float gadpp_tau = 0.f;
  // One launch per stage: the launches of a verify call (row assembly, forward, acceptance) are
  // captured into a graph per call shape on the shape's third appearance and replayed after.
  bool graphs_on = true;
  typedef std::pair<unsigned long long, unsigned long long> GraphKey;   // (kind | shape, further shape values)
  std::map<GraphKey, hipGraphExec_t> graphs;
  std::map<GraphKey, int> graph_seen;
  std::vector<int> last_k;       // k[b] of the last verify call

  // the drafter's encoder beside the verifier's: a stream of the library's own (default priority),
  // the second activation block, and the two events that order it against the context's stream
  hipStream_t stream2 = nullptr;
  hipEvent_t ev_fork = nullptr, ev_enc2 = nullptr;
  bool overlap_encoders = false, fork_recorded = false, enc2_pending = false;
  size_t act_shift = 0;          // 0, or plan.act2_shift while a forward works in the second block

  template <typename T> T* at(size_t off) const {
    return (T*)(ws + off + ((off >= plan.act_begin && off < plan.act_end) ? act_shift : 0));
  }
};

// (messages go into fixed buffers: reporting an error allocates nothing)
static int fail(ad_ctx* c, int code, const char* msg) {
  if (c) snprintf(c->err, sizeof(c->err), "%s", msg);
  set_global_error(msg);
  return code;
}
static int fail_hip(ad_ctx* c, const char* what, hipError_t e) {
  char msg[300];
  snprintf(msg, sizeof(msg), "%.200s: %.90s", what, hipGetErrorString(e));
  return fail(c, AD_EDEVICE, msg);
}
#define HIP_TRY(ctx, expr)                                          \
  do {                                                              \
    hipError_t e_ = (expr);                                         \
    if (e_ != hipSuccess) return fail_hip(ctx, #expr, e_);          \
  } while (0)

static double now_us() {
  return std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

// ---------------------------------------------------------------------------------------------
// Forward passes.  All launches go to ctx->stream; shapes were validated by the callers.

static const void* w_rows(const ad_ctx* c, const void* w, size_t rows, size_t cols) {
  return (const char*)w + rows * cols * (c->cfg.dtype == AD_BF16 ? 2 : 4);
}

static VerifyTables tables(const ad_ctx* c) {
  const Plan& p = c->plan;
  VerifyTables t;
  t.row_tok = c->at<int>(p.row_tok); t.row_pos = c->at<int>(p.row_pos); t.row_seq = c->at<int>(p.row_seq);
  t.row_dst = c->at<int>(p.row_dst); t.row_dst2 = c->at<int>(p.row_dst2); t.row_start = c->at<int>(p.row_start);
  t.self_desc = c->at<SeqDesc>(p.self_desc); t.cross_desc = c->at<SeqDesc>(p.cross_desc);
  return t;
}

// s = x + A W^T + bias; the LayerNorm s -> (x, xa) is left to the next consumer of the rows:
// gemm_rows() applies it while staging its operand where the kernel can, flush_ln() runs it as
// a launch of its own.
static void gemm_resid_ln(ad_ctx* c, const void* A, const void* W, const float* bias, int M, int N, int K,
                          const LnW& ln) {
  const Plan& p = c->plan;
  Epi e{};
  e.mode = EPI_RESID; e.bias = bias; e.out0 = c->at<float>(p.s); e.resid = c->at<float>(p.x);
  launch_gemm(c->cfg.dtype, A, W, M, N, K, e, c->stream);
  c->ln_pending = &ln;
}
static void flush_ln(ad_ctx* c, int M) {
  if (!c->ln_pending) return;
  const Plan& p = c->plan;
  launch_layernorm(c->cfg.dtype, c->at<float>(p.s), c->ln_pending->g, c->ln_pending->b, M, c->cfg.d_model,
                   c->at<float>(p.x), c->at<void>(p.xa), c->stream);
  c->ln_pending = nullptr;
}
// GEMM over the current rows (xa, or the pending LayerNorm of s)
static int gemm_rows(ad_ctx* c, const void* W, int M, int N, const Epi& e) {
  const Plan& p = c->plan;
  LnA ln{};
  if (c->ln_pending) {
    ln.x = c->at<float>(p.s); ln.g = c->ln_pending->g; ln.b = c->ln_pending->b; ln.y = c->at<float>(p.x);
    c->ln_pending = nullptr;
  }
  return launch_gemm(c->cfg.dtype, c->at<void>(p.xa), W, M, N, c->cfg.d_model, e, c->stream, ln);
}

static void ffn_block(ad_ctx* c, const FfnW& f, const LnW& ln, int M) {
  const Plan& p = c->plan;
  const int d = c->cfg.d_model, F = c->cfg.d_ffn;
  Epi e{};
  e.mode = EPI_RELU; e.bias = f.b1; e.out0 = c->at<void>(p.f);
  gemm_rows(c, f.w1, M, F, e);
  gemm_resid_ln(c, c->at<void>(p.f), f.w2, f.b2, M, d, F, ln);
}

// Self-attention block: q,k,v projection with the key/value rows written to (Kl, Vl) at
// row_dst, attention, output projection + residual + LayerNorm.
// head_rows > 0: from the attention on, only the first head_rows packed rows are needed (they are
// the queries of the first head_nseq descriptors, at most head_max_rows each): keys and values are
// still projected from all M rows.
static void self_attn_block(ad_ctx* c, const AttnW& a, const LnW& ln, int M, void* Kl, void* Vl, int max_keys,
                            int head_rows = 0, int head_nseq = 0, int head_max_rows = 0) {
  const Plan& p = c->plan;
  const int d = c->cfg.d_model, H = c->cfg.n_heads;
  VerifyTables t = tables(c);
  Epi e{};
  e.mode = EPI_QKV; e.d = d; e.bias = a.bqkv; e.out0 = c->at<void>(p.q); e.out1 = Kl; e.out2 = Vl; e.row_dst = t.row_dst;
  gemm_rows(c, a.wqkv, M, 3 * d, e);
  if (head_rows > 0) { c->fw_nseq = head_nseq; c->fw_max_rows = head_max_rows; M = head_rows; }
  // (a bound of at most 64 keys selects the compact attention kernel; it is part of the call shape's graph key)
  const int key_bound = c->fw_self_keys > 0 && c->fw_self_keys <= 64 ? 64 : max_keys;
  launch_attention(c->cfg.dtype, c->at<void>(p.q), Kl, Vl, c->at<void>(p.att), t.self_desc, c->fw_nseq, c->fw_max_rows,
                   H, d / H, key_bound, c->stream);
  gemm_resid_ln(c, c->at<void>(p.att), a.wo, a.bo, M, d, d, ln);
}

static void cross_attn_block(ad_ctx* c, const AttnW& a, const LnW& ln, int M, const void* Km, const void* Vm) {
  const Plan& p = c->plan;
  const int d = c->cfg.d_model, H = c->cfg.n_heads;
  VerifyTables t = tables(c);
  // query projection (with the pending LayerNorm) and attention in one launch where the shape allows
  LnA la{};
  if (c->ln_pending) {
    la.x = c->at<float>(p.s); la.g = c->ln_pending->g; la.b = c->ln_pending->b; la.y = c->at<float>(p.x);
  }
  // (only a bound of at most 64 keys replaces the capacity: it selects the compact kernels, whose results for such key
  // counts are those of every other kernel; a bound between the classes of longer ranges could change the summation order)
  const int key_bound = c->fw_cross_keys > 0 && c->fw_cross_keys <= 64 ? 64 : c->cfg.max_src;
  if (c->fuse_crossq &&
      launch_crossq_attention(c->cfg.dtype, la, c->at<void>(p.xa), a.wqkv, a.bqkv, Km, Vm,
                              c->at<void>(p.att), t.cross_desc, c->fw_nseq, c->fw_max_rows, H, d / H, key_bound,
                              c->stream)) {
    c->ln_pending = nullptr;
  } else {
    Epi e{};
    e.mode = EPI_STORE; e.bias = a.bqkv; e.out0 = c->at<void>(p.q);
    gemm_rows(c, a.wqkv, M, d, e);
    launch_attention(c->cfg.dtype, c->at<void>(p.q), Km, Vm, c->at<void>(p.att), t.cross_desc, c->fw_nseq,
                     c->fw_max_rows, H, d / H, key_bound, c->stream);
  }
  gemm_resid_ln(c, c->at<void>(p.att), a.wo, a.bo, M, d, d, ln);
}

static void embed_rows(ad_ctx* c, const ModelW& w, int M) {
  const Plan& p = c->plan;
  c->ln_pending = nullptr;
  VerifyTables t = tables(c);
  launch_embed(c->cfg.dtype, w.emb, c->at<float>(p.pe), t.row_tok, t.row_pos, M, c->cfg.d_model,
               sqrtf((float)c->cfg.d_model), c->at<float>(p.x), c->at<void>(p.xa), c->stream);
}

// Output projection fused with the per-row arg max; `A` holds Mv rows.
static int vocab_argmax(ad_ctx* c, const ModelW& w, const void* A, int Mv, const LnW* ln_of_s = nullptr,
                        const void* out_w = nullptr /* another copy of w.out_w (timing) */,
                        const PartialBuf* pb = nullptr /* null: the workspace's partial buffers */) {
  const Plan& p = c->plan;
  Epi e{};
  e.mode = EPI_ARGMAX;
  e.part_val = pb ? pb->val : c->at<float>(p.part_val); e.part_idx = pb ? pb->idx : c->at<int>(p.part_idx);
  e.n_strips = pb ? pb->stride : p.n_strips; e.logits = c->cfg.debug_logits ? c->at<float>(p.logits) : nullptr;
  LnA ln{};
  if (ln_of_s) { ln.x = c->at<float>(p.s); ln.g = ln_of_s->g; ln.b = ln_of_s->b; ln.y = c->at<float>(p.x); }
  return launch_gemm(c->cfg.dtype, A, out_w ? out_w : w.out_w, Mv, c->cfg.vocab, c->cfg.d_model, e, c->stream, ln);
}
static void vocab_finish(ad_ctx* c, int Mv, int n_part, const PartialBuf* pb = nullptr) {
  const Plan& p = c->plan;
  launch_argmax_finish(pb ? pb->val : c->at<float>(p.part_val), pb ? pb->idx : c->at<int>(p.part_idx), Mv,
                       pb ? pb->stride : p.n_strips, n_part, c->at<int>(p.o_hat), c->at<float>(p.o_val), c->stream);
}

// The verify forward over the M packed rows the tables describe.  ev (optional) brackets the
// output-projection kernel.
// finish = false: the caller finishes the arg max itself (n_part partials per row are returned)
// plain_rows = true: the last LayerNorm runs as a launch of its own, so the rows the output
// projection multiplies are in memory (xa) for whoever multiplies them again
// embedded = true: the rows are embedded already (x, xa)
static int verify_forward(ad_ctx* c, int M, hipEvent_t ev_a = nullptr, hipEvent_t ev_b = nullptr, bool finish = true,
                          bool plain_rows = false, bool embedded = false, const PartialBuf* pb = nullptr) {
  const Plan& p = c->plan;
  const ModelW& w = c->w[AD_VERIFIER];
  if (embedded) c->ln_pending = nullptr;
  else embed_rows(c, w, M);
  for (int l = 0; l < c->cfg.dec_layers; ++l) {
    const DecLayerW& L = w.dec[l];
    self_attn_block(c, L.self, L.ln1, M, c->ws + p.cache_k + l * p.cache_layer_stride,
                    c->ws + p.cache_v + l * p.cache_layer_stride, p.l_cap);
    cross_attn_block(c, L.cross, L.ln2, M, c->ws + p.mem_k[0] + l * p.mem_layer_stride,
                     c->ws + p.mem_v[0] + l * p.mem_layer_stride);
    ffn_block(c, L.ffn, L.ln3, M);
  }
  if (plain_rows) flush_ln(c, M);
  if (ev_a) (void)hipEventRecord(ev_a, c->stream);
  c->ln_vocab = c->ln_pending;
  c->ln_pending = nullptr;
  const int n_part = vocab_argmax(c, w, c->at<void>(p.xa), M, c->ln_vocab, nullptr, pb);
  if (ev_b) (void)hipEventRecord(ev_b, c->stream);
  if (finish) vocab_finish(c, M, n_part, pb);
  return n_part;
}

static int check_batch(ad_ctx* c, const int32_t* src, const int32_t* src_len, int B) {
  if (!c) return fail(nullptr, AD_EINVAL, "null context");
  if (!src || !src_len) return fail(c, AD_EINVAL, "null source buffer");
  if (B < 1 || B > c->cfg.max_batch) return fail(c, AD_EINVAL, "B outside [1, max_batch]");
  for (int b = 0; b < B; ++b) {
    if (src_len[b] < 1 || src_len[b] > c->cfg.max_src) return fail(c, AD_EINVAL, "src_len outside [1, max_src]");
    for (int i = 0; i < src_len[b]; ++i) {
      int32_t t = src[(size_t)b * c->cfg.max_src + i];
      if (t < 0 || t >= c->cfg.vocab) return fail(c, AD_EINVAL, "source token id outside the vocabulary");
    }
  }
  return AD_OK;
}

// Device-backed verifier for the host loops.
struct GpuBackend : Backend {
  ad_ctx* c;
  explicit GpuBackend(ad_ctx* ctx) : c(ctx) {}
  int verify(const int32_t* draft, const int32_t* k, int32_t* n_accept, int32_t* next) override {
    return ad_verify(c, draft, k, n_accept, next, nullptr);
  }
  int draft(int k, int32_t* out) override { return ad_draft_nat(c, k, out); }
};

static LoopIO make_io(ad_ctx* c, int B, const int32_t* max_out) {
  LoopIO io;
  io.B = B; io.k_max = c->cfg.k_max; io.eos = c->cfg.eos; io.bos = c->cfg.bos;
  io.max_out.resize(B);
  for (int b = 0; b < B; ++b) io.max_out[b] = max_out ? max_out[b] : c->cfg.max_len;
  return io;
}
static void write_out(ad_ctx* c, const LoopIO& io, int32_t* out, int32_t* out_len, ad_stats* stats, double t_enc) {
  for (int b = 0; b < io.B; ++b) {
    out_len[b] = (int)io.o[b].size() - 1;
    for (int i = 0; i < out_len[b]; ++i) out[(size_t)b * c->cfg.max_len + i] = io.o[b][i + 1];
  }
  if (stats) { *stats = io.stats; stats->t_encode_us = t_enc; }
}

// =================================================================================================
extern "C" {

const char* ad_last_error(const ad_ctx* ctx) { return ctx ? ctx->err : ad::global_error(); }

size_t ad_workspace_bytes(const ad_config* cfg, int with_drafter) {
  if (ad_config_check(cfg) != AD_OK) return 0;
  return make_plan(*cfg, with_drafter != 0).total;
}

int ad_create(const ad_config* cfg, const void* verifier_w, const void* drafter_w, void* workspace,
              size_t workspace_bytes, void* hip_stream, ad_ctx** out) {
  if (!out) return fail(nullptr, AD_EINVAL, "null out pointer");
  *out = nullptr;
  int rc = ad_config_check(cfg);
  if (rc != AD_OK) return rc;
  if (!verifier_w || !workspace) return fail(nullptr, AD_EINVAL, "null verifier weights or workspace");
  if (((uintptr_t)verifier_w | (uintptr_t)drafter_w | (uintptr_t)workspace) & 255)
    return fail(nullptr, AD_EINVAL, "device pointers must be 256-byte aligned");
  Plan plan = make_plan(*cfg, drafter_w != nullptr);
  if (workspace_bytes < plan.total) return fail(nullptr, AD_ENOMEM, "workspace smaller than ad_workspace_bytes()");
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return fail(nullptr, AD_EDEVICE, "no HIP device");
  ad_ctx* c = new ad_ctx();
  c->cfg = *cfg;
  c->plan = plan;
  c->ws = (char*)workspace;
  c->stream = (hipStream_t)hip_stream;
  c->w[0] = bind_weights(*cfg, verifier_w);
  c->has_drafter = drafter_w != nullptr;
  if (c->has_drafter) c->w[1] = bind_weights(*cfg, drafter_w);
  const size_t B = cfg->max_batch;
  c->pl = make_pin_layout(*cfg, plan);
  c->last_k.assign(B, 0);
  auto bail = [&](const char* what, hipError_t e) {
    if (c->pin) (void)hipHostFree(c->pin);
    for (hipEvent_t ev : {c->ev0, c->ev1, c->ev2, c->ev3, c->ev_up[0], c->ev_up[1], c->ev_fork, c->ev_enc2})
      if (ev) (void)hipEventDestroy(ev);
    if (c->stream2) (void)hipStreamDestroy(c->stream2);
    delete c;
    return fail_hip(nullptr, what, e);
  };
  hipError_t e;
  // mapped and coherent: the device reads words the host rewrites between graph replays and the
  // host watches words the device writes in mid-stream, neither side may keep a stale copy
  if ((e = hipHostMalloc((void**)&c->pin, c->pl.total * 4, hipHostMallocMapped | hipHostMallocCoherent)) != hipSuccess)
    return bail("hipHostMalloc", e);
  memset(c->pin, 0, c->pl.total * 4);
  // this device's copy of the static scratch array (ad_verify_static); looked up once per device
  c->scratch_dev = static_scratch_for_current_device();
  {
    void* dp = nullptr;
    if (hipHostGetDevicePointer(&dp, c->pin, 0) == hipSuccess) c->pin_dev = (int32_t*)dp;
    else (void)hipGetLastError();
  }
  if ((e = hipEventCreate(&c->ev0)) != hipSuccess) return bail("hipEventCreate", e);
  if ((e = hipEventCreate(&c->ev1)) != hipSuccess) return bail("hipEventCreate", e);
  if ((e = hipEventCreate(&c->ev2)) != hipSuccess) return bail("hipEventCreate", e);
  if ((e = hipEventCreate(&c->ev3)) != hipSuccess) return bail("hipEventCreate", e);
  for (int i = 0; i < 2; ++i)
    if ((e = hipEventCreateWithFlags(&c->ev_up[i], hipEventDisableTiming)) != hipSuccess) return bail("hipEventCreate", e);
  if (c->has_drafter && c->stream != nullptr) {
    // the drafter's encoder runs beside the verifier's (both are needed before the first draft and
    // neither depends on the other): a second stream at the default priority; if it cannot be had
    // the two encoders simply run one after the other on the context's stream
    if (hipStreamCreateWithFlags(&c->stream2, hipStreamNonBlocking) == hipSuccess &&
        hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) == hipSuccess &&
        hipEventCreateWithFlags(&c->ev_enc2, hipEventDisableTiming) == hipSuccess) {
      c->overlap_encoders = true;
    } else {
      (void)hipGetLastError();
    }
  }
  // sinusoidal positions: PE(p, 2i) = sin(p / 10000^(2i/d)), PE(p, 2i+1) = cos(same)
  {
    const int d = cfg->d_model;
    std::vector<float> pe((size_t)plan.max_pos * d);
    for (int i = 0; i < d / 2; ++i) {
      const double freq = pow(10000.0, -2.0 * i / d);
      for (int pos = 0; pos < plan.max_pos; ++pos) {
        pe[(size_t)pos * d + 2 * i] = (float)sin(pos * freq);
        pe[(size_t)pos * d + 2 * i + 1] = (float)cos(pos * freq);
      }
    }
    if ((e = hipMemcpyAsync(c->ws + plan.pe, pe.data(), pe.size() * 4, hipMemcpyHostToDevice, c->stream)) != hipSuccess)
      return bail("hipMemcpyAsync(pe)", e);
    if ((e = hipStreamSynchronize(c->stream)) != hipSuccess) return bail("hipStreamSynchronize", e);
  }
  // the memory key/value projections of all decoder layers, side by side: one product per encode
  for (int i = 0; i < (c->has_drafter ? 2 : 1); ++i) {
    const size_t d = cfg->d_model, wb = 2 * d * d * plan.esz;
    for (int l = 0; l < cfg->dec_layers; ++l) {
      const AttnW& a = c->w[i].dec[l].cross;
      if ((e = hipMemcpyAsync(c->ws + plan.kv_w[i] + l * wb, w_rows(c, a.wqkv, d, d), wb, hipMemcpyDeviceToDevice, c->stream)) != hipSuccess ||
          (e = hipMemcpyAsync(c->ws + plan.kv_b[i] + l * 2 * d * 4, a.bqkv + d, 2 * d * 4, hipMemcpyDeviceToDevice, c->stream)) != hipSuccess)
        return bail("hipMemcpyAsync(memory projections)", e);
    }
  }
  if ((e = hipStreamSynchronize(c->stream)) != hipSuccess) return bail("hipStreamSynchronize", e);
  c->h_len.assign(B, 0); c->h_finished.assign(B, 1); c->h_max_out.assign(B, 0);
  c->h_src_len[0].assign(B, 0); c->h_src_len[1].assign(B, 0);
  *out = c;
  return AD_OK;
}

int ad_destroy(ad_ctx* c) {
  if (!c) return AD_EINVAL;
  if (c->stream2) (void)hipStreamSynchronize(c->stream2);
  (void)hipStreamSynchronize(c->stream);
  if (c->pin) (void)hipHostFree(c->pin);
  for (auto& kv : c->graphs) (void)hipGraphExecDestroy(kv.second);
  for (hipEvent_t ev : {c->ev0, c->ev1, c->ev2, c->ev3, c->ev_up[0], c->ev_up[1], c->ev_fork, c->ev_enc2})
    if (ev) (void)hipEventDestroy(ev);
  if (c->stream2) (void)hipStreamDestroy(c->stream2);
  delete c;
  return AD_OK;
}

}  // extern "C"

// rows < 2^26, longest block < 2^14, sequences < 2^13, knob < 2^6 (the configuration check's
// capacities): disjoint bit fields, bits 62 and 63 left to the caller
static unsigned long long shape_key(int rows, int max_rows, int n_seq, int knob) {
  return (unsigned long long)rows | ((unsigned long long)max_rows << 26) | ((unsigned long long)n_seq << 40) |
         ((unsigned long long)knob << 53);
}
// Runs `launches` (kernel launches and device-to-device copies on the context's stream, nothing
// else) as a graph: replay if
// this call shape has one, capture + instantiate + launch on the shape's third appearance.
// false = nothing was launched, the caller launches eagerly.  Any failure switches graphs off
// for the context (a stream that cannot be captured, e.g. the null stream, is such a failure).
template <typename F>
static bool run_as_graph(ad_ctx* c, hipStream_t stream, unsigned long long shape, const F& launches,
                         unsigned long long more = 0) {
  if (!c->graphs_on) return false;
  const ad_ctx::GraphKey key(shape, more);
  auto it = c->graphs.find(key);
  if (it != c->graphs.end()) {
    if (hipGraphLaunch(it->second, stream) == hipSuccess) return true;
    (void)hipGetLastError();
    c->graphs_on = false;
    return false;
  }
  if (++c->graph_seen[key] < 3 || c->graphs.size() >= 512) return false;   // worth building once a shape keeps coming back
  if (hipStreamBeginCapture(stream, hipStreamCaptureModeThreadLocal) != hipSuccess) {
    (void)hipGetLastError();
    c->graphs_on = false;
    return false;
  }
  launches();
  hipGraph_t g = nullptr;
  hipGraphExec_t ge = nullptr;
  hipError_t e = hipStreamEndCapture(stream, &g);
  if (e == hipSuccess && g) e = hipGraphInstantiate(&ge, g, nullptr, nullptr, 0);
  if (g) (void)hipGraphDestroy(g);
  if (e != hipSuccess || !ge) {
    (void)hipGetLastError();
    c->graphs_on = false;
    return false;
  }
  c->graphs[key] = ge;
  if (hipGraphLaunch(ge, stream) == hipSuccess) return true;
  (void)hipGetLastError();
  c->graphs_on = false;
  return false;
}

extern "C" {

int ad_encode(ad_ctx* c, int model, const int32_t* src, const int32_t* src_len, int B, const int32_t* max_out) {
  int rc = check_batch(c, src, src_len, B);
  if (rc != AD_OK) return rc;
  if (model != AD_VERIFIER && model != AD_DRAFTER) return fail(c, AD_EINVAL, "model must be AD_VERIFIER or AD_DRAFTER");
  if (model == AD_DRAFTER && !c->has_drafter) return fail(c, AD_ESTATE, "context has no drafter weights");
  if (max_out)
    for (int b = 0; b < B; ++b)
      if (max_out[b] < 1 || max_out[b] > c->cfg.max_len) return fail(c, AD_EINVAL, "max_out outside [1, max_len]");
  const ad_config& cf = c->cfg;
  const Plan& p = c->plan;
  const int d = cf.d_model, S = cf.max_src;
  // The two encoders of a draft-then-verify decode side by side (their forwards are independent and
  // both are needed before the first draft): the verifier's encode marks the point of the
  // context's stream it starts at; the drafter's encode that follows runs on the library's second
  // stream, in the second activation block, behind that mark only (i.e. behind everything that
  // read the drafter's previous memory, not behind the verifier's encoder), and the first
  // ad_draft_nat makes the context's stream wait for it.
  struct SideGuard {   // the context's stream / activation block for the length of this call
    ad_ctx* c; hipStream_t main; bool on;
    ~SideGuard() { if (on) { c->stream = main; c->act_shift = 0; } }
  } side{c, c->stream, false};
  if (c->overlap_encoders && model == AD_VERIFIER) {
    HIP_TRY(c, hipEventRecord(c->ev_fork, c->stream));
    c->fork_recorded = true;
  } else if (c->overlap_encoders && model == AD_DRAFTER && c->fork_recorded) {
    HIP_TRY(c, hipStreamWaitEvent(c->stream2, c->ev_fork, 0));
    c->fork_recorded = false;
    side.on = true;
    c->stream = c->stream2;
    c->act_shift = p.act2_shift;
  }
  // src_len[B], max_out[B], src[B, max_src] go into a part of the staging buffer that no other
  // call writes (one part per model).  The device reads them there (mapped memory) or gets them by
  // one copy; either way the call returns without waiting (what follows on the stream is ordered
  // behind it), so only the next ad_encode of the same model has to make sure they have been read.
  int32_t* h = c->pin + c->pl.enc[model];
  const bool mapped = c->pin_dev != nullptr;
  if (c->up_pending[model]) {
    HIP_TRY(c, hipEventSynchronize(c->ev_up[model]));
    c->up_pending[model] = false;
  }
  int M = 0;
  for (int b = 0; b < B; ++b) {
    h[b] = src_len[b];
    h[B + b] = max_out ? max_out[b] : cf.max_len;
    M += src_len[b];
  }
  memcpy(h + 2 * B, src, (size_t)B * S * 4);
  int* dev = mapped ? c->pin_dev + (h - c->pin) : c->at<int>(p.src_dev);
  if (!mapped) {
    HIP_TRY(c, hipMemcpyAsync(dev, h, (size_t)(2 * B + B * S) * 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipEventRecord(c->ev_up[model], c->stream));
    c->up_pending[model] = true;
  }
  VerifyTables t = tables(c);
  c->fw_nseq = B;
  c->fw_max_rows = *std::max_element(src_len, src_len + B);
  // kernels and device-to-device copies of the encoder forward: replayed as a graph per call shape
  auto launches = [&]() {
    const ModelW& w = c->w[model];
    const bool ver = model == AD_VERIFIER;
    launch_assemble_embed_encoder(cf.dtype, dev + 2 * B, S, dev, dev + B, B, S, t, c->at<int>(p.src_len[model]),
                                  c->at<int>(p.max_out), ver ? c->at<int>(p.len) : nullptr, c->at<int>(p.pending),
                                  c->at<int>(p.finished), cf.bos, M, w.emb, c->at<float>(p.pe), d, sqrtf((float)d),
                                  c->at<float>(p.x), c->at<void>(p.xa), c->stream);
    c->ln_pending = nullptr;
    for (int l = 0; l < cf.enc_layers; ++l) {
      const EncLayerW& L = w.enc[l];
      // the sentence's own keys/values live in the packed temporaries: key row = packed row
      Epi e{};
      e.mode = EPI_QKV; e.d = d; e.bias = L.self.bqkv; e.out0 = c->at<void>(p.q);
      e.out1 = c->at<void>(p.tk); e.out2 = c->at<void>(p.tv); e.row_dst = t.row_dst;
      gemm_rows(c, L.self.wqkv, M, 3 * d, e);
      launch_attention(cf.dtype, c->at<void>(p.q), c->at<void>(p.tk), c->at<void>(p.tv), c->at<void>(p.att),
                       t.self_desc, B, c->fw_max_rows, cf.n_heads, d / cf.n_heads, c->fw_max_rows <= 64 ? 64 : S, c->stream);
      gemm_resid_ln(c, c->at<void>(p.att), L.self.wo, L.self.bo, M, d, d, L.ln1);
      ffn_block(c, L.ffn, L.ln2, M);
    }
    // cross-attention keys and values of every decoder layer: memory . [wk; wv]^T + [bk; bv], the
    // layers' matrices side by side (copied so at ad_create), the encoder's last LayerNorm applied
    // while the rows are staged
    {
      Epi e{};
      e.mode = EPI_KV; e.d = d; e.bias = c->at<float>(p.kv_b[model]);
      e.out1 = c->ws + p.mem_k[model]; e.out2 = c->ws + p.mem_v[model];
      e.layer_stride = p.mem_layer_stride;
      e.row_dst = t.row_dst2;
      gemm_rows(c, c->ws + p.kv_w[model], M, cf.dec_layers * 2 * d, e);
    }
  };
  const unsigned long long key = (1ull << 63) | ((unsigned long long)model << 62) | shape_key(M, c->fw_max_rows, B, side.on ? 1 : 0);
  if (!run_as_graph(c, c->stream, key, launches)) launches();
  if (side.on) {
    HIP_TRY(c, hipEventRecord(c->ev_enc2, c->stream));
    c->enc2_pending = true;
  }
  if (mapped) {
    HIP_TRY(c, hipEventRecord(c->ev_up[model], c->stream));
    c->up_pending[model] = true;
  }
  HIP_TRY(c, hipGetLastError());
  c->h_src_len[model].assign(src_len, src_len + B);
  c->encoded[model] = true;
  if (model == AD_VERIFIER) {
    c->B = B;
    for (int b = 0; b < B; ++b) {
      c->h_len[b] = 0; c->h_finished[b] = 0; c->h_max_out[b] = max_out ? max_out[b] : cf.max_len;
    }
    c->encoded[AD_DRAFTER] = false;   // a new decode needs a fresh drafter memory
    c->last_M = 0;
  }
  return AD_OK;
}

}  // extern "C"

// What a verify call's launches need beyond the context: where the device reads k and the draft,
// where the acceptance kernel puts the result, whether it posts the call's ticket, and where the
// arg-max partials of the output projection live (the workspace's, or the static scratch array).
struct VerifyLaunch {
  const int* k_src;
  const int* draft_src;
  const int* rows_src;               // the packed row list (device view of the staging buffer), null: the kernel finds the rows from k
  int rows_stride;
  int* result_dst;
  const int* ticket_in;              // device view, null: no ticket
  unsigned long long* ticket_out;    // device view
  float* part_val;
  int* part_idx;
  int part_stride;
  int M, B;
};
// The launches of one verify call: row assembly + embedding, the forward, arg-max finish + acceptance.
static void verify_launches(ad_ctx* c, const VerifyLaunch& v) {
  const ad_config& cf = c->cfg;
  const Plan& p = c->plan;
  const int km = cf.k_max;
  VerifyTables t = tables(c);
  const bool gadpp = c->gadpp_beta > 1;
  auto accept = [&](const float* pv, const int* pi, int stride, int n_part, const GadppIn& gp) {
    launch_argmax_accept(pv, pi, stride, n_part, c->at<int>(p.o_hat), c->at<float>(p.o_val), v.k_src, v.draft_src, km,
                         t.row_start, v.B, cf.eos, cf.max_len, c->at<int>(p.max_out), c->at<int>(p.len),
                         c->at<int>(p.pending), c->at<int>(p.finished), c->at<int>(p.out), v.result_dst, v.ticket_in,
                         v.ticket_out, c->fw_max_rows, v.M, c->stream, gp);
  };
  launch_assemble_embed_verify(cf.dtype, v.k_src, v.draft_src, v.rows_src, v.rows_stride, km, c->at<int>(p.len), c->at<int>(p.pending),
                               c->at<int>(p.src_len[0]), v.B, p.l_cap, cf.max_src, t, v.M, c->w[AD_VERIFIER].emb,
                               c->at<float>(p.pe), cf.d_model, sqrtf((float)cf.d_model), c->at<float>(p.x),
                               c->at<void>(p.xa), c->stream);
  PartialBuf pb{v.part_val, v.part_idx, v.part_stride};
  if (!gadpp) {
    const int n_part = verify_forward(c, v.M, nullptr, nullptr, false, false, true, &pb);
    accept(v.part_val, v.part_idx, v.part_stride, n_part, GadppIn{});
    return;
  }
  // GAD++ (Section 3.2.3): arg max as before; then the score of every row's drafted token,
  // a second pass of the output projection that counts the columns scoring above it (the
  // logits still never reach memory), the relaxed replacement of o_hat, and acceptance
  const ModelW& w = c->w[AD_VERIFIER];
  (void)verify_forward(c, v.M, nullptr, nullptr, true, true, true, &pb);
  launch_draft_logit(cf.dtype, c->at<void>(p.xa), w.out_w, v.M, cf.vocab, cf.d_model, t.row_seq, t.row_start,
                     v.draft_src, km, c->at<float>(p.draft_lp), c->at<int>(p.draft_col), c->stream);
  Epi e{};
  e.mode = EPI_COUNT; e.part_idx = v.part_idx; e.n_strips = v.part_stride; e.thr = c->at<float>(p.draft_lp);
  const int n_cnt = launch_gemm(cf.dtype, c->at<void>(p.xa), w.out_w, v.M, cf.vocab, cf.d_model, e, c->stream);
  // (the relaxed replacement of o_hat happens inside the acceptance kernel)
  GadppIn gp;
  gp.part_cnt = v.part_idx; gp.stride = v.part_stride; gp.n_part = n_cnt;
  gp.lp = c->at<float>(p.draft_lp); gp.col = c->at<int>(p.draft_col);
  gp.beta = c->gadpp_beta; gp.tau = c->gadpp_tau;
  accept(c->at<float>(p.o_val), c->at<int>(p.o_hat), 1, 1, gp);
}

// ad_verify and its no-allocation variant.  static_scratch: the arg-max partials go to the
// library's static device array, every launch is made eagerly (no graph is built or replayed) and
// nothing on the way allocates.
static int verify_call(ad_ctx* c, const int32_t* draft, const int32_t* k, int32_t* n_accept, int32_t* next_token,
                       int32_t* verified, bool static_scratch) {
  if (!c) return fail(nullptr, AD_EINVAL, "null context");
  if (!draft || !k || !n_accept || !next_token) return fail(c, AD_EINVAL, "null buffer");
  if (!c->encoded[AD_VERIFIER]) return fail(c, AD_ESTATE, "ad_verify before ad_encode(AD_VERIFIER)");
  const ad_config& cf = c->cfg;
  const Plan& p = c->plan;
  const PinLayout& pl = c->pl;
  const int B = c->B, km = cf.k_max;
  int M = 0, max_rows = 0;
  for (int b = 0; b < B; ++b) {
    if (k[b] < 0 || k[b] > km) return fail(c, AD_EINVAL, "k[b] outside [0, k_max]");
    if (k[b] && c->h_finished[b]) return fail(c, AD_ESTATE, "k[b] > 0 for a finished sequence");
    for (int i = 0; i < k[b]; ++i) {
      int32_t t = draft[(size_t)b * km + i];
      if (t == AD_NEVER ? i != k[b] - 1 : (t < 0 || t >= cf.vocab))
        return fail(c, AD_EINVAL, "draft id outside the vocabulary (AD_NEVER is allowed last only)");
    }
    M += k[b];
    max_rows = std::max(max_rows, (int)k[b]);
  }
  if (static_scratch) {
    if (!c->scratch_dev) return fail(c, AD_ESTATE, "the static scratch array is unavailable on this device");
    if ((size_t)M * p.n_strips * 8 > kStaticScratchBytes)
      return fail(c, AD_EINVAL, "ad_verify_static: rows x (vocab / 16) x 8 bytes exceed the static scratch array (4 MiB)");
  }
  if (M == 0) {
    for (int b = 0; b < B; ++b) { n_accept[b] = 0; next_token[b] = 0; }
    return AD_OK;
  }
  int32_t* h = c->pin;
  memcpy(h + pl.k, k, (size_t)B * 4);
  for (int b = 0; b < B; ++b) memcpy(h + pl.draft + (size_t)b * km, draft + (size_t)b * km, (size_t)km * 4);
  // The two small kernels that need k and the draft read them where they are, in the pinned
  // (device-visible) staging buffer, and the result is written there too: no copy operations
  // around the forward.
  const bool mapped = c->pin_dev != nullptr;
  VerifyLaunch v{};
  v.M = M; v.B = B;
  if (mapped) {
    v.k_src = c->pin_dev + pl.k; v.draft_src = c->pin_dev + pl.draft; v.result_dst = c->pin_dev + pl.result;
    // with several sequences also the list of packed rows, so that the row's workgroup needs one trip over the bus
    // (its own entry) instead of two (the counts, then its token)
    if (B > 1) {
      int32_t* rows = h + pl.rows;
      const size_t cap = p.mv_cap;
      int m = 0;
      for (int b = 0; b < B; ++b)
        for (int i = 0; i < k[b]; ++i, ++m) {
          rows[m] = (b << 14) | i;
          rows[cap + m] = i == 0 ? -1 : draft[(size_t)b * km + i - 1];
        }
      v.rows_src = c->pin_dev + pl.rows;
      v.rows_stride = (int)cap;
    }
  } else {
    HIP_TRY(c, hipMemcpyAsync(c->at<int>(p.k_dev), h + pl.k, (size_t)B * 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->at<int>(p.draft_dev), h + pl.draft, (size_t)B * km * 4, hipMemcpyHostToDevice, c->stream));
    v.k_src = c->at<int>(p.k_dev); v.draft_src = c->at<int>(p.draft_dev); v.result_dst = c->at<int>(p.result);
  }
  if (static_scratch) {
    v.part_val = (float*)c->scratch_dev;
    v.part_idx = (int*)((char*)c->scratch_dev + kStaticScratchBytes / 2);
  } else {
    v.part_val = c->at<float>(p.part_val);
    v.part_idx = c->at<int>(p.part_idx);
  }
  v.part_stride = p.n_strips;
  c->fw_nseq = B;
  c->fw_max_rows = max_rows;
  int self_keys = 0;
  for (int b = 0; b < B; ++b)
    if (k[b] > 0) self_keys = std::max(self_keys, c->h_len[b] + (int)k[b]);
  c->fw_self_keys = self_keys;
  const int cross_keys = *std::max_element(c->h_src_len[AD_VERIFIER].begin(), c->h_src_len[AD_VERIFIER].begin() + B);
  c->fw_cross_keys = cross_keys;
  c->last_nseq = B; c->last_max_rows = max_rows; c->last_self_keys = self_keys; c->last_cross_keys = cross_keys;
  // The result lands in host memory the device writes directly, as ONE 8-byte word per sequence that
  // carries the call's ticket, and the host watches for the ticket instead of waiting for the
  // stream to drain (the end of the kernel, its completion signal and the runtime's wake-up are off
  // the critical path).
  int32_t* ticket_in = c->pin + pl.v_ticket;
  unsigned long long* ticket_out = (unsigned long long*)(c->pin + pl.v_slots);
  const bool watch = mapped && c->spin_wait && !verified;
  if (watch) {
    if (++c->ticket >= (1 << 18)) c->ticket = 1;
    *ticket_in = c->ticket;
    for (int b = 0; b < B; ++b) ticket_out[b] = 0;   // whatever an earlier call left in these words
    v.ticket_in = c->pin_dev + pl.v_ticket;
    v.ticket_out = (unsigned long long*)(c->pin_dev + pl.v_slots);
  }
  // every launch argument is a function of (rows, sequences, longest block), of the GAD++
  // setting, of whether the acceptance kernel posts the ticket, and of pointers fixed for the
  // context's life
  const bool gadpp = c->gadpp_beta > 1;
  bool launched = false;
  if (mapped && !static_scratch) {
    const unsigned long long key = shape_key(M, max_rows, B, (gadpp ? 1 : 0) | (watch ? 2 : 0) | (c->fuse_crossq ? 4 : 0) | (self_keys <= 64 ? 8 : 0) | (cross_keys <= 64 ? 16 : 0));
    unsigned tau_bits;
    memcpy(&tau_bits, &c->gadpp_tau, 4);
    const unsigned long long more = gadpp ? ((unsigned long long)c->gadpp_beta << 32) | tau_bits : 0;
    launched = run_as_graph(c, c->stream, key, [&]() { verify_launches(c, v); }, more);
  }
  if (!launched) verify_launches(c, v);
  int32_t* res = c->pin + pl.result;
  int32_t* oh = c->pin + pl.o_hat;
  if (!mapped) HIP_TRY(c, hipMemcpyAsync(res, c->at<int>(p.result), (size_t)B * 8, hipMemcpyDeviceToHost, c->stream));
  if (verified) HIP_TRY(c, hipMemcpyAsync(oh, c->at<int>(p.o_hat), (size_t)M * 4, hipMemcpyDeviceToHost, c->stream));
  bool seen = false;
  if (watch) {
    const int want = c->ticket;
    const auto t_end = std::chrono::steady_clock::now() + std::chrono::milliseconds(50);
    for (unsigned spin = 1;; ++spin) {
      int b = 0;
      while (b < B && (int)(__atomic_load_n(ticket_out + b, __ATOMIC_ACQUIRE) >> 46) == want) ++b;
      if (b == B) { seen = true; break; }
      if ((spin & 1023u) == 0 && std::chrono::steady_clock::now() > t_end) break;   // fall back to the stream
      __builtin_ia32_pause();
    }
  }
  if (!seen) {
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    HIP_TRY(c, hipGetLastError());
  }
  int r0 = 0;
  for (int b = 0; b < B; ++b) {
    if (watch) {
      // (after the fall-back to the stream the words are there as well: the kernel has finished)
      const unsigned long long w = __atomic_load_n(ticket_out + b, __ATOMIC_ACQUIRE);
      n_accept[b] = (int)((w >> 32) & 0x3fff);
      next_token[b] = (int)(unsigned)w;
    } else {
      n_accept[b] = res[2 * b];
      next_token[b] = res[2 * b + 1];
    }
    if (k[b]) {
      c->h_len[b] += n_accept[b];
      c->h_finished[b] = (n_accept[b] > 0 && next_token[b] == cf.eos) || c->h_len[b] >= c->h_max_out[b];
    }
    if (verified) {
      for (int i = 0; i < km; ++i) verified[(size_t)b * km + i] = i < k[b] ? oh[r0 + i] : AD_NEVER;
    }
    c->last_k[b] = k[b];
    r0 += k[b];
  }
  c->last_M = M;
  c->last_logit_rows = M;
  return AD_OK;
}

extern "C" {

int ad_verify(ad_ctx* c, const int32_t* draft, const int32_t* k, int32_t* n_accept, int32_t* next_token,
              int32_t* verified) {
  return verify_call(c, draft, k, n_accept, next_token, verified, false);
}

int ad_verify_static(ad_ctx* c, const int32_t* draft, const int32_t* k, int32_t* n_accept, int32_t* next_token,
                     int32_t* verified) {
  return verify_call(c, draft, k, n_accept, next_token, verified, true);
}

int ad_draft_nat(ad_ctx* c, int k, int32_t* draft_out) {
  if (!c) return fail(nullptr, AD_EINVAL, "null context");
  if (!draft_out) return fail(c, AD_EINVAL, "null buffer");
  if (!c->has_drafter) return fail(c, AD_ESTATE, "context has no drafter weights");
  if (!c->encoded[AD_VERIFIER] || !c->encoded[AD_DRAFTER])
    return fail(c, AD_ESTATE, "ad_draft_nat needs ad_encode for both models (verifier first)");
  const ad_config& cf = c->cfg;
  const Plan& p = c->plan;
  if (k < 1 || k > cf.k_max) return fail(c, AD_EINVAL, "k outside [1, k_max]");
  const int B = c->B, km = cf.k_max;
  if (c->enc2_pending) {
    // the drafter's memory comes from the second stream
    HIP_TRY(c, hipStreamWaitEvent(c->stream, c->ev_enc2, 0));
    c->enc2_pending = false;
  }
  int M = 0, live = 0;
  for (int b = 0; b < B; ++b)
    if (!c->h_finished[b]) { M += c->h_len[b] + 1 + k; ++live; }
  if (live == 0) {
    for (size_t i = 0; i < (size_t)B * km; ++i) draft_out[i] = AD_NEVER;
    return AD_OK;
  }
  VerifyTables t = tables(c);
  int max_rows = k, self_keys = 0;
  for (int b = 0; b < B; ++b)
    if (!c->h_finished[b]) {
      max_rows = std::max(max_rows, c->h_len[b] + 1);
      self_keys = std::max(self_keys, c->h_len[b] + 1 + k);   // every row of a sequence sees its prefix and the k masks
    }
  const int Mv = live * k;
  int32_t* h = c->pin + c->pl.d_copy;
  unsigned long long* slots = (unsigned long long*)(c->pin + c->pl.d_slots);   // [B, k_max]
  int32_t* ticket_in = c->pin + c->pl.d_ticket;
  const bool watch = c->pin_dev != nullptr && c->spin_wait;
  // the drafter forward's launches (made one by one: the prefix is recomputed every iteration,
  // so a call shape seldom comes back and a graph per shape costs more to build than it saves).
  // The mask rows are the first Mv packed rows; two attention problems per sequence (mask rows and
  // prefix rows as queries).  In the last layer only the mask rows go on after the key/value
  // projection: nothing reads the prefix rows' outputs.
  auto launches = [&]() {
    const ModelW& w = c->w[AD_DRAFTER];
    c->ln_pending = nullptr;
    launch_assemble_embed_drafter(cf.dtype, c->at<int>(p.out), cf.max_len, c->at<int>(p.len), c->at<int>(p.finished),
                                  c->at<int>(p.src_len[1]), B, k, cf.bos, cf.mask, cf.max_src, t, M, w.emb,
                                  c->at<float>(p.pe), cf.d_model, sqrtf((float)cf.d_model), c->at<float>(p.x),
                                  c->at<void>(p.xa), c->stream);
    int rows = M;
    c->fw_nseq = 2 * live;
    c->fw_max_rows = max_rows;
    c->fw_self_keys = self_keys;
    c->fw_cross_keys = *std::max_element(c->h_src_len[AD_DRAFTER].begin(), c->h_src_len[AD_DRAFTER].begin() + B);
    for (int l = 0; l < cf.dec_layers; ++l) {
      const DecLayerW& L = w.dec[l];
      if (l + 1 == cf.dec_layers) {
        self_attn_block(c, L.self, L.ln1, M, c->at<void>(p.tk), c->at<void>(p.tv), cf.max_len + km, Mv, live, k);
        rows = Mv;
      } else {
        self_attn_block(c, L.self, L.ln1, M, c->at<void>(p.tk), c->at<void>(p.tv), cf.max_len + km);
      }
      cross_attn_block(c, L.cross, L.ln2, rows, c->ws + p.mem_k[1] + l * p.mem_layer_stride,
                       c->ws + p.mem_v[1] + l * p.mem_layer_stride);
      ffn_block(c, L.ffn, L.ln3, rows);
    }
    // the last LayerNorm goes into the output projection's staging, as in the verify forward
    const LnW* ln_last = c->ln_pending;
    c->ln_pending = nullptr;
    const int n_part = vocab_argmax(c, w, c->at<void>(p.xa), Mv, ln_last);
    if (watch) {
      // the drafted tokens go straight to the host: (ticket, token) per 8-byte slot of the mapped buffer
      launch_argmax_draft(c->at<float>(p.part_val), c->at<int>(p.part_idx), Mv, p.n_strips, n_part, c->at<int>(p.o_hat),
                          c->at<int>(p.finished), B, k, km, c->pin_dev + c->pl.d_ticket,
                          (unsigned long long*)(c->pin_dev + c->pl.d_slots), c->stream);
    } else {
      vocab_finish(c, Mv, n_part);
      launch_draft_scatter(c->at<int>(p.o_hat), c->at<int>(p.finished), B, k, km, c->at<int>(p.draft_out), c->stream);
    }
  };
  if (watch) {
    if (++c->ticket >= (1 << 18)) c->ticket = 1;
    *ticket_in = c->ticket;
    for (int b = 0; b < B; ++b)
      if (!c->h_finished[b])
        for (int i = 0; i < k; ++i) slots[(size_t)b * km + i] = 0;
  }
  launches();
  bool seen = false;
  if (watch) {
    // wait for the last slot of every live sequence first (it is written about when the others are),
    // then make sure of all of them
    const auto t_end = std::chrono::steady_clock::now() + std::chrono::milliseconds(50);
    seen = true;
    for (int b = 0; b < B && seen; ++b) {
      if (c->h_finished[b]) continue;
      for (int i = k - 1; i >= 0 && seen; --i)
        for (unsigned spin = 1; (int)(__atomic_load_n(slots + (size_t)b * km + i, __ATOMIC_ACQUIRE) >> 32) != c->ticket; ++spin) {
          if ((spin & 1023u) == 0 && std::chrono::steady_clock::now() > t_end) { seen = false; break; }
          __builtin_ia32_pause();
        }
    }
    if (seen) {
      for (int b = 0; b < B; ++b)
        for (int i = 0; i < km; ++i)
          draft_out[(size_t)b * km + i] = !c->h_finished[b] && i < k ? (int32_t)(unsigned)slots[(size_t)b * km + i] : AD_NEVER;
    } else {
      // fall back to the stream: the tokens are in o_hat; scatter them as the other path does
      launch_draft_scatter(c->at<int>(p.o_hat), c->at<int>(p.finished), B, k, km, c->at<int>(p.draft_out), c->stream);
    }
  }
  if (!seen) {
    HIP_TRY(c, hipMemcpyAsync(h, c->at<int>(p.draft_out), (size_t)B * km * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    HIP_TRY(c, hipGetLastError());
    memcpy(draft_out, h, (size_t)B * km * 4);
  }
  c->last_logit_rows = Mv;
  c->last_M = 0;   // the row tables now describe the drafter's rows
  return AD_OK;
}

int ad_output(ad_ctx* c, int32_t* out, int32_t* out_len) {
  if (!c) return fail(nullptr, AD_EINVAL, "null context");
  if (!out || !out_len) return fail(c, AD_EINVAL, "null buffer");
  if (!c->encoded[AD_VERIFIER]) return fail(c, AD_ESTATE, "no decode in progress");
  const int B = c->B, L = c->cfg.max_len;
  const int32_t* ho = c->pin + c->pl.out;
  HIP_TRY(c, hipMemcpyAsync(c->pin + c->pl.out, c->at<int>(c->plan.out), (size_t)B * L * 4, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  for (int b = 0; b < B; ++b) {
    out_len[b] = c->h_len[b];
    for (int i = 0; i < L; ++i) out[(size_t)b * L + i] = i < c->h_len[b] ? ho[(size_t)b * L + i] : c->cfg.pad;
  }
  return AD_OK;
}

// ---------------------------------------------------------------------------------------------
static int begin_decode(ad_ctx* c, const int32_t* src, const int32_t* src_len, int B, const int32_t* max_out,
                        bool drafter, double* t_enc) {
  double t0 = now_us();
  int rc = ad_encode(c, AD_VERIFIER, src, src_len, B, max_out);
  if (rc == AD_OK && drafter) rc = ad_encode(c, AD_DRAFTER, src, src_len, B, nullptr);
  *t_enc = now_us() - t0;
  return rc;
}

int ad_decode_greedy(ad_ctx* c, const int32_t* src, const int32_t* src_len, int B, const int32_t* max_out,
                     int32_t* out, int32_t* out_len, ad_stats* stats) {
  if (!c) return fail(nullptr, AD_EINVAL, "null context");
  if (!out || !out_len) return fail(c, AD_EINVAL, "null output buffer");
  double t_enc = 0;
  int rc = begin_decode(c, src, src_len, B, max_out, false, &t_enc);
  if (rc != AD_OK) return rc;
  LoopIO io = make_io(c, B, max_out);
  GpuBackend be(c);
  rc = loop_greedy(be, io);
  if (rc != AD_OK) return rc;
  write_out(c, io, out, out_len, stats, t_enc);
  return AD_OK;
}

int ad_decode_iad(ad_ctx* c, const int32_t* src, const int32_t* src_len, const int32_t* guide,
                  const int32_t* guide_len, int guide_stride, int B, const int32_t* max_out, int32_t* out,
                  int32_t* out_len, ad_stats* stats) {
  if (!c) return fail(nullptr, AD_EINVAL, "null context");
  if (!out || !out_len) return fail(c, AD_EINVAL, "null output buffer");
  if (guide && (!guide_len || guide_stride < 1)) return fail(c, AD_EINVAL, "guide without guide_len / stride");
  int rc = check_batch(c, src, src_len, B);
  if (rc != AD_OK) return rc;
  std::vector<std::vector<int32_t>> g(B);
  for (int b = 0; b < B; ++b) {
    const int32_t* row = guide ? guide + (size_t)b * guide_stride : src + (size_t)b * c->cfg.max_src;
    const int n = guide ? guide_len[b] : src_len[b];
    if (n < 0 || (guide && n > guide_stride)) return fail(c, AD_EINVAL, "guide_len outside [0, guide_stride]");
    for (int i = 0; i < n; ++i)
      if (row[i] < 0 || row[i] >= c->cfg.vocab) return fail(c, AD_EINVAL, "guide token id outside the vocabulary");
    g[b].assign(row, row + n);
  }
  double t_enc = 0;
  rc = begin_decode(c, src, src_len, B, max_out, false, &t_enc);
  if (rc != AD_OK) return rc;
  LoopIO io = make_io(c, B, max_out);
  GpuBackend be(c);
  rc = loop_iad(be, io, g);
  if (rc != AD_OK) return rc;
  write_out(c, io, out, out_len, stats, t_enc);
  return AD_OK;
}

int ad_decode_gad(ad_ctx* c, const int32_t* src, const int32_t* src_len, int B, int k, int use_drafter,
                  const int32_t* draft_override, const int32_t* override_len, int override_stride,
                  const int32_t* max_out, int32_t* out, int32_t* out_len, ad_stats* stats) {
  if (!c) return fail(nullptr, AD_EINVAL, "null context");
  if (!out || !out_len) return fail(c, AD_EINVAL, "null output buffer");
  if (k < 1 || k > c->cfg.k_max) return fail(c, AD_EINVAL, "k outside [1, k_max]");
  if (use_drafter && !c->has_drafter) return fail(c, AD_ESTATE, "context has no drafter weights");
  if (!use_drafter && !draft_override) return fail(c, AD_EINVAL, "need a drafter or a draft override");
  if (draft_override && (!override_len || override_stride < 1)) return fail(c, AD_EINVAL, "override without lengths");
  int rc = check_batch(c, src, src_len, B);
  if (rc != AD_OK) return rc;
  std::vector<std::vector<int32_t>> D(B);
  if (draft_override)
    for (int b = 0; b < B; ++b) {
      const int n = override_len[b];
      if (n < 0 || n > override_stride) return fail(c, AD_EINVAL, "override_len outside [0, override_stride]");
      const int32_t* row = draft_override + (size_t)b * override_stride;
      for (int i = 0; i < n; ++i)
        if (row[i] < 0 || row[i] >= c->cfg.vocab) return fail(c, AD_EINVAL, "override token id outside the vocabulary");
      D[b].assign(row, row + n);
    }
  double t_enc = 0;
  rc = begin_decode(c, src, src_len, B, max_out, use_drafter != 0, &t_enc);
  if (rc != AD_OK) return rc;
  LoopIO io = make_io(c, B, max_out);
  GpuBackend be(c);
  rc = loop_gad(be, io, k, use_drafter != 0, draft_override ? &D : nullptr);
  if (rc != AD_OK) return rc;
  write_out(c, io, out, out_len, stats, t_enc);
  return AD_OK;
}

int ad_set_gadpp(ad_ctx* c, int beta, float tau) {
  if (!c) return fail(nullptr, AD_EINVAL, "null context");
  if (beta < 1 || beta > c->cfg.vocab) return fail(c, AD_EINVAL, "beta outside [1, vocab]");
  if (!(tau >= 0.f) || tau > 3.0e38f) return fail(c, AD_EINVAL, "tau must be finite and >= 0");
  c->gadpp_beta = beta;
  c->gadpp_tau = tau;
  return AD_OK;
}

int ad_set_option(ad_ctx* c, int option, int value) {
  if (!c) return fail(nullptr, AD_EINVAL, "null context");
  if (option == AD_OPT_GRAPHS) {
    if (value != 0 && value != 1) return fail(c, AD_EINVAL, "AD_OPT_GRAPHS must be 0 or 1");
    c->graphs_on = value != 0;
    return AD_OK;
  }
  if (option == AD_OPT_SPIN_WAIT) {
    if (value != 0 && value != 1) return fail(c, AD_EINVAL, "AD_OPT_SPIN_WAIT must be 0 or 1");
    c->spin_wait = value != 0;
    return AD_OK;
  }
  if (option == AD_OPT_FUSE_CROSSQ) {
    if (value != 0 && value != 1) return fail(c, AD_EINVAL, "AD_OPT_FUSE_CROSSQ must be 0 or 1");
    c->fuse_crossq = value != 0;
    return AD_OK;
  }
  if (option == AD_OPT_OVERLAP_ENCODERS) {
    if (value != 0 && value != 1) return fail(c, AD_EINVAL, "AD_OPT_OVERLAP_ENCODERS must be 0 or 1");
    if (value && !c->stream2) return fail(c, AD_ESTATE, "no second stream (no drafter, or the context runs on the null stream)");
    c->overlap_encoders = value != 0;
    c->fork_recorded = false;
    return AD_OK;
  }
  return fail(c, AD_EINVAL, "unknown option");
}
int ad_get_option(ad_ctx* c, int option, int* value) {
  if (!c) return fail(nullptr, AD_EINVAL, "null context");
  if (!value) return fail(c, AD_EINVAL, "null pointer");
  if (option == AD_OPT_GRAPHS) *value = c->graphs_on ? 1 : 0;
  else if (option == AD_OPT_GRAPHS_CAPTURED) *value = (int)c->graphs.size();
  else if (option == AD_OPT_SPIN_WAIT) *value = c->spin_wait ? 1 : 0;
  else if (option == AD_OPT_FUSE_CROSSQ) *value = c->fuse_crossq ? 1 : 0;
  else if (option == AD_OPT_OVERLAP_ENCODERS) *value = c->overlap_encoders ? 1 : 0;
  else return fail(c, AD_EINVAL, "unknown option");
  return AD_OK;
}

int ad_debug_logits(ad_ctx* c, float* logits, int rows_cap, int* rows) {
  if (!c) return fail(nullptr, AD_EINVAL, "null context");
  if (!logits || !rows) return fail(c, AD_EINVAL, "null buffer");
  if (!c->cfg.debug_logits) return fail(c, AD_ESTATE, "context was created without debug_logits");
  if (c->last_logit_rows < 1) return fail(c, AD_ESTATE, "no forward has run yet");
  if (rows_cap < c->last_logit_rows) return fail(c, AD_EINVAL, "rows_cap too small");
  HIP_TRY(c, hipMemcpyAsync(logits, c->at<float>(c->plan.logits), (size_t)c->last_logit_rows * c->cfg.vocab * 4,
                            hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  *rows = c->last_logit_rows;
  return AD_OK;
}

int ad_calibration_copy(void* dst_dev, const void* src_dev, size_t bytes, void* stream) {
  if (!dst_dev || !src_dev || bytes % 16) return fail(nullptr, AD_EINVAL, "ad_calibration_copy: null pointer or size not a multiple of 16");
  if (launch_calibration_copy(dst_dev, src_dev, bytes, (hipStream_t)stream) != hipSuccess)
    return fail(nullptr, AD_EDEVICE, "ad_calibration_copy: launch failed");
  return AD_OK;
}

int ad_calibration_mfma(void* scratch_dev, size_t scratch_bytes, int iters, void* stream, double* tflops) {
  const int wgs = 512;   // two workgroups per CU on 256 CUs: two waves per SIMD
  if (!scratch_dev || !tflops || iters < 1 || scratch_bytes < (size_t)wgs * 256 * 4)
    return fail(nullptr, AD_EINVAL, "ad_calibration_mfma: null pointer, iters < 1 or scratch smaller than 512 KiB");
  hipStream_t s = (hipStream_t)stream;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  float ms = 0;
  bool ok = hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess &&
            launch_calibration_mfma((float*)scratch_dev, wgs, iters, s) == hipSuccess && hipEventRecord(e0, s) == hipSuccess &&
            launch_calibration_mfma((float*)scratch_dev, wgs, iters, s) == hipSuccess && hipEventRecord(e1, s) == hipSuccess &&
            hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (!ok || ms <= 0) { (void)hipGetLastError(); return fail(nullptr, AD_EDEVICE, "ad_calibration_mfma: launch or timing failed"); }
  *tflops = (double)wgs * 4 * iters * 8 * (2.0 * 16 * 16 * 32) / (ms * 1e-3) / 1e12;
  return AD_OK;
}

int ad_time_verify_forward(ad_ctx* c, int reps, double* forward_us, double* vocab_kernel_us,
                           double* vocab_back_to_back_us) {
  if (!c) return fail(nullptr, AD_EINVAL, "null context");
  if (reps < 1 || !forward_us || !vocab_kernel_us) return fail(c, AD_EINVAL, "bad argument");
  if (c->last_M < 1) return fail(c, AD_ESTATE, "the last forward was not an ad_verify");
  double tot = 0, voc = 0;
  c->fw_nseq = c->last_nseq; c->fw_max_rows = c->last_max_rows; c->fw_self_keys = c->last_self_keys; c->fw_cross_keys = c->last_cross_keys;
  verify_forward(c, c->last_M);   // warm
  // the whole forward, reps times back to back between two events
  HIP_TRY(c, hipEventRecord(c->ev0, c->stream));
  for (int r = 0; r < reps; ++r) verify_forward(c, c->last_M);
  HIP_TRY(c, hipEventRecord(c->ev3, c->stream));
  HIP_TRY(c, hipEventSynchronize(c->ev3));
  float a = 0, b = 0;
  HIP_TRY(c, hipEventElapsedTime(&a, c->ev0, c->ev3));
  tot = a * 1e3;
  // the output projection + arg max kernel: one launch at a time, bracketed by two events inside
  // a forward (the figure a kernel trace reports for it)
  for (int r = 0; r < reps; ++r) {
    verify_forward(c, c->last_M, c->ev1, c->ev2);
    HIP_TRY(c, hipEventSynchronize(c->ev2));
    HIP_TRY(c, hipEventElapsedTime(&b, c->ev1, c->ev2));
    voc += b * 1e3;
  }
  voc /= reps;
  tot /= reps;
  if (vocab_back_to_back_us) {
    // ... and reps launches back to back on the rows the forward left (launch overheads overlap)
    const ModelW& w = c->w[AD_VERIFIER];
    HIP_TRY(c, hipEventRecord(c->ev1, c->stream));
    for (int r = 0; r < reps; ++r) (void)vocab_argmax(c, w, c->at<void>(c->plan.xa), c->last_M, c->ln_vocab);
    HIP_TRY(c, hipEventRecord(c->ev2, c->stream));
    HIP_TRY(c, hipEventSynchronize(c->ev2));
    HIP_TRY(c, hipEventElapsedTime(&b, c->ev1, c->ev2));
    *vocab_back_to_back_us = b * 1e3 / reps;
  }
  HIP_TRY(c, hipGetLastError());
  *forward_us = tot;
  *vocab_kernel_us = voc;
  return AD_OK;
}

int ad_time_output_projection(ad_ctx* c, const void* w_copies, size_t copy_stride_bytes, int n_copies, int reps,
                              double* us_per_launch) {
  if (!c) return fail(nullptr, AD_EINVAL, "null context");
  if (!w_copies || n_copies < 1 || reps < 1 || !us_per_launch) return fail(c, AD_EINVAL, "bad argument");
  const size_t need = (size_t)c->cfg.vocab * c->cfg.d_model * (c->cfg.dtype == AD_BF16 ? 2 : 4);
  if (copy_stride_bytes < need || copy_stride_bytes % 16) return fail(c, AD_EINVAL, "copy stride smaller than the matrix or not a multiple of 16");
  if (c->last_M < 1) return fail(c, AD_ESTATE, "the last forward was not an ad_verify");
  c->fw_nseq = c->last_nseq; c->fw_max_rows = c->last_max_rows; c->fw_self_keys = c->last_self_keys; c->fw_cross_keys = c->last_cross_keys;
  verify_forward(c, c->last_M);   // the rows (and the pending LayerNorm) the projection works on
  const ModelW& w = c->w[AD_VERIFIER];
  auto copy = [&](int r) { return (const char*)w_copies + (size_t)(r % n_copies) * copy_stride_bytes; };
  for (int r = 0; r < n_copies; ++r) (void)vocab_argmax(c, w, c->at<void>(c->plan.xa), c->last_M, c->ln_vocab, copy(r));
  HIP_TRY(c, hipEventRecord(c->ev1, c->stream));
  for (int r = 0; r < reps; ++r) (void)vocab_argmax(c, w, c->at<void>(c->plan.xa), c->last_M, c->ln_vocab, copy(r));
  HIP_TRY(c, hipEventRecord(c->ev2, c->stream));
  HIP_TRY(c, hipEventSynchronize(c->ev2));
  float b = 0;
  HIP_TRY(c, hipEventElapsedTime(&b, c->ev1, c->ev2));
  HIP_TRY(c, hipGetLastError());
  *us_per_launch = b * 1e3 / reps;
  return AD_OK;
}

}  // extern "C"

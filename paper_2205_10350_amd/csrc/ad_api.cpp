// Context, workspace plan and the forward passes (encode, verify, draft) behind the C ABI.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <chrono>
#include <functional>
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
  size_t pe, x, s, xa, q, att, tk, tv, f, part_val, part_idx, o_hat, o_val, logits, draft_lp, draft_col;
  size_t cache_k, cache_v, cache_layer_stride;          // [NL][B*l_cap, d]
  size_t mem_k[2], mem_v[2], mem_layer_stride;          // per model: [NL][B*max_src, d]
  size_t row_tok, row_pos, row_seq, row_dst, row_dst2, row_start, self_desc, cross_desc;
  size_t len, pending, finished, max_out, src_len[2], out, result, k_dev, draft_dev, src_dev, draft_out;
  size_t stages, bar, stamps;   // fused forward: stage program, barrier words, optional stage clock stamps
  int stage_cap = 0;
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
  p.x = take(m * d * 4);
  p.s = take(m * d * 4);
  p.xa = take(m * d * p.esz);
  p.q = take(m * d * p.esz);
  p.att = take(m * d * p.esz);
  p.tk = take(m * d * p.esz);
  p.tv = take(m * d * p.esz);
  p.f = take(m * (size_t)c.d_ffn * p.esz);
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
  p.row_tok = take(m * 4); p.row_pos = take(m * 4); p.row_seq = take(m * 4); p.row_dst = take(m * 4); p.row_dst2 = take(m * 4);
  p.row_start = take((B + 1) * 4);
  p.self_desc = take(2 * B * sizeof(SeqDesc));    // the drafter has two per sequence (mask rows, prefix rows)
  p.cross_desc = take(2 * B * sizeof(SeqDesc));
  p.len = take(B * 4); p.pending = take(B * 4); p.finished = take(B * 4); p.max_out = take(B * 4);
  p.out = take(B * c.max_len * 4);
  p.result = take(B * 2 * 4 + 16);   // [B,2] results, then one int: the fused forward's abort flag copy
  p.stage_cap = 8 * c.dec_layers + 1;
  p.stages = take((size_t)p.stage_cap * sizeof(Stage));
  p.stamps = take((size_t)(8 * 64 + 64 + 4 * 64) * 8);   // stage clock stamps; also scratch for the placement probe
  p.bar = take(8 * (size_t)kBarWords);   // barrier words of the persistent forward
  p.k_dev = take(B * 4 + B * c.k_max * 4);   // k[B] followed by draft[B, k_max]: one upload
  p.draft_dev = p.k_dev + B * 4;
  p.src_dev = take(B * 4 * 2 + B * c.max_src * 4);   // src_len[B], max_out[B], src[B, max_src]: one upload
  p.draft_out = take(B * c.k_max * 4);
  p.total = off;
  return p;
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
  size_t pin_ints = 0;
  std::string err;
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
  // persistent fused forward (bf16)
  int fused_rows = 0;            // largest M it takes; 0 = off
  // LayerNorm deferred into the next GEMM's operand staging: s -> (x, xa) with these parameters
  const LnW* ln_pending = nullptr;
  const LnW* ln_vocab = nullptr;  // the one the last verify forward's output projection applied (timing)
  int ticket = 0;                 // number of the last ad_verify call that waited by watching memory
  bool spin_wait = true;
  bool fuse_crossq = true;   // cross-attention: query projection + attention as one launch (AD_OPT_FUSE_CROSSQ)
  int gadpp_beta = 1;             // GAD++ (Section 3.2.3): 1 = plain top-1 verification
  float gadpp_tau = 0.f;
  int fused_grid = 0, fused_stages = 0, fused_teams = 0;
  size_t fused_lds = 0;
  unsigned long long dev_base = 0, team_base[kMaxTeams] = {};
  bool last_fused = false;
  // One launch per stage: the launches of a verify call (row assembly, forward, acceptance) are
  // captured into a graph per call shape on the shape's third appearance and replayed after.
  bool graphs_on = true;
  typedef std::pair<unsigned long long, unsigned long long> GraphKey;   // (kind | shape, further shape values)
  std::map<GraphKey, hipGraphExec_t> graphs;
  std::map<GraphKey, int> graph_seen;
  std::vector<int> last_k;       // k[b] of the last verify call

  template <typename T> T* at(size_t off) const { return (T*)(ws + off); }
};

static int fail(ad_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg;
  set_global_error(msg.c_str());
  return code;
}
#define HIP_TRY(ctx, expr)                                                                      \
  do {                                                                                          \
    hipError_t e_ = (expr);                                                                     \
    if (e_ != hipSuccess) return fail(ctx, AD_EDEVICE, std::string(#expr ": ") + hipGetErrorString(e_)); \
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
  launch_attention(c->cfg.dtype, c->at<void>(p.q), Kl, Vl, c->at<void>(p.att), t.self_desc, c->fw_nseq, c->fw_max_rows,
                   H, d / H, max_keys, c->stream);
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
  if (c->fuse_crossq &&
      launch_crossq_attention(c->cfg.dtype, la, c->at<void>(p.xa), a.wqkv, a.bqkv, Km, Vm,
                              c->at<void>(p.att), t.cross_desc, c->fw_nseq, c->fw_max_rows, H, d / H, c->cfg.max_src,
                              c->stream)) {
    c->ln_pending = nullptr;
  } else {
    Epi e{};
    e.mode = EPI_STORE; e.bias = a.bqkv; e.out0 = c->at<void>(p.q);
    gemm_rows(c, a.wqkv, M, d, e);
    launch_attention(c->cfg.dtype, c->at<void>(p.q), Km, Vm, c->at<void>(p.att), t.cross_desc, c->fw_nseq,
                     c->fw_max_rows, H, d / H, c->cfg.max_src, c->stream);
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
                        const void* out_w = nullptr /* another copy of w.out_w (timing) */) {
  const Plan& p = c->plan;
  Epi e{};
  e.mode = EPI_ARGMAX; e.part_val = c->at<float>(p.part_val); e.part_idx = c->at<int>(p.part_idx);
  e.n_strips = p.n_strips; e.logits = c->cfg.debug_logits ? c->at<float>(p.logits) : nullptr;
  LnA ln{};
  if (ln_of_s) { ln.x = c->at<float>(p.s); ln.g = ln_of_s->g; ln.b = ln_of_s->b; ln.y = c->at<float>(p.x); }
  return launch_gemm(c->cfg.dtype, A, out_w ? out_w : w.out_w, Mv, c->cfg.vocab, c->cfg.d_model, e, c->stream, ln);
}
static void vocab_finish(ad_ctx* c, int Mv, int n_part) {
  const Plan& p = c->plan;
  launch_argmax_finish(c->at<float>(p.part_val), c->at<int>(p.part_idx), Mv, p.n_strips, n_part, c->at<int>(p.o_hat),
                       c->at<float>(p.o_val), c->stream);
}

// Layer-phase stage program of the verify forward for the persistent kernel (pointers are fixed
// for the life of the context; only the row tables' contents, the team shares, M and B change
// per call).  The output projection, its arg max and acceptance are fixed parts of the kernel.
static int build_verify_program(ad_ctx* c, std::vector<Stage>& prog) {
  const Plan& p = c->plan;
  const ad_config& cf = c->cfg;
  const ModelW& w = c->w[AD_VERIFIER];
  const int d = cf.d_model, F = cf.d_ffn;
  VerifyTables t = tables(c);
  auto gemm = [&](int a_mode, const void* a_src, const LnW* ln, const void* W, int N, int K, Epi e) {
    Stage s{};
    s.type = ST_GEMM; s.a_mode = a_mode; s.N = N; s.K = K; s.W = W; s.a_src = a_src;
    if (ln) { s.ln_g = ln->g; s.ln_b = ln->b; }
    s.x_out = (a_mode == A_LN || a_mode == A_EMBED) ? c->at<float>(p.x) : nullptr;
    s.epi = e;
    prog.push_back(s);
  };
  auto attn = [&](const void* K, const void* V, const SeqDesc* desc, int nk_cap) {
    Stage s{};
    s.type = ST_ATTN; s.q = c->at<void>(p.q); s.Kb = K; s.Vb = V; s.att_out = c->at<void>(p.att); s.desc = desc;
    s.nk_cap = nk_cap;
    prog.push_back(s);
  };
  auto resid = [&](const float* bias) {
    Epi e{};
    e.mode = EPI_RESID; e.bias = bias; e.out0 = c->at<float>(p.s); e.resid = c->at<float>(p.x);
    return e;
  };
  for (int l = 0; l < cf.dec_layers; ++l) {
    const DecLayerW& L = w.dec[l];
    Epi e{};
    e.mode = EPI_QKV; e.d = d; e.bias = L.self.bqkv; e.out0 = c->at<void>(p.q);
    e.out1 = c->ws + p.cache_k + l * p.cache_layer_stride; e.out2 = c->ws + p.cache_v + l * p.cache_layer_stride;
    e.row_dst = t.row_dst;
    if (l == 0) gemm(A_EMBED, w.emb, nullptr, L.self.wqkv, 3 * d, d, e);
    else gemm(A_LN, c->at<float>(p.s), &w.dec[l - 1].ln3, L.self.wqkv, 3 * d, d, e);
    attn(e.out1, e.out2, t.self_desc, p.l_cap);
    gemm(A_COPY, c->at<void>(p.att), nullptr, L.self.wo, d, d, resid(L.self.bo));
    Epi q{};
    q.mode = EPI_STORE; q.bias = L.cross.bqkv; q.out0 = c->at<void>(p.q);
    gemm(A_LN, c->at<float>(p.s), &L.ln1, L.cross.wqkv, d, d, q);
    attn(c->ws + p.mem_k[0] + l * p.mem_layer_stride, c->ws + p.mem_v[0] + l * p.mem_layer_stride, t.cross_desc,
         cf.max_src);
    gemm(A_COPY, c->at<void>(p.att), nullptr, L.cross.wo, d, d, resid(L.cross.bo));
    Epi r{};
    r.mode = EPI_RELU; r.bias = L.ffn.b1; r.out0 = c->at<void>(p.f);
    gemm(A_LN, c->at<float>(p.s), &L.ln2, L.ffn.w1, F, d, r);
    gemm(A_COPY, c->at<void>(p.f), nullptr, L.ffn.w2, d, F, resid(L.ffn.b2));
  }
  // every GEMM stage prefetches the next GEMM stage's weights; the last one the output projection's
  for (size_t i = 0; i < prog.size(); ++i) {
    prog[i].pf_stage = -1;
    if (prog[i].type != ST_GEMM) continue;
    prog[i].pf_stage = -2;
    for (size_t j = i + 1; j < prog.size(); ++j)
      if (prog[j].type == ST_GEMM) { prog[i].pf_stage = (int)j; break; }
  }
  Stage ln{};
  ln.pf_stage = -1;
  ln.type = ST_LN; ln.K = d; ln.a_src = c->at<float>(p.s);
  ln.ln_g = w.dec[cf.dec_layers - 1].ln3.g; ln.ln_b = w.dec[cf.dec_layers - 1].ln3.b;
  ln.epi.out0 = c->at<void>(p.xa);
  prog.push_back(ln);
  return (int)prog.size();
}

// Sets the persistent forward up if this context and device can run it; otherwise leaves it off.
static void setup_fused(ad_ctx* c) {
  c->fused_rows = 0;
  c->fused_grid = 0;
  if (c->cfg.dtype != AD_BF16) return;
  const ad_config& cf = c->cfg;
  const Plan& p = c->plan;
  const int d = cf.d_model, F = cf.d_ffn;
  // LayerNorm rows and A tiles are at most kFusedMaxWidth wide; wider GEMMs walk whole slices
  if (d > kFusedMaxWidth || d % 32 || F % 32 || (F > kFusedMaxWidth && F % kFusedMaxWidth)) return;
  const int dh_f = d / cf.n_heads;
  if (dh_f != 16 && dh_f != 32 && dh_f != 64) return;   // the head widths the persistent kernel is built for
  const size_t att_bytes = attn_lds_host(std::max(p.l_cap, cf.max_src), d / cf.n_heads, 2, kFusedWaves);
  const size_t lds = kFusedLdsBytes;
  if (att_bytes > lds || (size_t)cf.k_max * 4 > lds) return;
  hipDeviceProp_t prop;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) { (void)hipGetLastError(); return; }
  if (!prop.cooperativeLaunch) return;
  if (fused_max_blocks_per_cu(lds) < 1) return;
  const int grid = std::min(prop.multiProcessorCount, 64 * 16);
  // where do the workgroups of such a launch land?  Team t = workgroups with index % n == t must
  // share one XCD.
  int* xcc_dev = c->at<int>(p.stamps);
  std::vector<int> xcc(grid, -1);
  if (launch_probe_placement(xcc_dev, grid, lds, c->stream) != hipSuccess ||
      hipMemcpyAsync(xcc.data(), xcc_dev, (size_t)grid * 4, hipMemcpyDeviceToHost, c->stream) != hipSuccess ||
      hipStreamSynchronize(c->stream) != hipSuccess) {
    (void)hipGetLastError();
    return;
  }
  const int n_teams = *std::max_element(xcc.begin(), xcc.end()) + 1;
  if (n_teams < 1 || n_teams > kMaxTeams || grid < n_teams) return;
  // round-robin from a starting XCD that may differ from launch to launch
  for (int b = 0; b < grid; ++b)
    if (xcc[b] != (b + xcc[0]) % n_teams) return;
  std::vector<Stage> prog;
  const int n = build_verify_program(c, prog);
  if (n > p.stage_cap || n > kFusedMaxStages) return;
  if (hipMemcpyAsync(c->ws + p.stages, prog.data(), prog.size() * sizeof(Stage), hipMemcpyHostToDevice, c->stream) != hipSuccess ||
      hipMemsetAsync(c->ws + p.bar, 0, 8 * (size_t)kBarWords, c->stream) != hipSuccess || hipStreamSynchronize(c->stream) != hipSuccess) {
    (void)hipGetLastError();
    return;
  }
  c->fused_grid = grid;
  c->fused_teams = n_teams;
  c->fused_stages = n;
  c->fused_lds = lds;
  c->dev_base = 0;
  for (int t = 0; t < kMaxTeams; ++t) c->team_base[t] = 0;
  // Off unless asked for: one launch per stage is the faster path at every size measured (a
  // kernel boundary costs no more than a device-wide barrier inside the persistent kernel, and
  // the per-stage kernels pick their own grid).
  c->fused_rows = 0;
}

// One launch: the whole verify forward for the rows the tables describe.  k[b] = rows of
// sequence b; sequences go to the teams in contiguous runs of about M / n_teams rows.
static hipError_t fused_verify_forward(ad_ctx* c, const int* k, int M, int B, bool do_accept, bool stamps = false) {
  const Plan& p = c->plan;
  const ad_config& cf = c->cfg;
  VerifyTables t = tables(c);
  FusedArgs fa{};
  fa.stages = c->at<Stage>(p.stages); fa.n_stages = c->fused_stages;
  fa.M = M; fa.B = B; fa.d = cf.d_model; fa.H = cf.n_heads; fa.dh = cf.d_model / cf.n_heads; fa.V = cf.vocab;
  fa.sqrt_d = sqrtf((float)cf.d_model); fa.pe = c->at<float>(p.pe);
  fa.row_tok = t.row_tok; fa.row_pos = t.row_pos;
  const int nt = c->fused_teams;
  fa.n_teams = nt;
  {
    // sequence b goes to team floor(first row of b * n_teams / M): contiguous, balanced by rows
    int b = 0, rows = 0;
    for (int tm = 0; tm < nt; ++tm) {
      fa.team_seq[tm] = b; fa.team_row[tm] = rows;
      while (b < B && (tm == nt - 1 || (long long)rows * nt / M <= tm)) { rows += k[b]; ++b; }
    }
    fa.team_seq[nt] = B; fa.team_row[nt] = M;
  }
  for (int tm = 0; tm < nt; ++tm) fa.team_base[tm] = c->team_base[tm];
  fa.bar = c->at<unsigned long long>(p.bar); fa.dev_base = c->dev_base; fa.zero = 0;
  fa.out_w = c->w[AD_VERIFIER].out_w; fa.xa = c->at<void>(p.xa);
  fa.logits = cf.debug_logits ? c->at<float>(p.logits) : nullptr;
  fa.part_val = c->at<float>(p.part_val); fa.part_idx = c->at<int>(p.part_idx); fa.part_stride = p.n_strips;
  fa.o_hat = c->at<int>(p.o_hat); fa.o_val = c->at<float>(p.o_val);
  fa.do_accept = do_accept ? 1 : 0;
  fa.k = c->at<int>(p.k_dev); fa.draft = c->at<int>(p.draft_dev); fa.row_start = t.row_start;
  fa.max_out = c->at<int>(p.max_out); fa.k_max = cf.k_max; fa.eos = cf.eos; fa.max_len = cf.max_len;
  fa.len = c->at<int>(p.len); fa.pending = c->at<int>(p.pending); fa.finished = c->at<int>(p.finished);
  fa.out = c->at<int>(p.out); fa.result = c->at<int>(p.result);
  fa.stamps = stamps ? c->at<unsigned long long>(p.stamps) : nullptr;
  hipError_t e = launch_fused_forward(fa, c->fused_grid, c->fused_lds, c->stream);
  if (e == hipSuccess) {
    c->dev_base += 2;
    for (int tm = 0; tm < nt; ++tm)
      if (fa.team_row[tm + 1] > fa.team_row[tm]) {
        const int T = (c->fused_grid - tm + nt - 1) / nt;
        c->team_base[tm] += (unsigned long long)(c->fused_stages - 1) * T;
      }
  }
  return e;
}

// The verify forward over the M packed rows the tables describe.  ev (optional) brackets the
// output-projection kernel.
// finish = false: the caller finishes the arg max itself (n_part partials per row are returned)
// plain_rows = true: the last LayerNorm runs as a launch of its own, so the rows the output
// projection multiplies are in memory (xa) for whoever multiplies them again
// embedded = true: the rows are embedded already (x, xa)
static int verify_forward(ad_ctx* c, int M, hipEvent_t ev_a = nullptr, hipEvent_t ev_b = nullptr, bool finish = true,
                          bool plain_rows = false, bool embedded = false) {
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
  const int n_part = vocab_argmax(c, w, c->at<void>(p.xa), M, c->ln_vocab);
  if (ev_b) (void)hipEventRecord(ev_b, c->stream);
  if (finish) vocab_finish(c, M, n_part);
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

const char* ad_last_error(const ad_ctx* ctx) { return ctx ? ctx->err.c_str() : ad::global_error(); }

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
  // ad_verify's part [k | draft | result | o_hat | ticket + slots] <= B (6 + 2 k_max) + 8 ints, then ad_encode's
  // [src_len | max_out | src] once per model, then the persistent forward's flag words at the very end
  c->pin_ints = (12 * B + B * cfg->k_max * 2 + 2 * B * cfg->max_src + B * cfg->max_len + plan.mv_cap + 160 + 3) / 4 * 4;
  auto bail = [&](const char* what, hipError_t e) {
    std::string m = std::string(what) + ": " + hipGetErrorString(e);
    if (c->pin) (void)hipHostFree(c->pin);
    for (hipEvent_t ev : {c->ev0, c->ev1, c->ev2, c->ev3, c->ev_up[0], c->ev_up[1]})
      if (ev) (void)hipEventDestroy(ev);
    delete c;
    return fail(nullptr, AD_EDEVICE, m);
  };
  hipError_t e;
  if ((e = hipHostMalloc((void**)&c->pin, c->pin_ints * 4, hipHostMallocMapped)) != hipSuccess) return bail("hipHostMalloc", e);
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
  setup_fused(c);
  *out = c;
  return AD_OK;
}

int ad_destroy(ad_ctx* c) {
  if (!c) return AD_EINVAL;
  (void)hipStreamSynchronize(c->stream);
  if (c->pin) (void)hipHostFree(c->pin);
  for (auto& kv : c->graphs) (void)hipGraphExecDestroy(kv.second);
  for (hipEvent_t ev : {c->ev0, c->ev1, c->ev2, c->ev3, c->ev_up[0], c->ev_up[1]})
    if (ev) (void)hipEventDestroy(ev);
  delete c;
  return AD_OK;
}

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
static bool run_as_graph(ad_ctx* c, unsigned long long shape, const std::function<void()>& launches,
                         unsigned long long more = 0) {
  if (!c->graphs_on) return false;
  const ad_ctx::GraphKey key(shape, more);
  auto it = c->graphs.find(key);
  if (it != c->graphs.end()) {
    if (hipGraphLaunch(it->second, c->stream) == hipSuccess) return true;
    (void)hipGetLastError();
    c->graphs_on = false;
    return false;
  }
  if (++c->graph_seen[key] < 3 || c->graphs.size() >= 512) return false;   // worth building once a shape keeps coming back
  if (hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal) != hipSuccess) {
    (void)hipGetLastError();
    c->graphs_on = false;
    return false;
  }
  launches();
  hipGraph_t g = nullptr;
  hipGraphExec_t ge = nullptr;
  hipError_t e = hipStreamEndCapture(c->stream, &g);
  if (e == hipSuccess && g) e = hipGraphInstantiate(&ge, g, nullptr, nullptr, 0);
  if (g) (void)hipGraphDestroy(g);
  if (e != hipSuccess || !ge) {
    (void)hipGetLastError();
    c->graphs_on = false;
    return false;
  }
  c->graphs[key] = ge;
  if (hipGraphLaunch(ge, c->stream) == hipSuccess) return true;
  (void)hipGetLastError();
  c->graphs_on = false;
  return false;
}

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
  // src_len[B], max_out[B], src[B, max_src] go into a part of the staging buffer that no other
  // call writes (one part per model).  The device reads them there (mapped memory) or gets them by
  // one copy; either way the call returns without waiting (what follows on the stream is ordered
  // behind it), so only the next ad_encode of the same model has to make sure they have been read.
  const size_t enc_ints = (size_t)cf.max_batch * (2 + S);
  int32_t* h = c->pin + (size_t)cf.max_batch * (6 + 2 * cf.k_max) + 8 + (size_t)model * enc_ints;
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
                       t.self_desc, B, c->fw_max_rows, cf.n_heads, d / cf.n_heads, S, c->stream);
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
  const unsigned long long key = (1ull << 63) | ((unsigned long long)model << 62) | shape_key(M, c->fw_max_rows, B, 0);
  if (!run_as_graph(c, key, launches)) launches();
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

int ad_verify(ad_ctx* c, const int32_t* draft, const int32_t* k, int32_t* n_accept, int32_t* next_token,
              int32_t* verified) {
  if (!c) return fail(nullptr, AD_EINVAL, "null context");
  if (!draft || !k || !n_accept || !next_token) return fail(c, AD_EINVAL, "null buffer");
  if (!c->encoded[AD_VERIFIER]) return fail(c, AD_ESTATE, "ad_verify before ad_encode(AD_VERIFIER)");
  const ad_config& cf = c->cfg;
  const Plan& p = c->plan;
  const int B = c->B, km = cf.k_max;
  int M = 0;
  for (int b = 0; b < B; ++b) {
    if (k[b] < 0 || k[b] > km) return fail(c, AD_EINVAL, "k[b] outside [0, k_max]");
    if (k[b] && c->h_finished[b]) return fail(c, AD_ESTATE, "k[b] > 0 for a finished sequence");
    for (int i = 0; i < k[b]; ++i) {
      int32_t t = draft[(size_t)b * km + i];
      if (t == AD_NEVER ? i != k[b] - 1 : (t < 0 || t >= cf.vocab))
        return fail(c, AD_EINVAL, "draft id outside the vocabulary (AD_NEVER is allowed last only)");
    }
    M += k[b];
  }
  if (M == 0) {
    for (int b = 0; b < B; ++b) { n_accept[b] = 0; next_token[b] = 0; }
    return AD_OK;
  }
  int32_t* h = c->pin;
  memcpy(h, k, (size_t)B * 4);
  for (int b = 0; b < B; ++b) memcpy(h + B + (size_t)b * km, draft + (size_t)b * km, (size_t)km * 4);
  const bool gadpp = c->gadpp_beta > 1;
  bool fused = c->fused_rows > 0 && M <= c->fused_rows && !gadpp;
  // One launch per stage: the two small kernels that need k and the draft read them where they
  // are, in the pinned (device-visible) staging buffer, and the result is written there too: no
  // copy operations around the forward.  The persistent kernel works on device copies at
  // k_dev = [k | draft] laid out for max_batch.
  const bool mapped = c->pin_dev != nullptr;
  const int* k_src = mapped ? c->pin_dev : nullptr;
  const int* draft_src = mapped ? c->pin_dev + B : nullptr;
  if (fused || !mapped) {
    HIP_TRY(c, hipMemcpyAsync(c->at<int>(p.k_dev), h, (size_t)B * 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->at<int>(p.draft_dev), h + B, (size_t)B * km * 4, hipMemcpyHostToDevice, c->stream));
    k_src = c->at<int>(p.k_dev);
    draft_src = c->at<int>(p.draft_dev);
  }
  VerifyTables t = tables(c);
  c->fw_nseq = B;
  c->fw_max_rows = *std::max_element(k, k + B);
  c->last_nseq = B; c->last_max_rows = c->fw_max_rows;
  auto assemble = [&]() {
    launch_assemble_verify(k_src, draft_src, km, c->at<int>(p.len), c->at<int>(p.pending),
                           c->at<int>(p.src_len[0]), B, p.l_cap, cf.max_src, t, c->stream);
  };
  if (fused) assemble();
  int32_t* res = c->pin + (size_t)B * (1 + km);
  int32_t* oh = res + 2 * B;
  unsigned long long* flags = (unsigned long long*)(c->pin + c->pin_ints - 2 * (kBarPlacement - kBarAbort + 2) - 2);
  // the call's ticket, then one 8-byte slot per sequence (8-byte aligned)
  int32_t* ticket_in = c->pin + (((size_t)(oh - c->pin) + p.mv_cap + 1) & ~(size_t)1);
  unsigned long long* ticket_out = (unsigned long long*)(ticket_in + 2);
  bool watch = false, seen_ticket = false;
  for (;;) {
    if (fused) {
      HIP_TRY(c, fused_verify_forward(c, k, M, B, true));
      HIP_TRY(c, hipMemcpyAsync(res, c->at<int>(p.result), (size_t)B * 8, hipMemcpyDeviceToHost, c->stream));
    } else {
      int* result_dst = mapped ? c->pin_dev + (res - c->pin) : c->at<int>(p.result);
      // The result lands in host memory the device writes directly; the call's ticket follows it,
      // and the host watches for the ticket instead of waiting for the stream to drain (the end of
      // the kernel, its completion signal and the runtime's wake-up are off the critical path).
      watch = mapped && c->spin_wait && !verified;
      if (watch) {
        if (++c->ticket >= (1 << 18)) c->ticket = 1;
        *ticket_in = c->ticket;
        for (int b = 0; b < B; ++b) ticket_out[b] = 0;   // whatever an earlier call left in these words
      }
      auto accept = [&](const float* pv, const int* pi, int stride, int n_part, const GadppIn& gp = GadppIn{}) {
        launch_argmax_accept(pv, pi, stride, n_part, c->at<int>(p.o_hat), c->at<float>(p.o_val), k_src, draft_src, km,
                             t.row_start, B, cf.eos, cf.max_len, c->at<int>(p.max_out), c->at<int>(p.len),
                             c->at<int>(p.pending), c->at<int>(p.finished), c->at<int>(p.out), result_dst,
                             watch ? c->pin_dev + (ticket_in - c->pin) : nullptr,
                             watch ? (unsigned long long*)(c->pin_dev + ((int32_t*)ticket_out - c->pin)) : nullptr,
                             c->fw_max_rows, M, c->stream, gp);
      };
      auto launches = [&]() {
        launch_assemble_embed_verify(cf.dtype, k_src, draft_src, km, c->at<int>(p.len), c->at<int>(p.pending),
                                     c->at<int>(p.src_len[0]), B, p.l_cap, cf.max_src, t, M, c->w[AD_VERIFIER].emb,
                                     c->at<float>(p.pe), cf.d_model, sqrtf((float)cf.d_model), c->at<float>(p.x),
                                     c->at<void>(p.xa), c->stream);
        if (!gadpp) {
          const int n_part = verify_forward(c, M, nullptr, nullptr, false, false, true);
          accept(c->at<float>(p.part_val), c->at<int>(p.part_idx), p.n_strips, n_part);
          return;
        }
        // GAD++ (Section 3.2.3): arg max as before; then the score of every row's drafted token,
        // a second pass of the output projection that counts the columns scoring above it (the
        // logits still never reach memory), the relaxed replacement of o_hat, and acceptance
        const ModelW& w = c->w[AD_VERIFIER];
        (void)verify_forward(c, M, nullptr, nullptr, true, true, true);
        launch_draft_logit(cf.dtype, c->at<void>(p.xa), w.out_w, M, cf.vocab, cf.d_model, t.row_seq, t.row_start,
                           draft_src, km, c->at<float>(p.draft_lp), c->at<int>(p.draft_col), c->stream);
        Epi e{};
        e.mode = EPI_COUNT; e.part_idx = c->at<int>(p.part_idx); e.n_strips = p.n_strips; e.thr = c->at<float>(p.draft_lp);
        const int n_cnt = launch_gemm(cf.dtype, c->at<void>(p.xa), w.out_w, M, cf.vocab, cf.d_model, e, c->stream);
        // (the relaxed replacement of o_hat happens inside the acceptance kernel)
        GadppIn gp;
        gp.part_cnt = c->at<int>(p.part_idx); gp.stride = p.n_strips; gp.n_part = n_cnt;
        gp.lp = c->at<float>(p.draft_lp); gp.col = c->at<int>(p.draft_col);
        gp.beta = c->gadpp_beta; gp.tau = c->gadpp_tau;
        accept(c->at<float>(p.o_val), c->at<int>(p.o_hat), 1, 1, gp);
      };
      // every launch argument is a function of (rows, sequences, longest block), of the GAD++
      // setting and of pointers fixed for the context's life
      // (and of whether the acceptance kernel posts the ticket)
      const unsigned long long key = shape_key(M, c->fw_max_rows, B, (gadpp ? 1 : 0) | (watch ? 2 : 0) | (c->fuse_crossq ? 4 : 0));
      unsigned tau_bits;
      memcpy(&tau_bits, &c->gadpp_tau, 4);
      const unsigned long long more = gadpp ? ((unsigned long long)c->gadpp_beta << 32) | tau_bits : 0;
      if (!mapped || !run_as_graph(c, key, launches, more)) launches();
      if (!mapped) HIP_TRY(c, hipMemcpyAsync(res, c->at<int>(p.result), (size_t)B * 8, hipMemcpyDeviceToHost, c->stream));
    }
    flags[0] = 0; flags[kBarPlacement - kBarAbort] = 1; flags[kBarPlacement - kBarAbort + 1] = 1;
    const int place_word = kBarPlacement - kBarAbort + (int)(((c->dev_base >> 1) + 1) & 1);   // of the launch above
    if (fused)
      HIP_TRY(c, hipMemcpyAsync(flags, c->at<unsigned long long>(p.bar) + kBarAbort,
                                8 * (size_t)(kBarPlacement - kBarAbort + 2), hipMemcpyDeviceToHost, c->stream));
    if (verified) HIP_TRY(c, hipMemcpyAsync(oh, c->at<int>(p.o_hat), (size_t)M * 4, hipMemcpyDeviceToHost, c->stream));
    bool seen = false;
    seen_ticket = false;
    if (watch && !fused) {
      const int want = c->ticket;
      const auto t_end = std::chrono::steady_clock::now() + std::chrono::milliseconds(50);
      for (unsigned spin = 1;; ++spin) {
        int b = 0;
        while (b < B && (int)(__atomic_load_n(ticket_out + b, __ATOMIC_ACQUIRE) >> 46) == want) ++b;
        if (b == B) { seen = seen_ticket = true; break; }
        if ((spin & 1023u) == 0 && std::chrono::steady_clock::now() > t_end) break;   // fall back to the stream
        __builtin_ia32_pause();
      }
    }
    if (!seen) {
      HIP_TRY(c, hipStreamSynchronize(c->stream));
      HIP_TRY(c, hipGetLastError());
    }
    if (flags[0]) {
      // a barrier timed out: the decode state is undefined; switch the persistent path off
      c->fused_rows = 0;
      c->encoded[AD_VERIFIER] = false;
      return fail(c, AD_EDEVICE, "persistent forward: a barrier timed out (state lost, encode again)");
    }
    if (fused && (flags[place_word] & (flags[place_word] - 1)) != 0) {
      // a team was spread over several XCDs: the kernel left the decode state alone;
      // run this call, and all later ones, with one launch per stage
      c->fused_rows = 0;
      fused = false;
      continue;
    }
    break;
  }
  c->last_fused = fused;
  c->last_k.assign(k, k + B);
  int r0 = 0;
  for (int b = 0; b < B; ++b) {
    if (seen_ticket) {
      const unsigned long long v = ticket_out[b];
      n_accept[b] = (int)((v >> 32) & 0x3fff);
      next_token[b] = (int)(unsigned)v;
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
    r0 += k[b];
  }
  c->last_M = M;
  c->last_logit_rows = M;
  return AD_OK;
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
  int M = 0, live = 0;
  for (int b = 0; b < B; ++b)
    if (!c->h_finished[b]) { M += c->h_len[b] + 1 + k; ++live; }
  if (live == 0) {
    for (size_t i = 0; i < (size_t)B * km; ++i) draft_out[i] = AD_NEVER;
    return AD_OK;
  }
  VerifyTables t = tables(c);
  int max_rows = k;
  for (int b = 0; b < B; ++b)
    if (!c->h_finished[b]) max_rows = std::max(max_rows, c->h_len[b] + 1);
  const int Mv = live * k;
  int32_t* h = c->pin;
  unsigned long long* slots = (unsigned long long*)c->pin;          // [B, k_max]
  int32_t* ticket_in = c->pin + 2 * (size_t)B * km;                 // behind the slots
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
                          c->at<int>(p.finished), B, k, km, c->pin_dev + (ticket_in - c->pin),
                          (unsigned long long*)c->pin_dev, c->stream);
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
  HIP_TRY(c, hipMemcpyAsync(c->pin, c->at<int>(c->plan.out), (size_t)B * L * 4, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  for (int b = 0; b < B; ++b) {
    out_len[b] = c->h_len[b];
    for (int i = 0; i < L; ++i) out[(size_t)b * L + i] = i < c->h_len[b] ? c->pin[(size_t)b * L + i] : c->cfg.pad;
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
  if (option != AD_OPT_FUSED_ROWS) return fail(c, AD_EINVAL, "unknown option");
  if (value < 0 || value > c->plan.mv_cap) return fail(c, AD_EINVAL, "AD_OPT_FUSED_ROWS must be in [0, max_batch * k_max]");
  if (value > 0 && c->fused_grid == 0) return fail(c, AD_ESTATE, "the persistent forward is unavailable for this context");
  c->fused_rows = value;
  return AD_OK;
}
int ad_get_option(ad_ctx* c, int option, int* value) {
  if (!c) return fail(nullptr, AD_EINVAL, "null context");
  if (!value) return fail(c, AD_EINVAL, "null pointer");
  if (option == AD_OPT_FUSED_ROWS) *value = c->fused_rows;
  else if (option == AD_OPT_FUSED_AVAILABLE) *value = c->fused_grid > 0 ? 1 : 0;
  else if (option == AD_OPT_GRAPHS) *value = c->graphs_on ? 1 : 0;
  else if (option == AD_OPT_GRAPHS_CAPTURED) *value = (int)c->graphs.size();
  else if (option == AD_OPT_SPIN_WAIT) *value = c->spin_wait ? 1 : 0;
  else if (option == AD_OPT_FUSE_CROSSQ) *value = c->fuse_crossq ? 1 : 0;
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
  c->fw_nseq = c->last_nseq; c->fw_max_rows = c->last_max_rows;
  if (c->last_fused && c->fused_rows > 0) {
    // one kernel: the whole forward (arg max included, acceptance skipped)
    const int* k = c->last_k.data();
    HIP_TRY(c, fused_verify_forward(c, k, c->last_M, c->last_nseq, false));
    for (int r = 0; r < reps; ++r) {
      HIP_TRY(c, hipEventRecord(c->ev0, c->stream));
      HIP_TRY(c, fused_verify_forward(c, k, c->last_M, c->last_nseq, false));
      HIP_TRY(c, hipEventRecord(c->ev3, c->stream));
      HIP_TRY(c, hipEventSynchronize(c->ev3));
      float a = 0;
      HIP_TRY(c, hipEventElapsedTime(&a, c->ev0, c->ev3));
      tot += a * 1e3;
    }
    *forward_us = tot / reps;
    *vocab_kernel_us = 0;
    if (vocab_back_to_back_us) *vocab_back_to_back_us = 0;
    unsigned long long flags[kBarPlacement - kBarAbort + 2];
    const int place_word = kBarPlacement - kBarAbort + (int)(((c->dev_base >> 1) + 1) & 1);   // of the last launch
    HIP_TRY(c, hipMemcpyAsync(flags, c->at<unsigned long long>(c->plan.bar) + kBarAbort, sizeof(flags), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (flags[0] || (flags[place_word] & (flags[place_word] - 1)) != 0) {
      c->fused_rows = 0;
      return fail(c, AD_EDEVICE, "persistent forward: barrier time-out or misplaced workgroup while timing");
    }
    return AD_OK;
  }
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
  c->fw_nseq = c->last_nseq; c->fw_max_rows = c->last_max_rows;
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

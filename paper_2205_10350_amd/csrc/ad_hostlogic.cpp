// Host-only logic: configuration checks, weight layout, the suffix match of Algorithm 1 and
// the decode loops (greedy, input-guided, draft-verify) written against an abstract
// verifier so that the very same loops run over the GPU and over a model-free stand-in.
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <chrono>
#include <string>

#include "ad_internal.h"

namespace ad {

// (a fixed buffer: reporting an error allocates nothing)
static thread_local char g_error[320] = "";
void set_global_error(const char* msg) { snprintf(g_error, sizeof(g_error), "%s", msg ? msg : ""); }
const char* global_error() { return g_error; }

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---------------------------------------------------------------------------------------------
std::vector<WEntry> weight_layout(const ad_config& c, size_t* total_bytes) {
  std::vector<WEntry> v;
  size_t off = 0;
  const int d = c.d_model, f = c.d_ffn;
  const int mb = c.dtype == AD_BF16 ? 2 : 4;   // matrix element bytes
  // bf16 matrices that feed a GEMM are stored as MFMA B-operand tiles (see ad.h); the embedding
  // table is gathered by row and stays row-major
  auto mat = [&](const std::string& n, int rows, int cols, bool gemm = true) {
    v.push_back({n, off, rows, cols, mb, (gemm && c.dtype == AD_BF16) ? 1 : 0});
    off += (size_t)rows * cols * mb;
  };
  auto vec = [&](const std::string& n, int cols) {
    v.push_back({n, off, 1, cols, 4, 0});
    off += (size_t)cols * 4;
  };
  auto group = [&]() { off = align_up(off, 256); };
  auto attn = [&](const std::string& p) {
    group(); mat(p + ".wq", d, d); mat(p + ".wk", d, d); mat(p + ".wv", d, d);   // one [3d, d]
    group(); mat(p + ".wo", d, d);
    group(); vec(p + ".bq", d); vec(p + ".bk", d); vec(p + ".bv", d);             // one [3d]
    group(); vec(p + ".bo", d);
  };
  auto ln = [&](const std::string& p) { group(); vec(p + ".g", d); group(); vec(p + ".b", d); };
  auto ffn = [&](const std::string& p) {
    group(); mat(p + ".w1", f, d); group(); vec(p + ".b1", f);
    group(); mat(p + ".w2", d, f); group(); vec(p + ".b2", d);
  };
  group(); mat("emb", c.vocab, d, false);
  // a tied output projection still gets its own (tiled) copy of the table in bf16 mode
  if (!c.tie_output || c.dtype == AD_BF16) { group(); mat("out.w", c.vocab, d); }
  for (int l = 0; l < c.enc_layers; ++l) {
    std::string p = "enc." + std::to_string(l);
    attn(p + ".self"); ln(p + ".ln1"); ffn(p + ".ffn"); ln(p + ".ln2");
  }
  for (int l = 0; l < c.dec_layers; ++l) {
    std::string p = "dec." + std::to_string(l);
    attn(p + ".self"); ln(p + ".ln1"); attn(p + ".cross"); ln(p + ".ln2"); ffn(p + ".ffn"); ln(p + ".ln3");
  }
  group();
  if (total_bytes) *total_bytes = off;
  return v;
}

ModelW bind_weights(const ad_config& c, const void* blob) {
  size_t total = 0;
  std::vector<WEntry> lay = weight_layout(c, &total);
  const char* base = (const char*)blob;
  auto find = [&](const std::string& n) -> const void* {
    for (const WEntry& e : lay)
      if (e.name == n) return base + e.offset;
    return nullptr;
  };
  auto attn = [&](const std::string& p) {
    AttnW a;
    a.wqkv = find(p + ".wq"); a.wo = find(p + ".wo");
    a.bqkv = (const float*)find(p + ".bq"); a.bo = (const float*)find(p + ".bo");
    return a;
  };
  auto ln = [&](const std::string& p) { return LnW{(const float*)find(p + ".g"), (const float*)find(p + ".b")}; };
  auto ffn = [&](const std::string& p) {
    return FfnW{find(p + ".w1"), find(p + ".w2"), (const float*)find(p + ".b1"), (const float*)find(p + ".b2")};
  };
  ModelW m;
  m.emb = find("emb");
  m.out_w = (c.tie_output && c.dtype != AD_BF16) ? m.emb : find("out.w");
  for (int l = 0; l < c.enc_layers; ++l) {
    std::string p = "enc." + std::to_string(l);
    m.enc.push_back({attn(p + ".self"), ln(p + ".ln1"), ffn(p + ".ffn"), ln(p + ".ln2")});
  }
  for (int l = 0; l < c.dec_layers; ++l) {
    std::string p = "dec." + std::to_string(l);
    m.dec.push_back({attn(p + ".self"), ln(p + ".ln1"), attn(p + ".cross"), ln(p + ".ln2"), ffn(p + ".ffn"),
                     ln(p + ".ln3")});
  }
  return m;
}

// ---------------------------------------------------------------------------------------------
// Algorithm 1, the if-test.  Grow the suffix o_{j-q..j} from q = 0; the first q for which it
// occurs at most once in x decides: once -> match at its end index, never -> no match.
int suffix_match(const int32_t* o, int o_len, const int32_t* x, int x_len, int* i_out) {
  const int j = o_len - 1;
  // candidates: end indices i in x where the current suffix matches; refine as q grows
  std::vector<int> cand;
  for (int i = 0; i < x_len; ++i)
    if (x[i] == o[j]) cand.push_back(i);
  for (int q = 0;; ++q) {
    if (cand.size() == 1) { *i_out = cand[0]; return 1; }
    if (cand.empty() || q == j) return 0;
    // extend by o_{j-q-1}: keep the candidates whose (q+1)-th token back agrees
    std::vector<int> next;
    for (int i : cand)
      if (i - q - 1 >= 0 && x[i - q - 1] == o[j - q - 1]) next.push_back(i);
    cand.swap(next);
  }
}

static double now_us() {
  return std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

// Appends what a verify call accepted.  The appended block is (draft_1..draft_{n-1}, next).
static void apply_result(LoopIO& io, int b, const int32_t* draft_row, int n, int32_t next) {
  for (int i = 0; i + 1 < n; ++i) io.o[b].push_back(draft_row[i]);
  if (n > 0) io.o[b].push_back(next);
}
static bool finished(const LoopIO& io, int b) {
  const std::vector<int32_t>& o = io.o[b];
  return (o.size() > 1 && o.back() == io.eos) || (int)o.size() - 1 >= io.max_out[b];
}

static int run_loop(Backend& be, LoopIO& io, int mode, int k_block, bool use_drafter,
                    const std::vector<std::vector<int32_t>>* aux) {
  const int B = io.B, kmax = io.k_max;
  std::vector<int32_t> draft((size_t)B * kmax), k(B), n_acc(B), next(B), nat((size_t)B * kmax);
  std::vector<std::vector<int32_t>> x(B);
  if (mode == 0)
    for (int b = 0; b < B; ++b) {   // x = ([BOS], guide, [PAD]) with [PAD] = the never-matching id
      x[b].push_back(io.bos);
      x[b].insert(x[b].end(), (*aux)[b].begin(), (*aux)[b].end());
      x[b].push_back(AD_NEVER);
    }
  io.o.assign(B, std::vector<int32_t>(1, io.bos));
  io.accepted.clear();
  io.stats = ad_stats{};
  for (;;) {
    double t0 = now_us();
    bool any = false;
    if (mode == 2 && use_drafter) {
      bool live = false;
      for (int b = 0; b < B; ++b) live = live || !finished(io, b);
      if (!live) break;
      double td = now_us();
      io.stats.t_host_us += td - t0;
      int rc = be.draft(k_block, nat.data());
      if (rc != AD_OK) return rc;
      t0 = now_us();
      io.stats.t_draft_us += t0 - td;
      for (int b = 0; b < B; ++b)
        if (!finished(io, b)) io.stats.draft_rows += (int64_t)io.o[b].size() + k_block;
    }
    for (int b = 0; b < B; ++b) {
      k[b] = 0;
      if (finished(io, b)) continue;
      any = true;
      const int j = (int)io.o[b].size() - 1;
      const int room = std::min(io.max_out[b] - j, kmax);
      int32_t* row = &draft[(size_t)b * kmax];
      int n = 0;
      if (mode == 0) {            // input-guided: rest of the guide after a unique suffix match
        int i = 0;
        if (suffix_match(io.o[b].data(), j + 1, x[b].data(), (int)x[b].size(), &i))
          for (int t = i + 1; t < (int)x[b].size() && n < room; ++t) row[n++] = x[b][t];
      } else if (mode == 2) {     // block draft: positional override, else the drafter's proposal
        const int kk = std::min(k_block, room);
        if (aux) {
          const std::vector<int32_t>& D = (*aux)[b];
          for (int t = j; t < (int)D.size() && n < kk; ++t) row[n++] = D[t];
        } else if (use_drafter) {
          for (int t = 0; t < kk; ++t) row[n++] = nat[(size_t)b * kmax + t];
        }
      }
      if (n == 0) row[n++] = AD_NEVER;   // plain autoregressive step
      // the never-matching id may only close a draft
      for (int t = 0; t + 1 < n; ++t)
        if (row[t] == AD_NEVER) { n = t + 1; break; }
      k[b] = n;
    }
    if (!any) break;
    io.stats.t_host_us += now_us() - t0;
    double tv = now_us();
    int rc = be.verify(draft.data(), k.data(), n_acc.data(), next.data());
    if (rc != AD_OK) return rc;
    io.stats.t_verify_us += now_us() - tv;
    t0 = now_us();
    std::vector<int> acc(B, 0);
    for (int b = 0; b < B; ++b) {
      if (!k[b]) continue;
      if (n_acc[b] < 1 || n_acc[b] > k[b]) return AD_EDEVICE;
      apply_result(io, b, &draft[(size_t)b * kmax], n_acc[b], next[b]);
      acc[b] = n_acc[b];
      io.stats.rows_verified += k[b];
      io.stats.tokens_out += n_acc[b];
    }
    io.accepted.push_back(acc);
    io.stats.iterations += 1;
    io.stats.t_host_us += now_us() - t0;
  }
  return AD_OK;
}

int loop_iad(Backend& be, LoopIO& io, const std::vector<std::vector<int32_t>>& guide) {
  return run_loop(be, io, 0, 0, false, &guide);
}
int loop_gad(Backend& be, LoopIO& io, int k, bool use_drafter,
             const std::vector<std::vector<int32_t>>* override_draft) {
  return run_loop(be, io, 2, k, use_drafter, override_draft);
}
int loop_greedy(Backend& be, LoopIO& io) { return run_loop(be, io, 1, 1, false, nullptr); }

// ---------------------------------------------------------------------------------------------
// Model-free stand-in for the verifier: knows the greedy output g of one sequence.  Row i is
// fed (o_<=j, draft_1..draft_{i-1}); if that prefix agrees with g the prediction is g's next
// token, otherwise (or past the end of g) a value no draft can equal.
struct FakeVerifier : Backend {
  std::vector<int32_t> g, o;   // o: accepted so far (without o_0)
  int eos, max_out, k_max;
  int verify(const int32_t* draft, const int32_t* k, int32_t* n_accept, int32_t* next) override {
    const int kb = k[0];
    if (kb < 1 || kb > k_max) return AD_EINVAL;
    if ((!o.empty() && o.back() == eos) || (int)o.size() >= max_out) return AD_ESTATE;
    bool ok = std::equal(o.begin(), o.end(), g.begin());
    std::vector<int32_t> o_hat(kb);
    for (int i = 0; i < kb; ++i) {
      size_t pos = o.size() + i;
      if (i > 0 && ok) ok = pos - 1 < g.size() && draft[i - 1] == g[pos - 1];
      o_hat[i] = (ok && pos < g.size()) ? g[pos] : -1000 - i;
    }
    int c = kb;
    for (int i = 0; i < kb; ++i)
      if (draft[i] != o_hat[i]) { c = i + 1; break; }
    int n = 0;
    for (int i = 0; i < c; ++i) {
      if ((int)o.size() >= max_out) break;
      o.push_back(o_hat[i]); ++n;
      if (o_hat[i] == eos) break;
    }
    n_accept[0] = n;
    next[0] = n ? o.back() : 0;
    return AD_OK;
  }
};

}  // namespace ad

// =================================================================================================
extern "C" {

int ad_config_check(const ad_config* c) {
  using ad::set_global_error;
  if (!c) { set_global_error("null config"); return AD_EINVAL; }
  if (c->dtype != AD_F32 && c->dtype != AD_BF16) { set_global_error("dtype must be AD_F32 or AD_BF16"); return AD_EINVAL; }
  if (c->d_model < 32 || c->d_model % 32 || c->d_model > 2048) { set_global_error("d_model must be a multiple of 32 in [32, 2048]"); return AD_EINVAL; }
  if (c->d_ffn < 32 || c->d_ffn % 32) { set_global_error("d_ffn must be a multiple of 32"); return AD_EINVAL; }
  if (c->n_heads < 1 || c->d_model % c->n_heads) { set_global_error("n_heads must divide d_model"); return AD_EINVAL; }
  const int dh = c->d_model / c->n_heads;
  if (dh != 16 && dh != 32 && dh != 64 && dh != 128) { set_global_error("head size must be 16, 32, 64 or 128"); return AD_EINVAL; }
  if (c->vocab < 16 || c->vocab % 16) { set_global_error("vocab must be a multiple of 16"); return AD_EINVAL; }
  if (c->enc_layers < 1 || c->dec_layers < 1) { set_global_error("need at least one encoder and one decoder layer"); return AD_EINVAL; }
  if (c->max_batch < 1 || c->max_src < 1 || c->max_len < 1 || c->k_max < 1) { set_global_error("capacities must be >= 1"); return AD_EINVAL; }
  if (c->max_batch > 4096 || c->max_src > 8192 || c->max_len > 8192 || c->k_max > 8192) { set_global_error("capacity too large"); return AD_EINVAL; }
  {
    // attention keeps one head's keys and values of a sequence in LDS (rows padded by a dword)
    const size_t nk = (size_t)std::max(c->max_src, c->max_len + c->k_max);
    const size_t esz = c->dtype == AD_BF16 ? 2 : 4;
    const size_t need = 2 * nk * ((size_t)dh * esz / 4 + 1) * 4 + 64 * (size_t)dh * 4 + 4 * nk * 4;
    if (need > 160 * 1024) { set_global_error("max_src / max_len + k_max too large: a head's keys and values must fit in 160 KB of LDS"); return AD_EINVAL; }
  }
  const int32_t ids[4] = {c->bos, c->pad, c->eos, c->mask};
  for (int i = 0; i < 4; ++i)
    if (ids[i] < 0 || ids[i] >= c->vocab) { set_global_error("special token id outside the vocabulary"); return AD_EINVAL; }
  return AD_OK;
}

int ad_weights_count(const ad_config* c) {
  if (ad_config_check(c) != AD_OK) return 0;
  return (int)ad::weight_layout(*c, nullptr).size();
}
size_t ad_weights_bytes(const ad_config* c) {
  if (ad_config_check(c) != AD_OK) return 0;
  size_t t = 0;
  ad::weight_layout(*c, &t);
  return t;
}
int ad_weights_entry(const ad_config* c, int index, char* name, size_t name_cap, size_t* offset,
                     int32_t* rows, int32_t* cols, int32_t* elem_bytes) {
  if (ad_config_check(c) != AD_OK) return AD_EINVAL;
  std::vector<ad::WEntry> v = ad::weight_layout(*c, nullptr);
  if (index < 0 || index >= (int)v.size()) { ad::set_global_error("weight entry index out of range"); return AD_EINVAL; }
  const ad::WEntry& e = v[index];
  if (name && name_cap) {
    strncpy(name, e.name.c_str(), name_cap - 1);
    name[name_cap - 1] = 0;
  }
  if (offset) *offset = e.offset;
  if (rows) *rows = e.rows;
  if (cols) *cols = e.cols;
  if (elem_bytes) *elem_bytes = e.elem_bytes;
  return AD_OK;
}

int ad_weights_pack(const ad_config* c, int index, const float* src, void* blob) {
  if (ad_config_check(c) != AD_OK) return AD_EINVAL;
  if (!src || !blob) { ad::set_global_error("null buffer"); return AD_EINVAL; }
  std::vector<ad::WEntry> v = ad::weight_layout(*c, nullptr);
  if (index < 0 || index >= (int)v.size()) { ad::set_global_error("weight entry index out of range"); return AD_EINVAL; }
  const ad::WEntry& e = v[index];
  char* dst = (char*)blob + e.offset;
  const size_t n = (size_t)e.rows * e.cols;
  if (e.elem_bytes == 4) {
    memcpy(dst, src, n * 4);
    return AD_OK;
  }
  auto bf16 = [](float f) {   // round to nearest, ties to even
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
  };
  uint16_t* d16 = (uint16_t*)dst;
  if (!e.tiled) {
    for (size_t i = 0; i < n; ++i) d16[i] = bf16(src[i]);
    return AD_OK;
  }
  // tile (s, u) = rows 16s..16s+15 x columns 32u..32u+31, 1 KB: lane l (0..63) owns 8 consecutive
  // columns 32u + 8*(l/16) .. of row 16s + l%16
  const int K = e.cols, ku = K / 32;
  for (int s = 0; s < e.rows / 16; ++s)
    for (int u = 0; u < ku; ++u)
      for (int l = 0; l < 64; ++l) {
        const float* sp = src + (size_t)(16 * s + l % 16) * K + 32 * u + 8 * (l / 16);
        uint16_t* dp = d16 + (((size_t)s * ku + u) * 64 + l) * 8;
        for (int j = 0; j < 8; ++j) dp[j] = bf16(sp[j]);
      }
  return AD_OK;
}

int ad_suffix_match(const int32_t* o, int o_len, const int32_t* x, int x_len, int* i_out) {
  if (!o || !x || !i_out || o_len < 1 || x_len < 1) return 0;
  return ad::suffix_match(o, o_len, x, x_len, i_out);
}

int ad_host_simulate(int mode, const int32_t* g, int g_len, const int32_t* aux, int aux_len, int k, int k_max,
                     int max_out, int eos, int bos, int32_t* out, int32_t* out_len, int32_t* accepted,
                     int acc_cap, ad_stats* stats) {
  if (!g || g_len < 0 || aux_len < 0 || (aux_len && !aux) || !out || !out_len || k_max < 1 || max_out < 1 ||
      (mode != 0 && mode != 1) || (mode == 1 && k < 1)) {
    ad::set_global_error("ad_host_simulate: bad argument");
    return AD_EINVAL;
  }
  ad::FakeVerifier fv;
  fv.g.assign(g, g + g_len);
  fv.eos = eos; fv.max_out = max_out; fv.k_max = k_max;
  ad::LoopIO io;
  io.B = 1; io.k_max = k_max; io.eos = eos; io.bos = bos;
  io.max_out.assign(1, max_out);
  std::vector<std::vector<int32_t>> a(1, std::vector<int32_t>(aux, aux + aux_len));
  int rc = mode == 0 ? ad::loop_iad(fv, io, a) : ad::loop_gad(fv, io, k, false, &a);
  if (rc != AD_OK) return rc;
  *out_len = (int)io.o[0].size() - 1;
  for (int i = 0; i < *out_len; ++i) out[i] = io.o[0][i + 1];
  if (accepted)
    for (int i = 0; i < acc_cap; ++i) accepted[i] = i < (int)io.accepted.size() ? io.accepted[i][0] : 0;
  if (stats) *stats = io.stats;
  return AD_OK;
}

}  // extern "C"

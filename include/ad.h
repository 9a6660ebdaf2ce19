/*
 * ad.h — C ABI of the MI355X-native Aggressive Decoding hot path.
 *
 * The library evaluates an encoder-decoder Transformer with hand-written gfx950
 * kernels and runs the draft-then-verify decoding of "Lossless Acceleration for
 * Seq2seq Generation with Aggressive Decoding": the parallel verification forward
 * (Section 3.2, verify paragraph), Input-guided Aggressive Decoding (Section 3.1,
 * Algorithm 1) and Generalized Aggressive Decoding (Section 3.2) with a
 * non-autoregressive block drafter (Section 3.2.1), plus plain greedy decoding
 * (Section 2) as the result every one of them must reproduce token for token.
 *
 * Conventions
 *  - Every `int32_t*` token / length buffer is HOST memory owned by the caller.
 *  - `verifier_w`, `drafter_w`, `workspace` are DEVICE pointers owned by the caller
 *    (allocate them with any allocator; they must outlive the context and the weights must
 *    not change while it lives: ad_create copies some of them into the workspace, side by
 *    side).  The library allocates no device memory, ever (its one device-side object of its
 *    own is the fixed 4 MiB static array ad_verify_static works in).  ad_create allocates one
 *    pinned, device-mapped host staging buffer, a few events and, with a drafter, one more stream
 *    of default priority (AD_OPT_OVERLAP_ENCODERS); later calls may allocate host
 *    memory for bookkeeping (the decode loops' token lists, a captured graph per call shape);
 *    ad_verify_static allocates nothing at all.
 *  - `hip_stream` is a hipStream_t (NULL = the null stream).  All device work of a
 *    context is enqueued on it.  Calls that return results return once the results are
 *    there; ad_encode returns as soon as its work is enqueued, and the tail of an ad_verify
 *    call's device work may still be running when it returns its result (AD_OPT_SPIN_WAIT).
 *    Work the caller enqueues on the same stream is ordered behind both; to touch the
 *    workspace from another stream, synchronize with this one first.
 *  - Every function returns AD_OK or a negative AD_E* code and, on error, leaves the
 *    context as it was.  Nothing throws or aborts across this boundary.
 *    ad_last_error() gives a static or per-context message for the last failure.
 *  - A context is not thread-safe.
 *
 * Token ids: [0, vocab).  AD_NEVER (-1) in a draft is the id that equals no
 * prediction (Algorithm 1 appends [PAD] to the guide for this purpose); it may
 * appear only as the LAST token of a sequence's draft because that token is
 * compared but never fed to the decoder.
 */
#ifndef AD_H_
#define AD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AD_NEVER (-1)

typedef struct ad_ctx ad_ctx;

/* Model and capacity description.  Both models (verifier, drafter) share it. */
typedef struct {
  int32_t enc_layers, dec_layers, d_model, n_heads, d_ffn, vocab;
  int32_t max_batch;   /* sequences decoded together                                  */
  int32_t max_src;     /* longest source sentence                                     */
  int32_t max_len;     /* most output tokens per sequence                             */
  int32_t k_max;       /* most rows verified (or drafted) per sequence in one call    */
  int32_t bos, pad, eos, mask;
  int32_t dtype;       /* AD_F32: fp32 weights and arithmetic; AD_BF16: bf16 weights,
                          bf16 GEMM/attention operands, fp32 accumulation, fp32 residual
                          stream, LayerNorm, softmax and logits                        */
  int32_t tie_output;  /* 1: the embedding table is also the output projection        */
  int32_t debug_logits;/* 1: keep the last forward's full logits for ad_debug_logits  */
} ad_config;

typedef struct {
  int64_t iterations;     /* verify forwards (an autoregressive step is one of k=1)   */
  int64_t rows_verified;  /* decoder rows fed to the verifier                          */
  int64_t draft_rows;     /* decoder rows fed to the drafter                           */
  int64_t tokens_out;     /* tokens emitted over the batch                             */
  double t_encode_us, t_draft_us, t_verify_us, t_host_us; /* wall time by phase       */
} ad_stats;

enum { AD_OK = 0, AD_EINVAL = -1, AD_ESTATE = -2, AD_ENOMEM = -3, AD_EDEVICE = -4 };
enum { AD_F32 = 0, AD_BF16 = 1 };
enum { AD_VERIFIER = 0, AD_DRAFTER = 1 };

/* ---- sizes and weight layout (host only, no GPU needed) ------------------------------- */

/* Validates a configuration.  AD_EINVAL with a message in ad_last_error(NULL) if a
 * dimension is unsupported (d_model % 32, d_ffn % 32, vocab % 16, head size in
 * {16,32,64,128}, capacities >= 1). */
int ad_config_check(const ad_config* cfg);

/* Bytes of device workspace ad_create needs for `cfg`; 0 if cfg is invalid.
 * `with_drafter` adds the drafter's encoder memory. */
size_t ad_workspace_bytes(const ad_config* cfg, int with_drafter);

/* A model's weights are one flat device blob.  Entry `index` (0 .. count-1) of its
 * layout: tensor name ("emb", "out.w", "enc.0.self.wq", "dec.3.ffn.b1", ... — a matrix
 * is [out_features, in_features]), byte offset, shape, and element size (2 = bf16,
 * 4 = fp32; vectors are always fp32).  ad_weights_bytes is the blob size.
 * ad_weights_entry returns AD_EINVAL past the end.
 *
 * Byte order inside an entry.  fp32 entries and the embedding table "emb" are row-major.
 * Every other bf16 matrix [N, K] is stored as the MFMA B operand reads it, so that a wave
 * fetches 1 KB contiguous per 16 x 32 tile: tile (s, u) = rows 16s..16s+15 x columns
 * 32u..32u+31 sits at element offset ((s * K/32 + u) * 64 + l) * 8 for l = 0..63, and lane
 * slot l holds the 8 consecutive columns 32u + 8*(l/16).. of row 16s + l%16.  In bf16 mode
 * "out.w" exists even with tie_output = 1 (fill it from the embedding table).
 * ad_weights_pack writes one entry into a HOST copy of the blob from a row-major fp32
 * tensor (rounding to bf16, nearest even, and tiling as needed); upload the blob afterwards. */
int    ad_weights_count(const ad_config* cfg);
size_t ad_weights_bytes(const ad_config* cfg);
int    ad_weights_entry(const ad_config* cfg, int index, char* name, size_t name_cap,
                        size_t* offset, int32_t* rows, int32_t* cols, int32_t* elem_bytes);
int    ad_weights_pack(const ad_config* cfg, int index, const float* src /* host, [rows, cols] */,
                       void* blob /* host, ad_weights_bytes() */);

/* ---- context --------------------------------------------------------------------------- */

/* Creates a context over caller-owned device memory.  `drafter_w` may be NULL (then
 * ad_draft_nat and the drafter in ad_decode_gad are unavailable).  `workspace_bytes`
 * must be >= ad_workspace_bytes().  Needs a GPU: AD_EDEVICE otherwise. */
int ad_create(const ad_config* cfg, const void* verifier_w, const void* drafter_w,
              void* workspace, size_t workspace_bytes, void* hip_stream, ad_ctx** out);
int ad_destroy(ad_ctx* ctx);
const char* ad_last_error(const ad_ctx* ctx /* NULL: last error of a context-free call */);

/* ---- the steps of one decoding iteration ------------------------------------------------- */

/* Encoder forward of `model` over B source sentences (x_1..x_n each, no sentinels;
 * `src` is [B, max_src], row b holds src_len[b] ids) and the cross-attention keys/values
 * of every decoder layer.  With model = AD_VERIFIER it also starts a new decode:
 * accepted length 0, pending decoder input [BOS], empty output, per-sequence output
 * limit max_out[b] (NULL: cfg.max_len).  1 <= src_len[b] <= max_src. */
int ad_encode(ad_ctx* ctx, int model, const int32_t* src, const int32_t* src_len, int B,
              const int32_t* max_out);

/* Parallel verification (Section 3.2: the verifier equation, the bifurcation position c
 * and the accepted block; Section 3.1.1 for the input-guided case).  For each sequence b
 * with k[b] > 0 the decoder is fed (o_j, draft[b][0..k[b]-2]) at positions j..j+k[b]-1
 * under a causal mask against its key/value cache; o_hat_i is the arg max (lowest id on
 * ties) at row i; c = first i with draft[b][i-1] != o_hat_i, else k[b].  The block
 * o_hat_1..o_hat_c (= matched draft prefix + first corrected token) is appended to the
 * output, cut after the first [EOS] and at the sequence's output limit; the cache keeps
 * exactly the rows of accepted tokens (rollback), and o_hat of the last appended token
 * becomes the pending decoder input.
 *   draft      [B, k_max] host, row b holds k[b] ids (AD_NEVER allowed last)
 *   k          [B] host, 0 = sequence sits this call out
 *   n_accept   [B] out: tokens appended for b (0 if k[b] = 0)
 *   next_token [B] out: last appended token (undefined if n_accept = 0)
 *   verified   [B, k_max] out, nullable: all o_hat of the call, for tests
 * AD_ESTATE before ad_encode(AD_VERIFIER) or if a finished sequence gets k[b] > 0;
 * AD_EINVAL for k[b] > k_max, ids outside the vocabulary, AD_NEVER not last. */
int ad_verify(ad_ctx* ctx, const int32_t* draft, const int32_t* k,
              int32_t* n_accept, int32_t* next_token, int32_t* verified);

/* ad_verify for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  Same arguments, same results and same effect on the decode
 * state as ad_verify.  The call allocates nothing, on the device or on the host: its kernels are
 * launched one by one (no graph is built or replayed) and the one scratch buffer they need
 * beyond the context's workspace, the per-workgroup arg-max partials of the output projection,
 * lives in a 4 MiB array the library holds statically on every GPU it runs on (until the process
 * ends).  Limit: rows x (vocab / 16) x 8 bytes <= 4 MiB, rows = sum of k[b] (262 rows at vocab
 * 32000); more gives AD_EINVAL and leaves the context as it was.  All contexts on one GPU share
 * that array and it keeps the last call's contents (every word a call reads it has written
 * before, so nothing needs clearing): calls that overlap in time on one GPU race, also from
 * different contexts or streams; serialise them.  AD_ESTATE if the array's address could not be
 * obtained on this device. */
int ad_verify_static(ad_ctx* ctx, const int32_t* draft, const int32_t* k,
                     int32_t* n_accept, int32_t* next_token, int32_t* verified);

/* Block drafter (Section 3.2, draft paragraph; Section 3.2.1): decoder input
 * (o_0..o_j, [MASK] x k) at positions 0..j+k with bidirectional self-attention and
 * cross-attention to the drafter's memory; draft_out[b][i] = arg max at mask row i.
 * All unfinished sequences draft k tokens (k <= k_max; finished rows get AD_NEVER).
 * Needs ad_encode(AD_DRAFTER) and ad_encode(AD_VERIFIER) for the same batch. */
int ad_draft_nat(ad_ctx* ctx, int k, int32_t* draft_out /* [B, k_max] host */);

/* Current output of the decode in progress: out [B, max_len], out_len [B]. */
int ad_output(ad_ctx* ctx, int32_t* out, int32_t* out_len);

/* ---- whole decodes ------------------------------------------------------------------------ */
/* All three take B sources as ad_encode does and write out [B, max_len] / out_len [B];
 * `stats` is nullable.  Their outputs are token-identical by construction. */

/* o_{t+1} = arg max P(. | o_{<=t}, x) one token at a time (Section 2): verify with k = 1. */
int ad_decode_greedy(ad_ctx* ctx, const int32_t* src, const int32_t* src_len, int B,
                     const int32_t* max_out, int32_t* out, int32_t* out_len, ad_stats* stats);

/* Algorithm 1.  The guide x (NULL: the source itself) is [B, guide_stride] with
 * guide_len[b] content ids per row; [BOS] is prepended and the never-matching [PAD]
 * appended internally.  Each iteration looks for the shortest suffix of the output that
 * occurs exactly once in the guide; on a match the rest of the guide (at most k_max
 * tokens) is verified in parallel, otherwise one autoregressive step is taken. */
int ad_decode_iad(ad_ctx* ctx, const int32_t* src, const int32_t* src_len,
                  const int32_t* guide, const int32_t* guide_len, int guide_stride, int B,
                  const int32_t* max_out, int32_t* out, int32_t* out_len, ad_stats* stats);

/* Draft k tokens, verify them, accept through the bifurcation, repeat (Section 3.2).
 * use_drafter != 0 runs the block drafter each iteration (needs drafter weights).
 * draft_override (nullable, [B, override_stride], override_len[b] entries per row) is a
 * positional draft D: output position p is proposed D[b][p]; when given it replaces the
 * drafter's proposal (the drafter, if enabled, still runs). */
int ad_decode_gad(ad_ctx* ctx, const int32_t* src, const int32_t* src_len, int B, int k,
                  int use_drafter, const int32_t* draft_override, const int32_t* override_len,
                  int override_stride, const int32_t* max_out,
                  int32_t* out, int32_t* out_len, ad_stats* stats);

/* ---- inspection ------------------------------------------------------------------------------ */

/* Full logits [rows, vocab] (fp32, host) of the last ad_verify or ad_draft_nat, rows in
 * packed order (sequence by sequence).  Needs cfg.debug_logits; AD_ESTATE otherwise. */
int ad_debug_logits(ad_ctx* ctx, float* logits, int rows_cap, int* rows);

/* Re-launches the kernels of the last ad_verify forward on the context's stream without touching
 * decode state (the appended cache rows are rewritten with the same values) and reports, by HIP
 * events on that stream: forward_us = the whole forward, mean of `reps` forwards back to back;
 * vocab_kernel_us = its output-projection/arg-max kernel, mean over `reps` forwards of one launch
 * bracketed by two events (what a kernel trace reports for it); vocab_back_to_back_us (may be
 * null) = the same kernel, `reps` launches back to back divided by reps (launch overheads of
 * consecutive launches overlap).  For roofline measurements. */
int ad_time_verify_forward(ad_ctx* ctx, int reps, double* forward_us, double* vocab_kernel_us,
                           double* vocab_back_to_back_us);

/* The output-projection/arg-max kernel of the last ad_verify forward, `reps` launches back to back on
 * the context's stream, launch r reading the matrix from copy r % n_copies of `w_copies` (DEVICE
 * memory, the caller's: n_copies images of the verifier's "out.w" entry, copy_stride_bytes apart,
 * a multiple of 16).  With copies that together exceed the GPU's last-level cache every launch
 * streams its matrix from HBM; with one copy it may come from that cache.  Mean microseconds per
 * launch by HIP events.  Results of the launches are discarded; decode state is not touched. */
int ad_time_output_projection(ad_ctx* ctx, const void* w_copies, size_t copy_stride_bytes, int32_t n_copies,
                              int32_t reps, double* us_per_launch);

/* Measurement aid, no part of the method: copies `bytes` (a multiple of 16) from src to dst, both
 * device memory, with one plain kernel (16 bytes per lane per step) on `stream`.  A hardware
 * memory-traffic counter read for this launch, whose traffic is known (`bytes` read, `bytes`
 * written), gives the factor that turns the counter's reading for other kernels into bytes.
 * Returns AD_OK or AD_EINVAL / AD_EDEVICE. */
int ad_calibration_copy(void* dst_dev, const void* src_dev, size_t bytes, void* stream);

/* Measurement aid, no part of the method: the rate at which the whole chip accepts the bf16 matrix
 * instruction the GEMMs and the attention are built on (v_mfma_f32_16x16x32_bf16, fp32 accumulate) when
 * nothing else limits it: 512 workgroups of 4 waves issue iters x 8 independent ones each on fixed
 * register operands, timed by HIP events on `stream`.  `scratch_dev`: at least 512 KiB of device
 * memory (receives values nobody needs).  *tflops: dense TFLOP/s, the measured counterpart of the
 * nominal peak.  Returns AD_OK or AD_EINVAL / AD_EDEVICE. */
int ad_calibration_mfma(void* scratch_dev, size_t scratch_bytes, int32_t iters, void* stream, double* tflops);

/* Launch-style knobs; results never depend on them.  AD_OPT_GRAPHS (0/1, default 1): the
 * launches of an ad_verify call are captured into a HIP graph per call
 * shape (rows, sequences, longest block) on the shape's third appearance and replayed afterwards
 * (at most 512 shapes); the library switches it off by itself when the context's stream cannot be
 * captured (the null stream cannot).  AD_OPT_GRAPHS_CAPTURED (read only): graphs held.
 * AD_OPT_SPIN_WAIT (0/1, default 1): ad_verify returns as soon as the device has written the
 * call's result into the (device-mapped) host staging buffer, which the calling thread watches,
 * instead of waiting for the stream to drain; later calls are ordered behind the unfinished rest
 * of the stream as usual.  After 50 ms without the result it waits for the stream.
 * AD_OPT_FUSE_CROSSQ (0/1, default 1): a decoder layer's
 * cross-attention runs its query projection and the attention as one launch (bf16, head width 64,
 * model width 512 or 1024; other shapes take two launches whatever the setting).  Same results bit
 * for bit either way.
 * AD_OPT_OVERLAP_ENCODERS (0/1, default 1 in contexts with a drafter whose stream is not the null
 * stream; elsewhere 0 and switching it on gives AD_ESTATE): ad_encode(AD_DRAFTER) that follows
 * ad_encode(AD_VERIFIER) runs on a second stream of the library's own (default priority), in a
 * second block of activation buffers, beside the verifier's encoder instead of behind it; the
 * first ad_draft_nat makes the context's stream wait for it.  Same results bit for bit. */
enum { AD_OPT_GRAPHS = 3, AD_OPT_GRAPHS_CAPTURED = 4, AD_OPT_SPIN_WAIT = 5, AD_OPT_FUSE_CROSSQ = 6,
       AD_OPT_OVERLAP_ENCODERS = 7 };
int ad_set_option(ad_ctx* ctx, int option, int value);
int ad_get_option(ad_ctx* ctx, int option, int* value);

/* GAD++, the relaxed verification of Section 3.2.3 (its two inequalities).  With beta > 1, every
 * later ad_verify (and the decode loops built on it) lets a drafted token stand where the
 * verifier ranks it among its top `beta` candidates AND the top-1 log-likelihood exceeds the
 * drafted token's by at most `tau`: verified[b][i] is then the drafted token instead of the arg
 * max, and the bifurcation is the first position whose drafted token meets neither that nor the
 * top-1 match.  Log-likelihood differences are taken as differences of the fp32 output scores
 * (the normaliser cancels); "among the top beta" means fewer than beta tokens score strictly
 * higher, so tokens that tie with the beta-th ranked one are in.  AD_NEVER is never accepted.
 * The output is no longer the greedy one.  beta = 1 (the default) restores top-1 matching;
 * tau is ignored then.  Costs a second pass of the output projection per call.
 * AD_EINVAL: beta outside [1, vocab], tau negative or not finite. */
int ad_set_gadpp(ad_ctx* ctx, int32_t beta, float tau);

/* ---- host-only logic, exposed so that it can be tested without a GPU -------------------------- */

/* The if-test of Algorithm 1: o = (o_0..o_j), x = guide with sentinels (x_0 = [BOS],
 * last = AD_NEVER).  Finds the smallest q >= 0 for which o_{j-q..j} occurs in x; if it
 * occurs exactly once, *i_out = the index in x of its last token and 1 is returned;
 * otherwise (never, or every suffix occurs several times) 0 is returned. */
int ad_suffix_match(const int32_t* o, int o_len, const int32_t* x, int x_len, int* i_out);

/* Runs the library's own decode loops (the same code ad_decode_iad / ad_decode_gad run)
 * over a model-free stand-in verifier that knows the greedy output g[0..g_len): fed a
 * prefix that agrees with g it predicts g's next token, after a disagreement it predicts
 * garbage.  mode 0: input-guided with `aux` = guide content ids; mode 1: positional
 * draft `aux` with block size k.  Writes the output, per-iteration accepted counts
 * (up to acc_cap) and stats. */
int ad_host_simulate(int mode, const int32_t* g, int g_len, const int32_t* aux, int aux_len,
                     int k, int k_max, int max_out, int eos, int bos,
                     int32_t* out, int32_t* out_len, int32_t* accepted, int acc_cap,
                     ad_stats* stats);

#ifdef __cplusplus
}
#endif
#endif /* AD_H_ */

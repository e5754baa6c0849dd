/*
 * dbl.h -- C ABI of libdbl: the target-side verify -> accept -> retrieve -> commit
 * step of Double (Double Retrieval Speculative Parallelism, arxiv 2601.05524) for
 * one AMD MI355X (gfx950).  Every step runs in HIP kernels of this library; there
 * is no CPU fallback.
 *
 * One "Retrieval Forward" (paper Eq. 2) is, per sequence:
 *     dbl_retrieve      d candidate tokens by n-gram match            (Alg. 3)
 *     dbl_build_window  pending token + candidates -> k window rows
 *     dbl_verify_block  one target forward over the k rows            (Sec. 2.1)
 *                       (dbl_verify_block_ragged: windows of different lengths in one batch)
 *     dbl_accept        s matched tokens + 1 correction               (Sec. 2.1, App. D.2)
 *     dbl_kv_commit     keep the accepted rows' KV, extend the history (Alg. 1, Alg. 2)
 *
 * Conventions
 *   - "dev" pointers are device memory the CALLER allocated on the context's GPU
 *     and keeps owning; "host" pointers are ordinary host memory.  The library
 *     never frees caller memory and does not keep caller pointers after the
 *     stream work of the call that received them has finished.
 *   - The context owns weights, KV cache, token history, per-sequence counters
 *     and all scratch.  B sequences (0 <= b < B <= max_batch) advance in lockstep
 *     (with dbl_verify_block_ragged a sequence may bring a shorter window or sit a step out).
 *   - The hot calls (retrieve, build_window, verify_block, accept, kv_commit) only
 *     enqueue work on the context's stream and return; results are valid once the
 *     caller has synchronised that stream.  Counters (kv_len, hist_len, n_acc) stay
 *     on the device, so the five calls chain without a host round trip.
 *   - Window convention: window[b][0] is the pending token (emitted by the last
 *     step, its KV not yet written); window[b][1..k) are k-1 drafted tokens.
 *     Row j sits at position kv_len[b]+j and its logits predict the token after
 *     window[b][j].  Verifying gamma drafts is k = gamma+1.
 *   - All functions return 0 (DBL_OK) or a negative dbl_status.  Argument checks
 *     come before any GPU call.  Nothing throws or aborts across this boundary.
 *   - Calls on one context are not thread-safe.
 *   - Measurement, diagnostics and tuning entry points (no part of a step) are declared in dbl_diag.h.
 */
#ifndef DBL_H
#define DBL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dbl_ctx dbl_ctx;

typedef enum {
  DBL_OK = 0,
  DBL_EINVAL = -1, /* bad argument: null pointer, size out of range, bad enum      */
  DBL_ESTATE = -2, /* call out of order (accept without verify_block, ...)         */
  DBL_ENOMEM = -3, /* host or device allocation failed                             */
  DBL_EHIP = -4,   /* a HIP runtime call failed; text in dbl_last_error            */
  DBL_ENODEV = -5  /* validate-only context: arguments were fine, nothing was run  */
} dbl_status;

enum { DBL_F32 = 0, DBL_BF16 = 1 };
enum { DBL_GREEDY = 0, DBL_SAMPLE = 1 };
enum {
  DBL_FLAG_VALIDATE_ONLY = 1, /* dbl_model_cfg.flags: no GPU is touched                */
  DBL_FLAG_PAGED_KV = 2       /* KV cache as a pool of 256-token pages, see dbl_create  */
};

/* Tensor ids for dbl_set_weights / dbl_get_weights.  Matrices are logical
 * row-major [out_features][in_features]. */
enum {
  DBL_T_EMB = 0,  /* [vocab][d_model]                 */
  DBL_T_LM = 1,   /* [vocab][d_model]  (untied)       */
  DBL_T_GF = 2,   /* final RMSNorm gain [d_model] f32 */
  DBL_T_G1 = 10,  /* pre-attention RMSNorm gain [d_model] f32 */
  DBL_T_WQ = 11,  /* [n_q_heads*head_dim][d_model]    */
  DBL_T_WK = 12,  /* [n_kv_heads*head_dim][d_model]   */
  DBL_T_WV = 13,  /* [n_kv_heads*head_dim][d_model]   */
  DBL_T_GQ = 14,  /* per-head q RMSNorm gain [head_dim] f32 (qk_norm) */
  DBL_T_GK = 15,  /* per-head k RMSNorm gain [head_dim] f32 (qk_norm) */
  DBL_T_WO = 16,  /* [d_model][n_q_heads*head_dim]    */
  DBL_T_G2 = 17,  /* pre-MLP RMSNorm gain [d_model] f32 */
  DBL_T_WG = 18,  /* gate [d_ffn][d_model]            */
  DBL_T_WU = 19,  /* up   [d_ffn][d_model]            */
  DBL_T_WD = 20   /* down [d_model][d_ffn]            */
};

/* Decoder shape (the paper's model table, App. C.1, gives layers / dim / FFN dim /
 * vocabulary; head counts are the public ones of those models) and capacities. */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rms_eps, rope_base;
  int32_t qk_norm; /* 1: per-head RMSNorm on q and k before RoPE (Qwen3)           */
  int32_t dtype;   /* DBL_F32 or DBL_BF16: type of weights, KV cache and of the
                      activations that feed projections; accumulation, residual
                      stream, norms, softmax and logits are always fp32           */
  int32_t max_batch, max_ctx, max_window, max_hist;
  int32_t flags;
} dbl_model_cfg;

/*
 * Create a context on the current HIP device.  Weights are generated on the GPU
 * from `weight_seed`: every matrix / embedding entry is 0.02 * (sum of the eight
 * 16-bit halves of Philox4x32-10(counter = {elem_lo, elem_hi, tensor id, layer},
 * key = seed) - 262140) / sqrt(8*(65536^2-1)/12), rounded to the model dtype;
 * every norm gain is 1.  `hip_stream` (a hipStream_t, NULL = default stream) is
 * borrowed: all later work of this context is enqueued on it.
 * Limits: head_dim in {64, 128}; n_q_heads % n_kv_heads == 0;
 * 1 <= max_window <= 32; max_batch*max_window <= 128; max_ctx % 64 == 0.
 * KV cache: by default one region of max_ctx positions per sequence.  With
 * DBL_FLAG_PAGED_KV (higher concurrency, App. D.1: many sequences of very different
 * lengths) it is a pool of pages of 256 positions shared by all sequences; flags >> 8 is the
 * number of pages (0: max_batch * max_ctx / 256, i.e. no saving), max_ctx % 256 == 0 is
 * required and max_ctx only bounds one sequence.  The library hands a sequence its pages when a
 * call needs them (dbl_verify_block, dbl_kv_fill: DBL_ENOMEM "KV page pool exhausted" when none
 * is left, nothing is enqueued then) and takes them back in dbl_reset and dbl_truncate; results do
 * not depend on the cache form.  Page hand-outs enqueue one small kernel each, so a captured
 * graph must not contain a call that crosses a page boundary for the first time.
 */
int dbl_create(const dbl_model_cfg* cfg, uint64_t weight_seed, void* hip_stream, dbl_ctx** out);
int dbl_destroy(dbl_ctx* ctx);

/* Text of the last error of this context (never NULL; "" if none). */
const char* dbl_last_error(const dbl_ctx* ctx);

/* Overwrite / read back one tensor.  `host` holds the logical row-major tensor in
 * the model dtype (bf16 as uint16_t bit patterns, or float); norm gains are always
 * float.  `bytes` must equal the tensor's size.  The library repacks into its own
 * layout.  Synchronises the stream. */
int dbl_set_weights(dbl_ctx* ctx, int tensor_id, int layer, const void* host, size_t bytes);
int dbl_get_weights(dbl_ctx* ctx, int tensor_id, int layer, void* host, size_t bytes);

/* Session flush (the paper's datastore is session-scoped, App. D.3): sequence
 * `seq` (or every sequence when seq < 0) gets kv_len = hist_len = 0 and an empty
 * rejected tier. */
int dbl_reset(dbl_ctx* ctx, int seq);

/* Measurement aid (bandwidth runs at contexts too long to prefill): pretend that the first
 * n_tokens positions of sequence `seq` are committed.  Their K and V rows get seeded values of
 * unit scale in every layer (not the model's own keys and values) and kv_len[seq] = n_tokens;
 * the history is not touched.  0 <= n_tokens <= max_ctx - max_window.  Only enqueues. */
int dbl_kv_fill(dbl_ctx* ctx, int seq, int32_t n_tokens, uint64_t seed);

/* Read / overwrite the cached keys and values of rows pos0 .. pos0+n-1 of sequence `seq` in one layer
 * (restoring a stored prefix cache; tests compare the cache with the oracle's and plant known rows).
 * host_k / host_v: [n][n_kv_heads][head_dim] in the model dtype (bf16 as uint16_t bit patterns, or float):
 * the keys as the cache holds them (after q/k-norm and RoPE) and the values.  The library converts from /
 * to its own tiled (or paged) layout.  kv_len is not touched: rows at or beyond it are dead until a commit
 * or dbl_kv_fill covers them.  0 <= pos0, pos0 + n <= max_ctx; a paged cache hands the sequence the pages
 * dbl_kv_set needs (DBL_ENOMEM when the pool is empty), dbl_kv_get needs them to be there.  Both allocate a
 * staging buffer and synchronise: set-up calls, not part of a step. */
int dbl_kv_set(dbl_ctx* ctx, int seq, int layer, int32_t pos0, int32_t n, const void* host_k, const void* host_v);
int dbl_kv_get(dbl_ctx* ctx, int seq, int layer, int32_t pos0, int32_t n, void* host_k, void* host_v);

/* Rollback (Alg. 1 "rollback M_q", Alg. 2 "rollback both models"): sequence `seq`
 * forgets the KV rows beyond kv_len and the history tokens beyond hist_len:
 * kv_len[seq] = min(kv_len[seq], kv_len), hist_len[seq] = min(hist_len[seq], hist_len);
 * a negative argument leaves that counter as it is.  Nothing is erased: the rows and
 * tokens are overwritten by later calls.  Only enqueues on the context's stream. */
int dbl_truncate(dbl_ctx* ctx, int seq, int32_t kv_len, int32_t hist_len);

/* Replace the token history of sequence `seq` by `n` host tokens (the prompt).
 * The history is what dbl_retrieve searches; it normally ends with the pending
 * token, i.e. hist_len = kv_len + 1.  0 <= n <= max_hist. */
int dbl_history_set(dbl_ctx* ctx, int seq, const int32_t* host_tokens, int n);

/* Copy the history of sequence `seq` to the host: min(hist_len, cap) tokens into
 * host_out, hist_len into *n_out.  Synchronises the stream. */
int dbl_history_get(dbl_ctx* ctx, int seq, int32_t* host_out, int cap, int32_t* n_out);

/*
 * Retrieval (Alg. 3's descending n-gram search of the sequence in itself; Eq. 2's
 * "retrieve d tokens").  For each sequence b < B: for n = min(n_max, len-1) down
 * to n_min, every start s <= len-n-1 with hist[s..s+n) == hist[len-n..len) is a
 * candidate whose continuation is the next min(max_cont, len-s-n) tokens; the
 * first n with a candidate wins, then the longest continuation, then the latest s.
 * Outputs (dev): cont[B][max_cont] (entries beyond cont_len are -1), cont_len[B],
 * match_n[B] (0 = miss), match_pos[B] (-1 = miss).
 * 1 <= n_min <= n_max <= 32, 1 <= max_cont <= 64.
 */
int dbl_retrieve(dbl_ctx* ctx, int B, int n_max, int n_min, int max_cont, int32_t* cont_dev,
                 int32_t* cont_len_dev, int32_t* match_n_dev, int32_t* match_pos_dev);

/*
 * Hierarchical datastore (Sec. 4.3, Alg. 3 "Retrieval Cache Mechanism").  Tiers, searched in
 * this priority for every n-gram length, longest length first:
 *   0  the prior: a static token stream shared by all sequences (dbl_prior_set);
 *   1  the session's generated text: the history beyond what dbl_history_set put there;
 *   2  the session's rejected draft chains (dbl_rejected_update);
 * and only if no length hits in any of them
 *   3  the plain search of the sequence in itself (what dbl_retrieve does).
 * A tier is a token buffer in which -1 separates segments: an n-gram never contains a
 * separator and a continuation stops in front of one.  Inside a tier: longest continuation
 * (<= max_cont), then the latest occurrence.  Outputs as dbl_retrieve, plus match_tier[B]
 * (-1 = miss); match_pos is the n-gram's start inside its tier's buffer.
 */
int dbl_retrieve_tiered(dbl_ctx* ctx, int B, int n_max, int n_min, int max_cont, int32_t* cont_dev,
                        int32_t* cont_len_dev, int32_t* match_n_dev, int32_t* match_pos_dev,
                        int32_t* match_tier_dev);

/*
 * dbl_retrieve_tiered for callers that cannot allocate and want no allocated scratch behind the call:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same results, same stream behaviour; the difference is where the search keeps its one piece of scratch
 * (one packed best key per sequence): not in memory the context allocated, but in a fixed array that is
 * part of the loaded library on every GPU it runs on (DBL_STATIC_MAX_BATCH x 8 bytes per GPU, held until
 * the process ends; its device address is looked up once per device, in dbl_create).  The call allocates
 * and frees nothing, runs no allocating library routine and records no memset: it enqueues one small fill
 * kernel (the array keeps the previous call's contents and is cleared first) and the two search kernels.
 * B > DBL_STATIC_MAX_BATCH is rejected with DBL_EINVAL.  All contexts on one GPU share the array: calls
 * that overlap on one GPU (two streams, two contexts) race on it -- run them one after the other.
 */
#define DBL_STATIC_MAX_BATCH 128
int dbl_retrieve_tiered_static(dbl_ctx* ctx, int B, int n_max, int n_min, int max_cont, int32_t* cont_dev,
                               int32_t* cont_len_dev, int32_t* match_n_dev, int32_t* match_pos_dev,
                               int32_t* match_tier_dev);

/* Mark the first prompt_len tokens of sequence `seq`'s history as the prompt; what follows
 * counts as the session's generated text (tier 1).  dbl_history_set marks all it sets as
 * prompt; this call is for a caller that restores a running session.  0 <= prompt_len;
 * clamped to the history length.  Synchronises. */
int dbl_session_mark(dbl_ctx* ctx, int seq, int32_t prompt_len);

/* Replace the prior tier by n host tokens (ids >= 0, or -1 as separator); n = 0 clears it.
 * Allocates device memory and synchronises: a set-up call, not part of a step. */
int dbl_prior_set(dbl_ctx* ctx, const int32_t* host_tokens, int n);

/* Alg. 3's cache update for the rejected tier; call between dbl_accept and dbl_kv_commit.
 * For every sequence of the last verified window (pending token + drafts), the drafts behind
 * the first rejection, window[n_acc+1 .. n_draft[b]], are appended to its rejected tier as
 * one segment: up to DBL_REJ_CTX tokens of the text in front of them (history, then the
 * accepted drafts), the rejected tokens, a separator.  n_draft_dev (dev, [B]) = number of
 * real drafts in the window (e.g. the cont_len a retrieval returned; clamped to 0..k-1);
 * NULL = k-1.  A segment that does not fit (capacity max_hist tokens per sequence) is
 * dropped.  dbl_reset empties the tier.  Only enqueues. */
#define DBL_REJ_CTX 4
int dbl_rejected_update(dbl_ctx* ctx, const int32_t* n_draft_dev);

/* Copy the rejected tier of sequence `seq` to the host (min(length, cap) tokens), length
 * into *n_out.  Synchronises. */
int dbl_rejected_get(dbl_ctx* ctx, int seq, int32_t* host_out, int cap, int32_t* n_out);

/* window[b][0] = last history token of b; window[b][1+i] = cont[b][i] for
 * i < min(cont_len[b], k-1), else pad_id.  cont rows have stride max_cont.
 * window_dev is [B][k].  Sequences with an empty history get pad_id in row 0. */
int dbl_build_window(dbl_ctx* ctx, int B, int k, int max_cont, const int32_t* cont_dev,
                     const int32_t* cont_len_dev, int32_t pad_id, int32_t* window_dev);

/*
 * The full Double round (Sec. 4.1 "Synchronous Parallel Execution", Sec. 4.2 "Target-Guided Verification",
 * Eq. 6, Alg. 1 / Alg. 2): a draft model and a target model as two contexts on two streams.  The calls below
 * keep every token of a round on the device; the caller enqueues them and synchronises once per round.
 * Per round, with x the text the target has verified and U the drafts behind it that it has not:
 *   target:  dbl_build_guided_window -> dbl_verify_block -> dbl_accept -> dbl_kv_commit      (x grows by E)
 *   draft:   gamma Retrieval Forwards from x + U (the calls at the top of this file), dbl_history_tail = X_q
 *   resolve: dbl_merge (needs both) -> dbl_history_splice on the draft -> next round's U
 *
 * dbl_build_guided_window: window[b] = pending token (last token of the history), then the n_ahead[b] unverified
 * drafts ahead[b][..] (dev, [B][max_ahead]; NULL with n_ahead NULL = none), then the target's own retrieved guidance
 * Y_p: the continuation dbl_retrieve's rule finds for the end of history + ahead, searched in history + ahead, at most
 * min(d, free rows) tokens; then pad_id up to k rows.  n_draft_dev[b] = drafts + guidance tokens in the window.
 * Nothing is written to the history.  n_ahead is clamped to 0..min(k-1, max_ahead).
 */
int dbl_build_guided_window(dbl_ctx* ctx, int B, int k, const int32_t* ahead_dev, const int32_t* n_ahead_dev, int max_ahead,
                            int n_max, int n_min, int d, int32_t pad_id, int32_t* window_dev, int32_t* n_draft_dev);

/*
 * Eq. 6 on the device, per sequence b.  In (dev): n_u[b] = |U| (drafts at the front of the target's window),
 * n_acc[b] and emit[b][k] as dbl_accept wrote them (E = emit[b][0..n_acc]: accepted window tokens + the target's own
 * next token), chain[b][max_chain] / n_chain[b] = X_q, the draft model's new tokens, which continue x + U, and
 * base_len[b] = length of the draft's history when that chain began (|x| + |U|; may be NULL).
 * The verified text grows by E in every case.  U' (the next round's unverified drafts) is empty if a token of U was
 * rejected (n_acc < n_u), if X_q differs from G = E[n_u..] somewhere, or if X_q ends inside G: then the target's tokens
 * stand (verified draft prefix + target suffix).  Otherwise U' = the tokens of X_q behind G, at most max_u.
 * Out (dev): u_out[b][max_u] (-1 beyond |U'|), n_u_out[b]; text_out[b][k + max_u] = E + U' and n_text_out[b]: what now
 * follows the old verified text; splice_pos[b] = base_len[b] - n_u[b] (0 without base_len): where that text starts in
 * the draft's history; record[b][8] = {n_u, n_acc, |E|, |X_q|, |U'|, leading tokens of X_q equal to G, length of the
 * draft's old text behind x that is still valid, 0}.  Only enqueues on ctx's stream (any context of the device will
 * do: nothing of the context is read).  1 <= k <= 32, 1 <= max_chain <= 4096, 1 <= max_u <= 64.
 */
int dbl_merge(dbl_ctx* ctx, int B, int k, const int32_t* n_u_dev, const int32_t* n_acc_dev, const int32_t* emit_dev,
              const int32_t* chain_dev, const int32_t* n_chain_dev, int max_chain, int max_u, const int32_t* base_len_dev,
              int32_t* u_out_dev, int32_t* n_u_out_dev, int32_t* text_out_dev, int32_t* n_text_out_dev,
              int32_t* splice_pos_dev, int32_t* record_dev);

/* tokens_out[b][0..n) = history tokens from position from_dev[b] to the end, n = min(their number, max_n) into
 * n_out[b]; entries beyond n are -1.  Only enqueues.  1 <= max_n <= 4096. */
int dbl_history_tail(dbl_ctx* ctx, int B, const int32_t* from_dev, int max_n, int32_t* tokens_out_dev, int32_t* n_out_dev);

/* Rollback and re-alignment in one step (Alg. 1 "rollback M_q", Alg. 2 "rollback both models"): the history of
 * sequence b becomes its first pos[b] tokens followed by tokens[b][0..n[b]) (dev, [B][max_n]).  KV rows of tokens that
 * did not change are kept; kv_len[b] = min(kv_len[b], first position that changed, new length - 1).
 * missing_out[b] (may be NULL) = tokens between the cache and the last token, whose KV a forward has to compute
 * (dbl_catchup_window builds that forward's window).  Only enqueues.  1 <= max_n <= 128. */
int dbl_history_splice(dbl_ctx* ctx, int B, const int32_t* pos_dev, const int32_t* tokens_dev, const int32_t* n_dev, int max_n,
                       int32_t* missing_out_dev);

/* window[b][j] = the history tokens at positions kv_len[b] + j that lie in front of the last token, at most k, then
 * pad_id; win_len[b] = their number.  Run dbl_verify_block_ragged on it and dbl_kv_commit(win_len) to bring the cache
 * up to the history again.  Only enqueues. */
int dbl_catchup_window(dbl_ctx* ctx, int B, int k, int32_t pad_id, int32_t* window_dev, int32_t* win_len_dev);

/* Copy the device-side counters kv_len[0..B) / hist_len[0..B) into caller buffers on the device (either may be NULL),
 * in stream order, without synchronising. */
int dbl_lengths_dev(dbl_ctx* ctx, int B, int32_t* kv_len_out_dev, int32_t* hist_len_out_dev);

/*
 * Verify forward (Sec. 2.1: one parallel target forward over the drafted tokens;
 * App. D.2: causal mask, row j conditioned on the prefix and rows < j).
 * window_dev is [B][k] token ids in [0, vocab).  For every row: embedding, n_layers
 * x [RMSNorm, q/k/v projections, (qk_norm), RoPE at position kv_len[b]+j, K/V
 * written to cache slot kv_len[b]+j, GQA attention over slots 0..kv_len[b]+j,
 * output projection + residual, RMSNorm, SwiGLU MLP + residual], final RMSNorm,
 * LM head.  The LM-head kernel also leaves, per row, the statistics dbl_accept
 * needs (arg-max; and when temperature > 0: log-sum-exp of logits/temperature, the
 * draft token's logit and the two largest Gumbel-perturbed scores, noise from
 * Philox4x32-10 keyed by `seed` with counter {step', b, j, 1 + v/4}, word v%4,
 * where step' = step + number of dbl_kv_commit calls this context has run).
 * kv_len is not advanced.  logits_opt_dev, if not NULL, receives the fp32 logits
 * [B][k][vocab].  (The library itself keeps the logits of a call only if logits_opt_dev is given or
 * temperature > 0 -- the one later reader is dbl_accept's residual draw under dense draft distributions;
 * a greedy step with logits_opt_dev == NULL writes no logits at all, only the row statistics.)  1 <= B <= max_batch, 1 <= k <= max_window, and for every b
 * kv_len[b] + k <= max_ctx (checked against the host's upper bound of kv_len).
 * temperature <= 0 means "greedy statistics only".
 * The step's calls (retrieve, build_window, verify_block, accept, kv_commit) only enqueue
 * kernels and one device-to-device copy, so they can be captured into a HIP graph and
 * replayed; the Philox step word advances with the device-side commit counter.  Replays
 * do not advance the host's upper bounds: the device clamps at max_ctx / max_hist and
 * raises the status word that dbl_kv_len / dbl_hist_len report.
 */
int dbl_verify_block(dbl_ctx* ctx, const int32_t* window_dev, int B, int k, float temperature,
                     uint64_t seed, uint64_t step, float* logits_opt_dev);

/*
 * The same forward for windows of different lengths in one batch (the higher-concurrency
 * regime of App. D.1: sequences with different numbers of drafts, or none, share a step).
 * win_len_dev[b] (device, int32, clamped to 0..k) is the number of real rows of sequence b:
 * its pending token and win_len[b]-1 drafts.  Rows beyond it are computed (all B*k rows run,
 * the projections are bound by the weights, not by the rows) but count as "no draft":
 * dbl_accept accepts at most win_len[b]-1 drafts and emits at most win_len[b] tokens, and
 * their logits are meaningless.  win_len[b] = 0 leaves sequence b untouched by the step:
 * dbl_accept reports n_acc[b] = -1 and emits nothing, dbl_kv_commit keeps nothing.
 * Every sequence still needs room for k rows (kv_len[b] + k <= max_ctx).  Everything else
 * as dbl_verify_block, including ownership, capture and error behaviour.
 */
int dbl_verify_block_ragged(dbl_ctx* ctx, const int32_t* window_dev, const int32_t* win_len_dev, int B, int k,
                            float temperature, uint64_t seed, uint64_t step, float* logits_opt_dev);

/*
 * Acceptance on the rows of the last dbl_verify_block (same B, k, window).
 * mode DBL_GREEDY (App. D.2): y_j = argmax of row j (lowest id on ties); n_acc =
 * number of leading drafts with window[j+1] == y_j; emit = those drafts then
 * y_{n_acc}; guide[j] = y_j for all j.
 * mode DBL_SAMPLE (Sec. 2.1; needs temperature > 0 in verify_block): p_j =
 * softmax(logits_j / temperature); draft x = window[j+1] is accepted iff
 * u_j * q_j(x) < p_j(x), u_j = ((w >> 9) + 0.5) / 2^23 with w = word 0 of
 * Philox(counter {step', b, j, 0}); q_probs_dev [B][k-1][vocab] (fp32) are the
 * draft distributions, NULL = deterministic (retrieved) drafts, q one-hot.  At the
 * first rejected row n the emitted token is drawn from max(0, p_n - q_n) (from p_n
 * if that is all zero); with no rejection the extra token is drawn from p_{k-1}.
 * Draws are argmax_v [log weight_v + Gumbel_v] with the noise described above.
 * guide[j] is row j's own draw from p_j for j <= n_acc and -1 after it (guidance
 * behind a rejection is discarded, Sec. 5.3 / App. D.2).
 * Outputs (dev): n_acc[B], emit[B][k] (entries beyond n_acc are -1), guide[B][k].
 */
int dbl_accept(dbl_ctx* ctx, int mode, const float* q_probs_dev, int32_t* n_acc_dev,
               int32_t* emit_dev, int32_t* guide_dev);

/*
 * Commit (Alg. 1 "rollback", Alg. 2): keep the KV of the first n_keep[b] window
 * rows (kv_len[b] += n_keep[b]; later rows are dead and get overwritten) and
 * append emit[b][0..n_keep[b]) of the last dbl_accept to the history.
 * n_keep_dev == NULL means n_keep[b] = n_acc[b] + 1 from the last dbl_accept.
 * With an explicit n_keep_dev (dev, [B], clamped to 0..k) only kv_len advances and
 * nothing is appended to the history (chunked prefill is verify_block + kv_commit
 * with n_keep = k, the history having been set beforehand).
 */
int dbl_kv_commit(dbl_ctx* ctx, const int32_t* n_keep_dev);

/* Synchronises the stream and copies kv_len[0..max_batch) / hist_len to the host;
 * also refreshes the host-side upper bounds used for argument checks.  Returns
 * DBL_ESTATE if a device-side capacity check (max_ctx, max_hist) had to clamp since the
 * last report; the condition is reported once (and forgotten by dbl_reset of all sequences). */
int dbl_kv_len(dbl_ctx* ctx, int32_t* host_out);
int dbl_hist_len(dbl_ctx* ctx, int32_t* host_out);

/* Read-only facts about the layout, for measurement: bytes of weights the verify
 * step streams once per call (all layer matrices + LM head), and KV bytes per
 * cached token (all layers). */
int dbl_model_bytes(const dbl_ctx* ctx, uint64_t* weight_bytes, uint64_t* kv_bytes_per_token);




#ifdef __cplusplus
}
#endif
#endif /* DBL_H */

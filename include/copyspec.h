/*
 * copyspec.h - C ABI of libcopyspec: the CopySpec copy-and-verify step on one MI355X.
 *
 * CopySpec (arXiv 2502.08923) speeds up greedy decoding by looking for an earlier
 * occurrence of the last gamma generated tokens in the context, copying the k tokens
 * that followed it as a draft, and verifying the draft with one forward pass of the
 * target model (Sec. 3.1-3.2, App. B).  This library is that step, as hand-written HIP
 * kernels for gfx950, behind plain C entry points.
 *
 * Conventions
 *   - Indices are 0-based.  A history is h[0..n).  gamma = match length, k = copy block
 *     size (|S_copyspec| in Sec. 3.2, m in App. B.1), tau = number of accepted drafts
 *     (App. B.1 calls it k; renamed to avoid the clash), L = valid KV length of a stream.
 *   - "host" / "device" in a parameter comment says where the pointer must point.
 *     Device pointers must be valid on the current HIP device.  `stream` is a
 *     hipStream_t passed as void* (NULL = the default stream).  Device entry points
 *     enqueue work on `stream` and return without synchronising unless stated.
 *   - The caller owns every buffer it passes.  The library owns what its handles point to
 *     (cs_model, cs_kv) and frees it in the matching *_destroy.
 *   - Return values: CS_OK (0) or a negative cs_status.  cs_last_error() returns a
 *     thread-local description of the most recent failure.  On an argument or capacity
 *     error nothing has been modified.
 *   - Calls on one handle are not re-entrant; calls that share a handle on different
 *     streams race.  Different handles are independent: each cs_kv carries the scratch of its
 *     own match scans, each cs_model its own workspace, so two models with their caches may
 *     step on two streams (or from two threads) at the same time.  The handle-less
 *     cs_find_match_batch_dev keeps one scratch buffer per (device, stream) it was ever called
 *     on: calls on different streams may overlap, calls on one stream are ordered by it.  That
 *     buffer is allocated by the first call on a stream and replaced by a larger one when a
 *     later call needs it (which waits for that stream only); buffers live until the process
 *     ends.  Only the instrumentation (cs_profile_*) is process-wide.
 */
#ifndef COPYSPEC_H
#define COPYSPEC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum cs_status {
    CS_OK = 0,
    CS_NO_MATCH = -1,    /* only as a position value, never as a status */
    CS_E_ARG = -2,       /* NULL pointer, gamma < 1, k < 0, size out of range ... */
    CS_E_CAPACITY = -3,  /* KV cache or history buffer too small for the request */
    CS_E_DEVICE = -4,    /* a HIP call failed; text in cs_last_error() */
    CS_E_STATE = -5,     /* handle used in a state the call does not allow */
    CS_E_UNSUPPORTED = -6, /* shape or values outside what the kernels are built for */
    CS_E_RANGE = -7      /* a synchronous loop finished, but activations left the float16 range of the
                            projections and were saturated (see cs_model_range_status) */
} cs_status;

enum { CS_POLICY_RIGHTMOST = 0, CS_POLICY_FIRST = 1, CS_POLICY_CONTEXT = 2 };
enum { CS_F32 = 0, CS_BF16 = 1 };

const char* cs_last_error(void);
/* Library version string (static storage). */
const char* cs_version(void);

/* ------------------------------------------------------------------------------------
 * Match search and draft extraction  (Sec. 3.1; Sec. 3.2 first paragraph and footnote;
 * App. B.1, the definitions of the match location p and the chunk size m; App. B.3 step 1)
 *
 *   M = { p : 0 <= p <= n - 2*gamma  and  h[p+j] == h[n-gamma+j] for all 0 <= j < gamma }
 *
 * The bound p <= n - 2*gamma is App. B.3 step 1c (the earlier occurrence must end before
 * the query suffix starts).  match_pos = max M (CS_POLICY_RIGHTMOST), min M
 * (CS_POLICY_FIRST), or (CS_POLICY_CONTEXT) the p in M whose preceding tokens agree longest
 * with the tokens preceding the suffix -- the largest e <= min(64, p) with
 * h[p-j] == h[n-gamma-j] for 1 <= j <= e, the rightmost p among equal e; this is one concrete
 * form of the candidate ranking the paper's Limitations section leaves to future work.
 * The policy never changes the emitted tokens, only which draft is proposed.
 * src_pos = match_pos + gamma is the first token to copy;
 * draft[i] = h[src_pos + i] for i < draft_len = min(k, n - src_pos).  If M is empty or
 * n < 2*gamma: match_pos = src_pos = -1, draft_len = 0.  Unused draft slots are set to -1.
 * The paper finds p with a hash map of all gamma-grams; this library scans the history,
 * which returns the same p.
 * ---------------------------------------------------------------------------------- */

/* One history in host memory; copies it to the device, scans, waits.  Returns src_pos
 * (>= gamma), -1 if there is no match, or a cs_status <= -2. Rightmost policy. */
int64_t cs_find_match(const int32_t* history /*host [len]*/, int64_t len, int32_t gamma);

/* As above with every output.  Any output pointer may be NULL.  draft: host [k]. */
int cs_find_match_ex(const int32_t* history /*host [len]*/, int64_t len, int32_t gamma,
                     int32_t k, int32_t policy, int64_t* match_pos, int64_t* src_pos,
                     int32_t* draft /*host [k]*/, int32_t* draft_len);

/* B histories resident on the device: stream b is d_hist[b*stride .. b*stride + d_len[b]).
 * Outputs (device): d_match_pos[B] (may be NULL), d_src_pos[B] (may be NULL),
 * d_draft[B][k], d_draft_len[B].  Requires 1 <= gamma <= 16, 0 <= k <= 256, B >= 0,
 * stride >= every length, B <= 65535.  B == 0 is a no-op.  Asynchronous on `stream` (see the
 * conventions above for its scratch buffer). */
int cs_find_match_batch_dev(const int32_t* d_hist /*device*/, int64_t stride,
                            const int32_t* d_len /*device [B]*/, int32_t B, int32_t gamma,
                            int32_t k, int32_t policy, int32_t* d_match_pos, int32_t* d_src_pos,
                            int32_t* d_draft, int32_t* d_draft_len, void* stream);

/* cs_find_match_batch_dev for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels,
 * same results; it calls no hipMalloc / hipFree or any other allocating routine.  The per-chunk
 * keys of the scan, which the call above keeps in allocated buffers, live in a fixed array of
 * CS_NOALLOC_MAX_CHUNKS 64-bit keys (512 KiB) inside the library's device image, held by every GPU
 * the library runs on until the process ends.  Limit: B * ceil(stride / 4096) <=
 * CS_NOALLOC_MAX_CHUNKS (e.g. 64 histories of 4 M tokens, or 8192 of 32768), otherwise
 * CS_E_CAPACITY and nothing is launched.  All calls on one GPU share that GPU's array: calls
 * that overlap in time on one GPU (different streams or threads) race; calls on one stream are
 * ordered by it.  Nothing needs clearing between calls (every key a call reads it has written
 * itself).  Asynchronous on `stream`. */
#define CS_NOALLOC_MAX_CHUNKS 65536
int cs_find_match_batch_dev_noalloc(const int32_t* d_hist /*device*/, int64_t stride,
                                    const int32_t* d_len /*device [B]*/, int32_t B, int32_t gamma,
                                    int32_t k, int32_t policy, int32_t* d_match_pos,
                                    int32_t* d_src_pos, int32_t* d_draft, int32_t* d_draft_len,
                                    void* stream);

/* ------------------------------------------------------------------------------------
 * Gamma-gram index  (Sec. 3.1: the dictionary that maps every gamma-token subsequence to the
 * places where it occurs and grows with the sequence; App. B.1, dictionary D; App. B.3 steps
 * 1b and 2d)
 *
 * The paper's own data structure as an alternative to the scan, for very long histories:
 * one hash table per stream on the device, keyed by the gamma tokens themselves (entries
 * are verified against the history, so results never depend on hash collisions).  At history
 * length n it holds the grams starting at p <= n - 2*gamma, the candidates App. B.3 step 1c
 * admits; each call first inserts the grams that became admissible since the previous call,
 * then looks up the last gamma tokens.  Results equal cs_find_match_batch_dev for
 * CS_POLICY_RIGHTMOST and CS_POLICY_FIRST (other policies: CS_E_UNSUPPORTED).
 * Histories may only grow between calls, and tokens already indexed must not change; call
 * cs_index_reset otherwise.  gamma is fixed at creation; max_len bounds stride.
 * max_new_positions: upper bound on how many tokens any stream gained since the previous
 * call (max_len for the first call); it only sizes the launch.  Asynchronous on `stream`;
 * calls on one index must be ordered on one stream.
 * ---------------------------------------------------------------------------------- */
typedef struct cs_index cs_index;
int cs_index_create(int32_t B, int64_t max_len, int32_t gamma, cs_index** out);
void cs_index_destroy(cs_index*);
int cs_index_reset(cs_index*, void* stream);
int cs_index_find_match_batch_dev(cs_index*, const int32_t* d_hist /*device*/, int64_t stride,
                                  const int32_t* d_len /*device [B]*/, int64_t max_new_positions,
                                  int32_t k, int32_t policy, int32_t* d_match_pos,
                                  int32_t* d_src_pos, int32_t* d_draft, int32_t* d_draft_len,
                                  void* stream);

/* ------------------------------------------------------------------------------------
 * Target model  (Sec. 4.1 names the families: Llama-3.1 / Qwen2.5 style decoders; the
 * paper does not restate the architecture).  Pre-norm decoder: RMSNorm, rotary position
 * embedding (rotate-half pairing of (j, j + head_dim/2), angle pos * theta^(-2j/head_dim)),
 * grouped-query attention (query head g uses KV head g / (n_heads/n_kv_heads)), SwiGLU
 * FFN, untied lm_head, no biases.
 * ---------------------------------------------------------------------------------- */

typedef struct cs_model_cfg {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ff, vocab;
    int32_t dtype;        /* CS_F32 or CS_BF16: storage type of weight matrices and KV cache */
    float rope_theta;
    float rms_eps;
    int32_t max_batch;    /* most streams one verify call will carry */
    int32_t max_k;        /* largest copy block k a verify call will carry */
} cs_model_cfg;

/* Linear weights are row-major [out_features][in_features] in cfg.dtype; norm gains are
 * float32 [d_model].  All pointers are device pointers. */
typedef struct cs_layer_weights {
    const void *wq, *wk, *wv;   /* [n_heads*hd][d], [n_kv_heads*hd][d], [n_kv_heads*hd][d] */
    const void *wo;             /* [d][n_heads*hd] */
    const void *wg, *wu;        /* [d_ff][d] gate and up projections */
    const void *wd;             /* [d][d_ff] */
    const float *norm1, *norm2; /* attention and FFN RMSNorm gains */
    const float *bq, *bk, *bv;  /* float32 biases of the q, k, v projections ([n_heads*hd],
                                   [n_kv_heads*hd] x 2; the Qwen2.5 family of Sec. 4.1), added
                                   before the rotary embedding; all three NULL: none */
} cs_layer_weights;

typedef struct cs_weights {
    const void* embed;              /* [vocab][d] */
    const void* lm_head;            /* [vocab][d] */
    const float* final_norm;        /* [d] */
    const cs_layer_weights* layers; /* host array [n_layers] of device pointers */
} cs_weights;

typedef struct cs_model cs_model;
typedef struct cs_kv cs_kv;

/* Value range of the tuned kernels.  For CS_BF16 models whose shape allows them (head_dim 64 or
 * 128, d_model, d_ff and n_heads*head_dim multiples of 128, vocab a multiple of 16) the projections
 * multiply float16 operands on the matrix cores: the library converts its copy of the weights
 * from bfloat16 (exactly for 2^-17 <= |w| <= 65504; smaller magnitudes are rounded to multiples
 * of 2^-24) and the kernels round every projection input to float16.  Supported range:
 *   - weights: finite, |w| <= 65504, otherwise cs_model_create fails with CS_E_UNSUPPORTED;
 *   - activations that feed a projection (RMSNorm outputs, attention outputs, SwiGLU outputs):
 *     |x| <= 65504.  A larger magnitude is saturated to +-65504 instead of becoming infinite, and
 *     the producing kernel raises a bit in a per-model status word on the device:
 *     CS_RANGE_NORM, CS_RANGE_ATTN, CS_RANGE_FFN.  A NaN raises the bit of its producer too.
 * cs_model_range_status waits for the device, returns the word in *flags (host) and clears it
 * if `clear` is non-zero; 0 means every result since the last clear is the exact-range result.
 * The asynchronous calls (cs_verify, cs_step) never fail for this reason: ask afterwards.  The
 * synchronous loops (cs_decode*, which clear the word when they start) deliver their tokens and
 * return CS_E_RANGE if the word is non-zero at the end.  Plain-kernel and CS_F32 models keep
 * float32 activations and never raise a bit. */
enum { CS_RANGE_NORM = 1, CS_RANGE_ATTN = 2, CS_RANGE_FFN = 4, CS_RANGE_WEIGHT = 8 };
int cs_model_range_status(cs_model* m, int32_t* flags /*host*/, int32_t clear);

/* Copies (and re-lays-out) the weights into library-owned device memory; the caller's
 * buffers may be freed afterwards.  Synchronous. */
int cs_model_create(const cs_model_cfg* cfg, const cs_weights* w, cs_model** out);
void cs_model_destroy(cs_model*);

/* Staged creation, for models whose caller-side weights should not sit in device memory next to
 * the library's copy all at once (the 70B-class models of Sec. 4.1 are 141 GB in bfloat16, half of
 * one GPU's memory): cs_model_create_staged allocates the library's storage and workspace,
 * cs_model_load_head and cs_model_load_layer then take the parts in any order, each call copying
 * (and re-laying-out) what it is given and returning when the caller's buffers may be freed.  A
 * layer may be loaded again (new weights).  Until the head and every layer have been loaded,
 * calls that run the model fail with CS_E_STATE.  cs_model_create is the same thing in one call.
 * Pointers are device pointers with the layouts of cs_weights / cs_layer_weights.  Synchronous. */
int cs_model_create_staged(const cs_model_cfg* cfg, cs_model** out);
int cs_model_load_head(cs_model* m, const void* embed, const void* lm_head, const float* final_norm);
int cs_model_load_layer(cs_model* m, int32_t layer, const cs_layer_weights* w);

/* Rotary frequencies of the model's own (checkpoints that rescale them, e.g. the Llama-3.1 models
 * of Sec. 4.1): pair (j, j + head_dim/2) at position p is rotated by p * inv_freq[j] instead of
 * p * rope_theta^(-2j/head_dim).  inv_freq: host array of head_dim/2 finite values, copied; NULL
 * goes back to rope_theta.  Synchronous (waits for the device); applies to the calls that
 * follow, so set it before the first prompt goes into a cache of this model. */
int cs_model_set_rope_inv_freq(cs_model* m, const double* inv_freq /*host [head_dim/2] or NULL*/);

/* KV cache for `batch` independent streams of up to `capacity` positions each, all layers.
 * Lengths start at 0. */
int cs_kv_create(const cs_model* m, int32_t batch, int64_t capacity, cs_kv** out);
void cs_kv_destroy(cs_kv*);
/* Set / read the valid length of one stream (App. B.2 truncation is exactly a smaller
 * length: rows at and beyond it are dead and are overwritten by later steps).
 * Both synchronise with the device. */
int cs_kv_set_len(cs_kv*, int32_t stream_idx, int64_t len);
int64_t cs_kv_len(cs_kv*, int32_t stream_idx);
/* Import / export cache rows [pos0, pos0+n) of one (layer, stream): k_rows and v_rows are
 * device buffers [n_kv_heads][n][head_dim] in cfg.dtype.  Does not change the length.
 * Synchronous.  Used to seed a cache with given contents and to inspect it in tests. */
int cs_kv_load(cs_kv*, int32_t layer, int32_t stream_idx, int64_t pos0, int64_t n,
               const void* k_rows, const void* v_rows);
int cs_kv_read(cs_kv*, int32_t layer, int32_t stream_idx, int64_t pos0, int64_t n,
               void* k_rows, void* v_rows);

/* ------------------------------------------------------------------------------------
 * Verification  (Sec. 3.2 second paragraph; App. B.2; App. B.3 step 2)
 *
 * For every stream b with valid length L_b the block [pending_b, draft_b[0..m_b)] with
 * m_b = draft_len[b] <= k is placed at positions L_b .. L_b+m_b and evaluated in one
 * forward pass against the cache.  a_i = argmax of the logits of block row i (lowest
 * index on ties).  tau_b = number of leading i < m_b with a_i == draft_b[i];
 * next_b = a_tau.  Afterwards L_b = L_b + tau_b + 1: the cache holds pending_b and the
 * accepted drafts (rows of rejected drafts are dead), and next_b is NOT in the cache: it
 * is the next call's pending token.  Every call advances each stream by tau_b + 1 tokens.
 *
 * All pointers are device pointers.  d_draft is [B][k] (row stride k); slots at and
 * beyond draft_len are ignored.  d_logits_out may be NULL; otherwise it receives
 * float32 [B][k+1][vocab] (rows beyond m_b are unspecified).  B must equal the batch of
 * `kv` and be <= cfg.max_batch; k <= cfg.max_k.  Returns CS_E_CAPACITY if some stream may
 * not have room for k+1 more rows.  Asynchronous on `stream`.
 * ---------------------------------------------------------------------------------- */
int cs_verify(cs_model* m, cs_kv* kv, const int32_t* d_pending /*[B]*/,
              const int32_t* d_draft /*[B][k]*/, const int32_t* d_draft_len /*[B]*/,
              int32_t k, int32_t* d_accepted_len /*[B]*/, int32_t* d_next_token /*[B]*/,
              float* d_logits_out, void* stream);

/* ------------------------------------------------------------------------------------
 * One whole copy-and-verify step on device-resident state  (App. B.3 steps 1, 2, 4)
 *
 * d_hist[b*stride .. +d_hist_len[b]) is the token sequence of stream b (prompt plus
 * everything emitted, Sec. 3.2 third paragraph); its last token is the pending token.
 * Contract: d_hist_len[b] >= 1 and the cache length of stream b equals d_hist_len[b] - 1 (the
 * cache holds every token but the pending one).  The library cannot check this without a host
 * round trip; a history longer than that is still searched in full, but the block is placed at
 * the cache length, not at the history length.  The call searches each history (gamma, policy),
 * drafts up to k tokens, clamps the draft to d_room[b] - 1 if d_room != NULL (room =
 * tokens the stream may still emit), verifies, then appends draft[0..tau) and next to the
 * history and advances d_hist_len[b] by tau+1 and d_room[b] by -(tau+1).  A stream with
 * d_room[b] <= 0 takes no part: nothing is drafted, accepted, emitted or appended, its cache
 * length stays, and its outputs are accepted_len 0 and next_token -1.
 * Outputs d_accepted_len[B], d_next_token[B], d_draft_len_out[B] (may be NULL).
 * No host synchronisation: the step can be enqueued back to back.
 * ---------------------------------------------------------------------------------- */
int cs_step(cs_model* m, cs_kv* kv, int32_t* d_hist, int64_t stride, int32_t* d_hist_len,
            int32_t* d_room, int32_t gamma, int32_t k, int32_t policy,
            int32_t* d_accepted_len, int32_t* d_next_token, int32_t* d_draft_len_out,
            void* stream);

typedef struct cs_stats {
    int64_t steps;      /* verify calls */
    int64_t attempts;   /* steps that carried a non-empty draft */
    int64_t drafted;    /* draft tokens sent to verification */
    int64_t accepted;   /* draft tokens accepted */
} cs_stats;

/* ------------------------------------------------------------------------------------
 * Decode loops  (Sec. 3.2; App. B.3 step 4: the procedure repeats until a stopping criterion)
 *
 * cs_decode: stream 0 of `kv` is reset, the prompt (host, >= 1 token) is run through the
 * model in blocks, then cs_step repeats until exactly max_new tokens are emitted or
 * eos_id (>= 0) is emitted (the output is cut after it).  out_tokens: host [max_new].
 * Requires kv batch == 1 and capacity >= prompt_len + max_new + k + 1.
 * cs_decode_greedy is plain greedy decoding through the same kernels (draft length 0);
 * by the paper's construction both emit the same tokens.  Synchronous.
 * Lengths, budgets and step outcomes live on the device; the loops enqueue up to four steps
 * (never more than the remaining budget needs at full acceptance) before the host reads their
 * outcome in one copy, so only a stop token can leave steps of a burst unused.  On return the
 * cache of a stream holds prompt_len + n_out - 1 rows (every token but the last one emitted).
 * ---------------------------------------------------------------------------------- */
int cs_decode(cs_model* m, cs_kv* kv, const int32_t* prompt /*host*/, int64_t prompt_len,
              int64_t max_new, int32_t gamma, int32_t k, int32_t policy, int32_t eos_id,
              int32_t* out_tokens /*host*/, int64_t* n_out, cs_stats* stats /*may be NULL*/);
int cs_decode_greedy(cs_model* m, cs_kv* kv, const int32_t* prompt /*host*/, int64_t prompt_len,
                     int64_t max_new, int32_t eos_id, int32_t* out_tokens /*host*/,
                     int64_t* n_out);

/* ------------------------------------------------------------------------------------
 * The same loop for all streams of a cache at once  (Sec. 3.2; App. B.3 step 4; the streams
 * are independent sequences, each with its own history, match and acceptance)
 *
 * cs_prefill_batch: prompts is a host array [B][prompt_stride], B = the batch of `kv`,
 * stream b's prompt being its first prompt_len[b] >= 1 tokens.  All lengths are reset; the
 * prompts are run through the model in lock step (every pass takes the same number of rows
 * from every stream, the workspace rows divided by B; a stream whose prompt is used up rides
 * along on padding rows that stay dead), leaving stream b with length prompt_len[b] - 1.
 * cs_decode_batch: cs_prefill_batch, then cs_step on all streams until every stream has
 * emitted max_new tokens or eos_id (>= 0; its output is cut after it).  A stream that is done
 * takes no further part (its emission budget is 0, see cs_step).  out_tokens: host
 * [B][max_new]; n_out: host [B]; stats: host [B] or NULL.  Every stream's output is what
 * cs_decode gives for that prompt alone.  Requires capacity >= longest prompt + max_new + k
 * + 1.  Synchronous.
 * ---------------------------------------------------------------------------------- */
int cs_prefill_batch(cs_model* m, cs_kv* kv, const int32_t* prompts /*host [B][prompt_stride]*/,
                     int64_t prompt_stride, const int64_t* prompt_len /*host [B]*/);
int cs_decode_batch(cs_model* m, cs_kv* kv, const int32_t* prompts /*host [B][prompt_stride]*/,
                    int64_t prompt_stride, const int64_t* prompt_len /*host [B]*/, int64_t max_new,
                    int32_t gamma, int32_t k, int32_t policy, int32_t eos_id,
                    int32_t* out_tokens /*host [B][max_new]*/, int64_t* n_out /*host [B]*/,
                    cs_stats* stats /*host [B], may be NULL*/);

/* ------------------------------------------------------------------------------------
 * CopySpec merged with draft-model speculative decoding  (Sec. 3.3; App. B.3 steps 1-4)
 *
 * Every step first looks for a copy opportunity (App. B.3 step 1).  With a match the copied
 * block is verified as in cs_decode (step 2).  Without one, a second, smaller model (its own
 * handle and its own single-stream cache, same vocabulary) proposes up to `delta` tokens
 * greedily, one per forward pass, continuing the accepted sequence (step 3a); the target
 * verifies them in one block with the same acceptance rule (step 3b) and both caches are cut
 * back to the accepted prefix (step 3c).  The draft model runs only when it is needed and
 * first reads the tokens accepted since it last ran.  The emitted tokens are the target's
 * greedy tokens whatever the draft model proposes.  delta = 0 is cs_decode.
 * Requires 0 <= delta <= the target's max_k, target capacity >= prompt_len + max_new +
 * max(k, delta) + 1, draft capacity >= prompt_len + max_new + delta + 1.  prompt and
 * out_tokens are host pointers.  Synchronous.
 * ---------------------------------------------------------------------------------- */
typedef struct cs_merged_stats {
    int64_t steps;            /* target verify calls */
    int64_t copy_attempts;    /* steps whose draft was copied from the history */
    int64_t copy_drafted;
    int64_t copy_accepted;
    int64_t spec_attempts;    /* steps whose draft came from the draft model */
    int64_t spec_drafted;
    int64_t spec_accepted;
    int64_t draft_forwards;   /* forward passes of the draft model (catch-up blocks + proposals) */
} cs_merged_stats;

int cs_decode_merged(cs_model* target, cs_kv* target_kv, cs_model* draft, cs_kv* draft_kv,
                     const int32_t* prompt /*host*/, int64_t prompt_len, int64_t max_new,
                     int32_t gamma, int32_t k, int32_t policy, int32_t delta, int32_t eos_id,
                     int32_t* out_tokens /*host*/, int64_t* n_out,
                     cs_merged_stats* stats /*may be NULL*/);

/* Run prompt[0 .. n-1) of one stream through the model, in blocks of up to
 * max(prompt block rows, max_k + 1) rows (cs_set_prompt_block_rows, 4096 by default), so that its cache holds them and its length is n-1 (the last
 * prompt token stays pending).  Resets the stream's length first.  Single-stream caches
 * only (stream_idx == 0).  prompt: host.  Synchronous. */
int cs_prefill(cs_model* m, cs_kv* kv, int32_t stream_idx, const int32_t* prompt /*host*/,
               int64_t prompt_len);

/* ------------------------------------------------------------------------------------
 * Single operations of the verify pass, exposed for per-kernel parity tests and timing.
 * All pointers are device pointers; asynchronous on `stream`.
 * ---------------------------------------------------------------------------------- */

/* Y[R][N] (float32) = X[R][K] * W[N][K]^T.  dtype CS_BF16: X and W are bfloat16, products
 * accumulate in float32 on the matrix cores (needs a model that runs the bf16 kernels,
 * N % 16 == 0, K % 128 == 0; W is first re-laid-out into the kernel's tiled weight format in
 * a temporary, and the call waits for completion); CS_F32: X and W float32. */
int cs_op_gemm(cs_model* m, int32_t dtype, const void* X, const void* W, float* Y,
               int32_t R, int32_t N, int32_t K, void* stream);

/* Block attention of one layer over the cache (Sec. 3.2: the block is appended to the
 * context and evaluated in one pass).  q: float32 [B][rows][n_heads][head_dim], already
 * rotated; row i of stream b sits at position L_b + i and sees cache rows 0 .. L_b + i,
 * which must already hold its own K/V.  out: float32 [B][rows][n_heads*head_dim].
 * Softmax in float32 with scale 1/sqrt(head_dim).  rows <= max_k + 1. */
int cs_op_attention(cs_model* m, cs_kv* kv, int32_t layer, const float* q, int32_t rows,
                    float* out, void* stream);

/* Greedy argmax per row fused with the accept rule (App. B.2).  logits: float32
 * [B][k+1][V]; draft [B][k]; draft_len [B].  Outputs accepted_len[B], next_token[B] and,
 * if not NULL, row_argmax [B][k+1]. */
int cs_op_argmax_accept(cs_model* m, const float* logits, int32_t B, int32_t k, int32_t V,
                        const int32_t* draft, const int32_t* draft_len, int32_t* accepted_len,
                        int32_t* next_token, int32_t* row_argmax, void* stream);

/* Asynchronous variant of cs_kv_set_len for all streams at once: lengths are copied from
 * the device array d_len[B] on `stream`; len_upper_bound (host) must be >= every one of
 * them and <= capacity.  Lets a benchmark or a serving loop rewind the cache without a
 * host round trip. */
int cs_kv_set_len_dev(cs_kv*, const int32_t* d_len /*device [B]*/, int64_t len_upper_bound,
                      void* stream);

/* ------------------------------------------------------------------------------------
 * Instrumentation: per-kernel-class device timing with HIP events recorded on the stream
 * the kernels run on.  cs_profile_enable(mask) selects classes (0 = off, the default);
 * cs_profile_read synchronises the device and returns the summed duration and the number
 * of launches of one class since the last cs_profile_reset.
 * ---------------------------------------------------------------------------------- */
enum {
    CS_PROF_SCAN = 1,      /* match scan kernel */
    CS_PROF_GEMM = 2,      /* every projection GEMM */
    CS_PROF_ATTN = 4,      /* block attention kernel (without the split merge) */
    CS_PROF_ATTN_MERGE = 8,
    CS_PROF_ARGMAX = 16,   /* vocabulary argmax kernel */
    CS_PROF_LMHEAD = 32    /* the lm_head GEMM alone */
};
void cs_profile_enable(int32_t class_mask);
void cs_profile_reset(void);
int cs_profile_read(int32_t cls, double* total_ms, int64_t* launches);

/* Select kernel variants for the following cs_model_create calls of the calling thread (the
 * setting is thread-local and read at creation only): 0 = tuned kernels where the shape allows
 * (default), 1 = plain reference kernels everywhere. */
void cs_set_plain_kernels(int32_t on);

/* Rows of one prompt block for the following cs_model_create calls of the calling thread
 * (thread-local, read at creation only; the workspace of a model is sized for it): cs_prefill ingests a prompt `rows` tokens at a time, cs_prefill_batch gives each
 * stream its share of them.  0 = the default (4096); other values are clamped to 16..8192.
 * A model whose max_k + 1 is larger uses that.  Results do not depend on it beyond rounding. */
void cs_set_prompt_block_rows(int32_t rows);

#ifdef __cplusplus
}
#endif
#endif /* COPYSPEC_H */

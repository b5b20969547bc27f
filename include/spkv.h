/*
 * spkv.h -- C ABI of the Self-Pruned KV (SP-KV) decode path for AMD MI355X (gfx950).
 *
 * The library keeps, for one attention layer, the two-part KV cache of SP-KV
 * (paper Sec. 2.1 and appendix "Inference Kernels"):
 *
 *   - a local window: the w most recent key/value pairs of every sequence, always
 *     attended (window indicator 1[0 <= t - s < w]; w = 128 by default), held in a
 *     ring buffer with the pair's utility logit beside it;
 *   - a long-term cache per (sequence, KV head): the pairs that have left the window
 *     and whose utility passed the threshold, z_s = 1[u_s >= tau] (Eq. 2), stored
 *     compacted in ascending position in fixed-size pages; pairs with z_s = 0 are
 *     dropped when they leave the window.
 *
 * and computes one decode step of gated attention (Eq. 3-5): the newest token of every
 * sequence attends to its window and to its heads' long-term caches,
 *   o_t = sum_s softmax_s(<q_t, k_s> * sm_scale) v_s   over available s.
 *
 * Conventions
 *   - Every pointer documented "device" is GPU memory owned by the caller (for example a
 *     PyTorch tensor) and must be 16-byte aligned; "host" pointers are ordinary memory.
 *     The library allocates no device memory: the cache lives in an arena the caller
 *     provides and keeps alive until spkv_cache_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls that
 *     enqueue work return without waiting for it; calls documented "synchronises" wait
 *     for `stream`.  One cache must be driven from one stream at a time.
 *   - Tensors are dense, row-major, innermost dimension last.  K, V and Q are bf16
 *     (bit pattern in uint16_t); utility logits are fp32 pre-sigmoid values f with
 *     u = sigmoid(f) (Eq. 1).  Query head j reads KV head j / (n_q_heads / n_kv_heads).
 *   - The gate is evaluated on the logit: z = 1[f >= theta], theta = log(tau / (1 - tau))
 *     computed in fp64 from the fp32 tau and rounded once to fp32.  This is Eq. 2 moved
 *     through the (strictly increasing) sigmoid.  tau <= 0 keeps every pair, tau >= 1
 *     keeps none.  NaN logits are dropped.
 *   - All functions return SPKV_OK (0) or a negative SPKV_E_* code; nothing is thrown and
 *     a failed call leaves the cache unchanged unless stated otherwise.
 */
#ifndef SPKV_H
#define SPKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPKV_OK            0
#define SPKV_E_INVAL      -1   /* null pointer, bad shape, misaligned pointer, bad option   */
#define SPKV_E_STATE      -2   /* decode on a sequence that holds no token yet              */
#define SPKV_E_CAPACITY   -3   /* page pool, page table or max_context would overflow       */
#define SPKV_E_HIP        -4   /* a HIP runtime call or kernel launch failed                */
#define SPKV_E_NOMEM      -5   /* host allocation failed                                    */
#define SPKV_E_DEVICE     -6   /* a kernel flagged an internal inconsistency (see stats)    */

#define SPKV_MAX_BATCH     512 /* sequences per cache                                       */
#define SPKV_PAGE_TOKENS   64  /* key/value pairs per long-term page                        */
#define SPKV_MAX_CHUNK_TOKENS 16 /* new tokens per sequence in one spkv_decode_chunk call   */

typedef struct spkv_cache spkv_cache_t;   /* opaque host object */

typedef struct spkv_config {
    int32_t batch;          /* sequences, 1 .. SPKV_MAX_BATCH                               */
    int32_t n_q_heads;      /* query heads; a multiple of n_kv_heads, group size <= 16      */
    int32_t n_kv_heads;     /* KV heads (one gate per KV head, listing appendix)            */
    int32_t head_dim;       /* 64 or 128                                                    */
    int32_t window;         /* w >= 1 (Sec. 2.1; 128 in the paper's main setting)           */
    int32_t page_tokens;    /* 0 or SPKV_PAGE_TOKENS                                        */
    float   tau;            /* gate threshold on the sigmoid (Eq. 2); 0.5 in the paper      */
    int32_t max_context;    /* largest number of tokens any one sequence will hold          */
    int64_t max_total_kept_tokens; /* long-term capacity summed over all (sequence, head)   */
} spkv_config_t;

typedef struct spkv_stats {
    int64_t total_tokens;      /* sum over sequences of tokens appended                     */
    int64_t evicted_tokens;    /* sum over (seq, head) of tokens that have left the window  */
    int64_t window_tokens;     /* sum over (seq, head) of min(T, w)                         */
    int64_t kept_tokens;       /* sum over (seq, head) of long-term entries                 */
    int64_t gate_on_tokens;    /* sum over (seq, head, position) of z (Eq. 8 numerator)     */
    double  density_evicted;   /* kept / evicted: the density the text reports (Eq. 8 note) */
    double  density_all;       /* gate_on / (n_kv_heads * total_tokens): Eq. 8 literally    */
    int64_t kept_kv_bytes;     /* (kept + window) * 2 * head_dim * 2: bytes a step must read*/
    int64_t dense_kv_bytes;    /* total_tokens * n_kv_heads * 2 * head_dim * 2              */
    int64_t pool_pages_used;
    int64_t pool_pages_total;
    int64_t arena_bytes;
    int32_t device_error;      /* nonzero if a kernel ever flagged an inconsistency         */
    int32_t n_work_items;      /* split-K work items the next decode call would launch      */
    int32_t n_work_items_last_call; /* the same lists cut by the partition the most recent
                                  decode call used (it is chosen from the host's upper bound
                                  of the lengths; far fewer items than n_work_items would mean
                                  that bound has drifted)                                   */
    int32_t reserved_;
} spkv_stats_t;

/* Options for spkv_cache_set_option. */
#define SPKV_OPT_ITEM_TARGET    1  /* split-K work items to aim for per decode, 1..32768;
                                      0 (default) = as many as the chip runs at once.  Items
                                      come in workgroups of up to four (SPKV_OPT_MERGE_WAVES),
                                      so a call may use up to four per (sequence, KV head)
                                      even for a target of 1                                 */
#define SPKV_OPT_KERNEL_TIMING  2  /* 1: bracket every split-K kernel launch with HIP events */
#define SPKV_OPT_SPLIT_ONLY     3  /* 1: spkv_decode_attention launches the split-K kernel
                                      only (no combine, `out` and `lse` left untouched):
                                      lets a harness time that kernel back to back        */
#define SPKV_OPT_SINK_TOKENS    4  /* n >= 0: the first n positions of every sequence are always
                                      kept when they leave the window, whatever their logit
                                      (attention sinks, an ablation variant in the paper; the
                                      default 0 is the paper's method).  Only while the cache is
                                      empty (after create or reset): SPKV_E_STATE otherwise. */
#define SPKV_OPT_MERGE_WAVES    5  /* work items per workgroup of the single-token decode kernels
                                      (they merge their results before anything is stored):
                                      1, 2 or 4; 0 (default) = chosen per call from the number
                                      of (sequence, KV head) pairs and their lengths           */

#define SPKV_OPT_STEP_LAUNCHES  6  /* kernel launches of spkv_decode_step and spkv_decode_attention:
                                      1: one -- the last workgroup of every (sequence, KV head) to
                                      finish merges the pair's partial results and, in the step,
                                      performs the pair's append; 2: a second launch merges (and
                                      appends); 0 (default) = the library's choice, at present two
                                      (measured faster at every cache size tried: the tickets and
                                      the merge inside the launch cost more than a launch).  Same
                                      results up to the order of fp32 sums                         */

/* Bytes of device arena a cache with this configuration needs (0 if cfg is invalid).
 * Host-only; touches no device.  Capacity rule (appendix "Inference Kernels": pages are
 * given out from a pool with headroom): the long-term cache can hold
 * max_total_kept_tokens pairs in total plus one partly filled page per (seq, head). */
size_t spkv_cache_required_bytes(const spkv_config_t* cfg);

/* Create a cache inside `dev_arena` (device, 256-byte aligned, >= required bytes) and
 * enqueue on `stream` the fill that zeroes it.  The arena stays owned by the caller and
 * must outlive the cache.  *out receives the handle.  (Sec. 2.1; appendix "Inference
 * Kernels": window ring + per-head long-term pages.) */
int spkv_cache_create(const spkv_config_t* cfg, void* dev_arena, size_t arena_bytes,
                      void* stream, spkv_cache_t** out);

/* Free the host object.  Synchronises nothing; the caller frees the arena afterwards. */
int spkv_cache_destroy(spkv_cache_t* cache);

/* Capacity growth ("Inference Kernels" appendix: the cache is given headroom and grows when
 * it runs out).  The library never allocates, so growth is a move: the caller provides a new,
 * larger arena for a configuration with the same shape (batch, heads, head_dim, window) and
 * max_context / max_total_kept_tokens not smaller than before; the call copies the whole
 * cache state into it on `stream` (page ids stay valid: pages are indices into the pool) and
 * the cache continues there.  The old arena must stay untouched until the work enqueued on
 * `stream` up to and including this call has completed; after that it is the caller's again.
 * new_cfg->tau is ignored (the live threshold stays).  Typical use: spkv_append returned
 * SPKV_E_CAPACITY -> grow -> repeat the append.
 * SPKV_E_INVAL: shape differs, a limit shrinks, arena too small, misaligned or overlapping
 * the current one (the cache is unchanged). */
int spkv_cache_grow(spkv_cache_t* cache, const spkv_config_t* new_cfg, void* new_dev_arena,
                    size_t new_arena_bytes, void* stream);

/* Forget every token (all sequences back to length 0); enqueues the zero fill. */
int spkv_cache_reset(spkv_cache_t* cache, void* stream);

/* Write path (Eq. 1-2; appendix "Inference Kernels").  Appends, for each sequence b,
 * the tokens in rows cu_seqlens[b] .. cu_seqlens[b+1]-1 (in position order):
 *   k, v         device bf16  [total_tokens, n_kv_heads, head_dim]
 *   util_logits  device fp32  [total_tokens, n_kv_heads]   (pre-sigmoid f)
 *   cu_seqlens   host   int32 [batch + 1], cu_seqlens[0] = 0, non-decreasing
 * Each new pair is written into its sequence's window ring together with its logit; a
 * pair pushed out of the window (position s when position s + w arrives) is appended to
 * its head's long-term cache if f_s >= theta and dropped otherwise.  A decode step is the
 * case cu_seqlens = 0, 1, .., batch (one token per sequence; sequences may also get 0).
 * Larger calls take a bulk path (ballot/prefix-sum stream compaction, stable order).
 * Errors: SPKV_E_CAPACITY if any sequence would exceed max_context, or if the pool could
 * overflow even when every pushed-out pair were kept, judged after refreshing the host's
 * bound from the device counters (synchronises only in that case); then nothing is
 * written.  Feed long prompts in chunks so that this worst case fits. */
int spkv_append(spkv_cache_t* cache, const void* k, const void* v, const float* util_logits,
                const int32_t* cu_seqlens, void* stream);

/* Read path (Eq. 3-5).  For every sequence, the newest appended token attends to its
 * window and to its heads' long-term caches:
 *   q    device bf16 [batch, n_q_heads, head_dim]   (query of the newest token)
 *   out  device bf16 [batch, n_q_heads, head_dim]
 *   lse  device fp32 [batch, n_q_heads] or NULL: log sum_s exp(sm_scale * <q, k_s>)
 *   sm_scale <= 0 selects 1 / sqrt(head_dim)
 * Call after spkv_append of the same step, so that the query's own key is in the window.
 * The first call after a multi-token append synchronises `stream` once to read the kept
 * lengths back (they size the split-K grid); decode steps in steady state never wait.
 * Errors: SPKV_E_STATE if some sequence holds no token. */
int spkv_decode_attention(spkv_cache_t* cache, const void* q, void* out, float* lse,
                          float sm_scale, void* stream);

/* spkv_decode_attention for callers that cannot allocate -- code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc -- and do not want the split-K
 * partial results in their arena either: the same kernels, with the partials in a 16 MiB
 * array that is part of the library's device image (one copy per GPU, held until the process
 * ends) instead of the cache's arena.  The call allocates nothing, on the host's device side
 * or through any library, and never waits for the device.  Inputs, outputs and result as
 * for spkv_decode_attention (the work partition is fitted to the slots the array holds, so
 * results can differ from spkv_decode_attention's in the last bits, as between any two
 * partitions).
 * The array keeps the last call's contents; every slot a call reads it has written before,
 * so nothing needs clearing.  All caches on a GPU share it: calls that overlap on one GPU
 * (different streams) race -- issue them on one stream, or order them with events.
 * Errors: SPKV_E_CAPACITY if the array cannot hold two partial slots per (sequence, KV head)
 * -- batch * n_kv_heads above 16 MiB / (8 * group size * (head_dim + 2)) -- checked first;
 * SPKV_E_STATE if some sequence holds no token, or if a multi-token append has been issued
 * since the lengths were last read back (spkv_decode_attention, spkv_cache_safe_steps and
 * spkv_cache_stats read them; this call will not wait for them); SPKV_E_HIP if the array's
 * address cannot be obtained. */
int spkv_decode_attention_static(spkv_cache_t* cache, const void* q, void* out, float* lse,
                                 float sm_scale, void* stream);

/* One whole decode step in one kernel launch (or two, SPKV_OPT_STEP_LAUNCHES) instead of
 * three: the same result and the same cache state as
 *     spkv_append(cache, k, v, util_logits, {0, 1, .., batch}, stream);
 *     spkv_decode_attention(cache, q, out, lse, sm_scale, stream);
 * (appendix "Inference Kernels" for the write, Eq. 3-5 for the read), for the case of exactly
 * one new token per sequence:
 *   k, v         device bf16 [batch, n_kv_heads, head_dim]   (the new token's pair)
 *   util_logits  device fp32 [batch, n_kv_heads]
 *   q, out, lse, sm_scale as for spkv_decode_attention
 * The split-K kernel attends to the cache as it stands, leaving out the pair the new token
 * pushes out of the window unless it passes the gate; the merge of the partial results adds
 * the new pair's own term, read from k / v, and the append follows it -- both by the last
 * workgroup of every (sequence, KV head) to finish (appendix "Inference Kernels": one fused
 * kernel per step), or by a second launch.  Sequences may be empty before the call.  Errors
 * as for spkv_append (SPKV_E_CAPACITY before any launch). */
int spkv_decode_step(spkv_cache_t* cache, const void* k, const void* v, const float* util_logits,
                     const void* q, void* out, float* lse, float sm_scale, void* stream);

/* Multi-token step: every sequence b receives n_b = cu_seqlens[b+1] - cu_seqlens[b] new
 * tokens (0 <= n_b <= SPKV_MAX_CHUNK_TOKENS, n_b <= window, n_b * group size <= 64) and gets
 * the attention output of each of them, computed as if the tokens had been appended and
 * decoded one at a time: token i of the chunk (position T_b + i) attends to the positions
 * s <= T_b + i that are inside its window or pass the gate (Eq. 3-5; the rows T_b .. of the
 * masked attention of the listing appendix).  Use: prompt feed in 16-token chunks (the chunk
 * size of the paper's chunked-prefill protocol); for draft tokens that may be rejected see
 * spkv_score_chunk.
 *   k, v         device bf16 [total, n_kv_heads, head_dim]    util_logits device fp32 [total, n_kv_heads]
 *   q, out       device bf16 [total, n_q_heads, head_dim]     lse device fp32 [total, n_q_heads] or NULL
 *   cu_seqlens   host int32 [batch + 1]
 * Afterwards the cache holds the chunk exactly as after spkv_append of the same tokens.
 * One pass over the cache serves all tokens of a chunk (each K/V tile is read once per
 * (sequence, KV head)).  Needs no workspace.  Two kernels stand behind the multi-token calls
 * and each shape has one owner: chunks that fit one group of 16 query columns
 * (n_b * group size <= 16 for every b) run on the split-K kernel of the decode step with the
 * columns (token, head); wider chunks run on the kernels of spkv_prefill_attention, here with
 * the staging rows in the cache's own arena.  spkv_prefill_attention routes the same way, so
 * the two calls cost the same on the shapes both accept.
 * Errors as for spkv_append; SPKV_E_INVAL if a chunk is too long. */
int spkv_decode_chunk(spkv_cache_t* cache, const void* k, const void* v, const float* util_logits,
                      const void* q, const int32_t* cu_seqlens, void* out, float* lse,
                      float sm_scale, void* stream);

/* Scoring of draft tokens (speculative decoding): the attention outputs of
 * spkv_decode_chunk for the same chunks, with the cache left exactly as it was -- nothing is
 * appended, no length changes.  Draft token i of a sequence attends as if drafts 0 .. i - 1
 * had been appended before it (Eq. 3-5; all of them lie inside its window, so their utility
 * logits play no part and are not passed).  The caller then appends the accepted prefix of
 * every sequence with spkv_append (rejected drafts never touch the cache; a token that
 * entered the window could not be taken back, because it overwrites the slot of the pair it
 * pushes out).
 *   k, v, q, cu_seqlens, out, lse, sm_scale   as for spkv_decode_chunk, same limits
 * Errors: SPKV_E_INVAL as for spkv_decode_chunk; never SPKV_E_CAPACITY. */
int spkv_score_chunk(spkv_cache_t* cache, const void* k, const void* v, const void* q,
                     const int32_t* cu_seqlens, void* out, float* lse, float sm_scale,
                     void* stream);

/* Prefill attention: the multi-token step without a length limit.  Every sequence b
 * receives n_b >= 0 new tokens and gets the attention output of each, token i (position
 * T_b + i) attending to the positions s <= T_b + i inside its window or passing the gate
 * (Eq. 3-5; causal inside the chunk), and the cache afterwards holds the chunk exactly as
 * after spkv_append.  With this call a prompt both fills the cache and gets its own
 * attention, in chunks of any size (the chunked-prefill protocol of the evaluation section;
 * gated-off keys outside the window are never read, the block skipping of Sec. 2.2 at the
 * granularity of single keys).
 *   k, v, util_logits, q, cu_seqlens, out, lse, sm_scale   as for spkv_decode_chunk
 *   workspace     device memory, 256-byte aligned; spkv_prefill_workspace_bytes(cache, n, t)
 *                 bytes are enough for every call with at most n tokens per sequence and
 *                 t tokens in all (a call with shorter chunks may need less, never more);
 *                 contents need not survive between calls; caller-owned
 * Work is cut per (sequence, KV head) into spans of consecutive tokens, one workgroup each:
 * 256 / group-size tokens on eight waves, fewer tokens on four or two waves when no sequence
 * brings more.  When the spans alone would not fill the chip, every span's keys are cut into
 * ranges as well (one workgroup each, merged by a second launch).
 * Calls that bring exactly one token for every sequence are handed to spkv_decode_step,
 * calls whose chunks all fit one group of 16 query columns (16 / group-size tokens) to
 * spkv_decode_chunk; the workspace is then not touched.
 * Errors as for spkv_append; SPKV_E_INVAL if the workspace cannot hold what the call
 * writes (checked before anything is written). */
size_t spkv_prefill_workspace_bytes(const spkv_cache_t* cache, int32_t max_tokens_per_sequence,
                                    int64_t max_total_tokens);
int spkv_prefill_attention(spkv_cache_t* cache, const void* k, const void* v,
                           const float* util_logits, const void* q, const int32_t* cu_seqlens,
                           void* out, float* lse, float sm_scale, void* workspace,
                           size_t workspace_bytes, void* stream);

/* Soft-gated attention forward (training phase 1, Eq. 6 and the soft branch of the
 * reference listing): causal attention over whole sequences in which a key inside the window
 * of its query (0 <= t - s < window) attends unchanged and every older key gets the additive
 * bias log u_s = log sigmoid(f_s) on its pre-softmax score -- the differentiable stand-in for
 * the hard gate, and the limit it is annealed from.  Stateless: no cache is involved.
 * log u is taken exactly, from the logit, as -softplus(-f) in fp32 (the listing's
 * log(u + 1e-8) guards a gradient, not the forward value).
 *   q, out       device bf16 [total, n_q_heads, head_dim]     lse device fp32 [total, n_q_heads] or NULL
 *   k, v         device bf16 [total, n_kv_heads, head_dim]    util_logits device fp32 [total, n_kv_heads]
 *   cu_seqlens   host int32 [batch + 1]: sequence b owns rows cu[b] .. cu[b+1]-1, positions 0..
 *   workspace    device memory, 256-byte aligned, spkv_soft_gated_workspace_bytes(...) bytes
 *                for the longest sequence of the call; caller-owned, contents disposable
 * Same kernels as spkv_prefill_attention (keys staged in the page layout, MFMA tile loop);
 * cost is that of dense causal attention.  Returns SPKV_E_INVAL for bad shapes, pointers or
 * a workspace that is too small. */
size_t spkv_soft_gated_workspace_bytes(int32_t batch, int32_t n_kv_heads, int32_t head_dim,
                                       int32_t window, int32_t max_tokens_per_sequence);
int spkv_soft_gated_attention(const void* q, const void* k, const void* v, const float* util_logits,
                              const int32_t* cu_seqlens, int32_t batch, int32_t n_q_heads,
                              int32_t n_kv_heads, int32_t head_dim, int32_t window, void* out,
                              float* lse, float sm_scale, void* workspace, size_t workspace_bytes,
                              void* stream);

/* Forget sequence b (for example when its request has finished): its window and long-term
 * entries are dropped, its pages return to the pool for reuse by any sequence, and slot b
 * holds an empty sequence that can be appended to again.  (The paper's cache manager grows
 * and shares one page pool across requests, appendix "Inference Kernels"; giving pages
 * back is the counterpart a serving loop needs.)  Synchronises `stream` once to read the
 * exact lengths, then enqueues the release.  A recycled page keeps its old bytes beyond the
 * new owner's length; they are masked in attention, which is exact as long as the old
 * values were finite. */
int spkv_cache_release_sequence(spkv_cache_t* cache, int32_t b, void* stream);

/* Utility predictor (Eq. 1; the listing's UtilityPredictor: Linear(d_model, d_hidden), SiLU,
 * Linear(d_hidden, n_kv_heads)), pre-sigmoid, for n_tokens tokens:
 *   logits[t, h] = b2[h] + sum_j w2[h, j] * silu(b1[j] + sum_k w1[j, k] * hidden[t, k])
 *   hidden  device bf16 [n_tokens, d_model]          w1  device bf16 [d_hidden, d_model]
 *   b1      device fp32 [d_hidden] or NULL           w2  device bf16 [n_kv_heads, d_hidden]
 *   b2      device fp32 [n_kv_heads] or NULL         logits  device fp32 [n_tokens, n_kv_heads]
 *   workspace  device fp32 [n_tokens * d_hidden] (hidden activations; caller-owned scratch)
 * (weights in the row-major [out, in] layout of a linear layer).  d_model must be a multiple
 * of 128, d_hidden of 16.  Products of bf16 values accumulate in fp32.  Stateless: no cache
 * involved; the output is what spkv_append / spkv_decode_step take as util_logits. */
int spkv_utility_logits(const void* hidden, const void* w1, const float* b1, const void* w2,
                        const float* b2, float* logits, float* workspace, int32_t n_tokens,
                        int32_t d_model, int32_t d_hidden, int32_t n_kv_heads, void* stream);

/* Fused step with the utility predictor: spkv_decode_step whose util_logits are not passed
 * in but computed here from the new tokens' hidden states (Eq. 1, the predictor of
 * spkv_utility_logits), at no launch of their own: the hidden layer runs in workgroups of
 * the split-K launch, the output layer in the append workgroups of the merge launch.  The
 * new token's logit decides nothing before the token leaves the window (Eq. 3-4), so the
 * attention of the step does not wait for it.
 *   hidden       device bf16 [batch, d_model], row b: hidden state of sequence b's new token
 *   w1 b1 w2 b2  as for spkv_utility_logits; d_model a multiple of 128, d_hidden of 16
 *   k, v, q, out, lse, sm_scale   as for spkv_decode_step
 *   util_logits  device fp32 [batch, n_kv_heads], OUTPUT: the logits the tokens were stored
 *                with (fp32 sums in this call's own order: equal to spkv_utility_logits'
 *                up to fp32 rounding, and the ones that decide the gate)
 *   workspace    device memory, 16-byte aligned, at least
 *                spkv_decode_step_predict_workspace_bytes(batch, d_hidden) bytes; caller-owned
 * Errors as for spkv_decode_step; SPKV_E_INVAL for a bad shape or a workspace too small. */
size_t spkv_decode_step_predict_workspace_bytes(int32_t batch, int32_t d_hidden);
int spkv_decode_step_predict(spkv_cache_t* cache, const void* hidden, const void* w1,
                             const float* b1, const void* w2, const float* b2, int32_t d_model,
                             int32_t d_hidden, const void* k, const void* v, const void* q,
                             void* out, float* lse, float* util_logits, void* workspace,
                             size_t workspace_bytes, float sm_scale, void* stream);

/* Replaying captured steps.  spkv_append (one token per sequence), spkv_decode_attention and
 * spkv_decode_step enqueue kernels only -- no allocation, no copy, no synchronisation as long
 * as the capacity bound holds -- so a serving loop may capture them into a HIP graph (one
 * graph node sequence per layer) and replay the graph step after step with new contents in the
 * same input buffers.  A replay bypasses the host's bookkeeping, hence two calls:
 *   spkv_cache_safe_steps  the "safe-step budget" of the appendix: how many further steps of
 *                          one token per sequence are guaranteed to fit (max_context, and the
 *                          pool even if every pair leaving a window is kept).  Reads the exact
 *                          lengths back first: synchronises `stream`.  Call it outside capture.
 *   spkv_cache_advance     tells the cache that n such steps were executed by replays.
 *                          SPKV_E_CAPACITY (nothing changed) if n exceeds what was safe.
 * The work partition frozen in a captured launch stays valid as the lists grow (work items
 * get longer, never out of bounds); re-capture now and then to rebalance it.  The threshold
 * and the sink count are frozen with the launch too. */
int spkv_cache_safe_steps(spkv_cache_t* cache, void* stream, int64_t* n_steps);
int spkv_cache_advance(spkv_cache_t* cache, int64_t n_steps);

/* Gate density and sizes (Eq. 8).  Synchronises `stream`.  kept_len (host int32
 * [batch * n_kv_heads], or NULL) receives the long-term length of every (seq, head). */
int spkv_cache_stats(spkv_cache_t* cache, spkv_stats_t* stats, int32_t* kept_len, void* stream);

/* The long-term region of one head (appendix "Inference Kernels": the pairs that left the
 * window with their gate on, Eq. 2-4), as positions:
 * Positions held by the long-term cache of (sequence b, KV head h), ascending, into
 * pos (host int32 [cap]); *n receives the count (the call fails with SPKV_E_INVAL if
 * cap is too small, after setting *n).  Synchronises `stream`. */
int spkv_cache_kept_positions(spkv_cache_t* cache, int32_t b, int32_t h, int32_t* pos,
                              int32_t cap, int32_t* n, void* stream);

/* The fp32 threshold theta the gate compares logits against. */
int spkv_cache_threshold_logit(const spkv_cache_t* cache, float* theta);

/* Change tau on a live cache ("tau can be adjusted a posteriori", Sec. 3 and the threshold
 * discussion of the appendix).  The window ring stores every pair's logit, so the new
 * threshold applies to every pair that leaves the window in calls issued after this one,
 * including pairs appended under the old value; decisions already taken stand (dropped
 * pairs are gone, kept pairs stay until spkv_cache_prune).  Host-side only: nothing is launched, calls already
 * enqueued keep the threshold they were issued with.  SPKV_E_INVAL for a NaN tau. */
int spkv_cache_set_tau(spkv_cache_t* cache, float tau);

/* Re-thresholds what is already kept: every long-term entry whose stored utility logit
 * fails the threshold now in force (spkv_cache_set_tau) is dropped, the lists are closed up
 * in place, in order, and the pages they no longer reach are recycled.  Entries dropped
 * earlier are gone for good, so lowering tau brings nothing back; sink positions stay.  The
 * decode attention afterwards reads only what remains (Sec. 3: tau is chosen after training,
 * per deployment; here also on a live cache).  Synchronises `stream` (the host re-reads the
 * lengths).  Cost: one pass over the kept pairs of every (sequence, head). */
int spkv_cache_prune(spkv_cache_t* cache, void* stream);

/* Tuning and instrumentation; see SPKV_OPT_*. */
int spkv_cache_set_option(spkv_cache_t* cache, int32_t option, int64_t value);

/* With SPKV_OPT_KERNEL_TIMING on: durations (milliseconds, HIP events recorded on the
 * launch stream immediately before and after the split-K decode kernel) of the launches
 * since the last call, oldest first, at most cap; *n receives the count.  Synchronises
 * those events. */
int spkv_cache_read_kernel_timing(spkv_cache_t* cache, float* ms, int32_t cap, int32_t* n);

/* Element offset (in bf16 elements from the start of a 64-pair page) at which the cache
 * stores head-dim element d of the pair with in-page index kidx; is_v selects the value
 * (1) or the key (0).  Returns -1 for arguments out of range.  Host-only; lets tests check
 * that the page layout is a bijection and matches the MFMA operand order. */
int64_t spkv_debug_layout_offset(int32_t head_dim, int32_t is_v, int32_t kidx, int32_t d);

/* Plain device-to-device copy of `bytes` (a multiple of 16; src, dst device, 16-byte
 * aligned, not overlapping) by a simple grid-stride kernel: a kernel of exactly known HBM
 * traffic (bytes read + bytes written) against which profiler byte counters are scaled. */
int spkv_debug_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Plain streaming read of exactly known traffic with the launch shape and access pattern of
 * the split-K decode kernel (one-wave workgroups, 16 KB chunks read as sixteen non-temporal
 * 1 KB wave-wide loads, 1 KB stored per workgroup at the end) and no arithmetic: the read
 * ceiling of this memory system for such a launch, against which the decode kernel's
 * bandwidth is put (the measurement protocol asks for the fraction of a measured streaming
 * read ceiling beside the fraction of the vendor peak).
 *   src           device, 16-byte aligned, region_bytes bytes, seen as runs of run_bytes
 *                 (a multiple of 16384; 32768 = one cache page: pages of a list are scattered
 *                 over the pool, bytes inside a page are contiguous)
 *   first_run, n_runs, stride   the launch reads the runs ((first_run + i) * stride) mod
 *                 (region_bytes / run_bytes), i = 0 .. n_runs - 1; a stride coprime to the
 *                 run count makes successive launches read distinct scattered runs
 *   n_workgroups  one-wave workgroups; each reads an equal share of the launch's chunks
 *   sink          device, n_workgroups * 1024 bytes, written
 * SPKV_E_INVAL for arguments out of range (nothing is launched). */
int spkv_debug_read(const void* src, size_t region_bytes, int32_t run_bytes, int64_t first_run,
                    int64_t n_runs, int64_t stride, int32_t n_workgroups, void* sink, void* stream);

/* Static text for an error code. */
const char* spkv_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SPKV_H */

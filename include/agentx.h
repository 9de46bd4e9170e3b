/*
 * agentx.h - C ABI of the MI355X extend / verify library.
 *
 * The library runs the target model's "extend" forward: T new tokens on top of a KV cache that
 * already holds P earlier tokens.  That one call serves both halves of the paper's pipeline:
 *   - prefill after prefix-cache reuse, where T is the uncached prompt suffix
 *     (paper Sec. 2.3 "Prefix caching"; Sec. 4.2), and
 *   - the verification phase of speculative decoding, where T = 1 + k: the most recent token
 *     followed by k drafts from the n-gram lookup table (Sec. 2.3 "Speculative decoding",
 *     Fig. 4; Sec. 4.3), after which rejected drafts are cut from the cache.
 *
 * Conventions
 *   - Handles are opaque.  Every call returns ax_status; nothing throws or aborts.
 *   - "device" pointers are HIP device allocations made by the caller (e.g. through PyTorch)
 *     and BORROWED: weights, the KV pool memory, the workspace and every `out` buffer of
 *     ax_extend*.  The library allocates no device memory.  It owns a few KB of pinned host
 *     staging memory per model.
 *   - "host" pointers (tokens, drafts, T_each, accepted, next_token) are ordinary host memory,
 *     read or written before the call returns.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  ax_extend*
 *     only enqueues work; ax_verify waits for its own result.
 *   - Calls on one model / pool must come from one host thread at a time.
 *   - A call that fails with AX_ERR_INVALID, AX_ERR_OOM or AX_ERR_UNSUPPORTED has launched
 *     nothing and has left every KV sequence exactly as it was.
 *
 * Decoder: pre-norm blocks with grouped-query attention (query head h reads KV head
 * h / (n_q_heads / n_kv_heads)), rotary positions pairing (j, j + head_dim/2), SwiGLU MLP,
 * RMSNorm, no biases, untied LM head.  Every matrix is row-major [out_features, in_features]
 * and is applied as y = x * W^T.
 */
#ifndef AGENTX_H
#define AGENTX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    AX_OK = 0,
    AX_ERR_INVALID = -1,     /* bad handle, NULL pointer, T <= 0, token id outside the vocabulary ... */
    AX_ERR_OOM = -2,         /* not enough free KV blocks, or workspace / pool memory too small      */
    AX_ERR_DEVICE = -3,      /* a HIP call failed                                                    */
    AX_ERR_UNSUPPORTED = -4, /* shape the kernels do not cover (see ax_model_create)                 */
    AX_ERR_STATE = -5        /* e.g. destroying a pool that still has live sequences                 */
} ax_status;

/* Storage type of the weights.  AX_F32: fp32 weights, fp32 KV cache, fp32 arithmetic.
 * AX_BF16: bf16 weights, fp16 KV cache (16 bits per entry, as the paper's cache sizes imply),
 * fp16 matrix-core products with fp32 accumulation; residual stream, norms and softmax in fp32. */
enum { AX_F32 = 0, AX_BF16 = 1 };

enum {                                       /* what ax_extend writes to `out` (device memory)        */
    AX_OUT_NONE = 0,                         /* nothing (building a prefix)                           */
    AX_OUT_LAST_LOGITS = 1,                  /* float[n_seq][vocab]: last row of each sequence        */
    AX_OUT_ALL_LOGITS = 2,                   /* float[sum T][vocab]                                   */
    AX_OUT_LAST_ARGMAX = 3,                  /* int32[n_seq]: greedy token, lowest id on ties         */
    AX_OUT_ALL_ARGMAX = 4                    /* int32[sum T]                                          */
};

typedef struct ax_model ax_model;
typedef struct ax_pool ax_pool;
typedef struct ax_kv ax_kv;

typedef struct {
    int n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ff, vocab;
    float rms_eps, rope_base;
    int dtype;        /* AX_F32 or AX_BF16 (type of every weight tensor)                           */
    int max_pos;      /* longest sequence (P + T) any KV of this model may reach                    */
    int max_tokens;   /* most rows (sum of T over the sequences) one ax_extend* call may carry      */
    int max_seqs;     /* most sequences one ax_extend_batch call may carry (>= 1)                   */
    int act_split;    /* AX_BF16 models: activations between kernels as hi + lo fp16 pairs (see below).
                         0 = automatic (on when n_layers * d_model >= 131072), 1 = on, -1 = off     */
} ax_model_config;

/* Precision of AX_BF16 models.  Between kernels an activation is one fp16 value (11 significant
 * bits); the residual stream, norms, softmax and all accumulators are fp32.  The rounding of the
 * activations is what separates the logits from the exact ones, and it grows with the square root
 * of the depth and with the width: measured on N(0, 0.02) weights, max-abs over all logits of 128
 * rows, 5e-3 for the ~1B shape (16 layers), 1.3e-2 for the ~3B shape (28 layers), 2.7e-2 for the
 * ~8B shape (32 layers).  With act_split every such activation is kept as two fp16 values whose
 * sum carries ~22 bits and every kernel multiplies both against the same weights: no extra weight
 * traffic (few-row calls cost the same), twice the matrix-core work in many-row calls; the ~8B
 * shape then stays near 1.2e-2.  The KV cache holds one fp16 per entry either way.
 * Range: fp16(x * gain) must stay finite, i.e. |residual stream * norm gain| < 65504 (tested up
 * to 6e3); beyond that the result is not finite. */

/* Device pointers, row-major [out, in] (y = x W^T).  Element type = config.dtype.
 * Per-layer members are HOST arrays of n_layers device pointers (copied at create time).
 * AX_F32: all tensors are borrowed for the life of the model.  AX_BF16: ax_model_create copies
 * the seven kinds of matrices (wqkv, wo, w_gate, w_up, w_down, lm_head) into the workspace in
 * the kernels' own layout and never reads the caller's copies again - they may be released
 * after the call; tok_emb and the three kinds of gain vectors stay borrowed. */
typedef struct {
    const void *tok_emb;            /* [vocab, d_model]                                             */
    const void *lm_head;            /* [vocab, d_model]                                             */
    const void *final_norm;         /* [d_model]                                                    */
    const void *const *wqkv;        /* [(n_q + 2 n_kv) * head_dim, d_model]: q heads, k heads, v heads */
    const void *const *wo;          /* [d_model, n_q * head_dim]                                    */
    const void *const *w_gate;      /* [d_ff, d_model]                                              */
    const void *const *w_up;        /* [d_ff, d_model]                                              */
    const void *const *w_down;      /* [d_model, d_ff]                                              */
    const void *const *norm_attn;   /* [d_model] gain of the norm before attention                  */
    const void *const *norm_mlp;    /* [d_model] gain of the norm before the MLP                    */
} ax_weights;

/* Bytes of device workspace ax_model_create needs for this config; 0 if the config is invalid. */
size_t ax_workspace_bytes(const ax_model_config *cfg);

/* Build a model over borrowed weights.  `workspace` is device memory of at least
 * ax_workspace_bytes(cfg) bytes, 256-byte aligned, owned by the caller and used by every call
 * on this model (activations, rotary table, per-call descriptors, split-attention partials
 * and, for AX_BF16, the repacked weight matrices: about as many bytes again as the weights).
 * AX_BF16 needs d_model, d_ff, head counts*head_dim and vocab to be multiples of 64,
 * head_dim in {64, 128} and every matrix entry finite in fp16 (|w| <= 65504: the matrices are
 * multiplied as fp16; a bf16 value below that bound converts exactly or, under 2^-14, to within
 * 2^-25) - AX_ERR_UNSUPPORTED otherwise; AX_F32 takes any sizes with an even head_dim <= 256.
 * Needs a GPU (uploads the rotary table, repacks the weights; synchronises the device).  Errors: INVALID, OOM (workspace too small),
 * UNSUPPORTED, DEVICE. */
ax_status ax_model_create(const ax_model_config *cfg, const ax_weights *weights,
                          void *workspace, size_t workspace_bytes, ax_model **out);
void ax_model_destroy(ax_model *m);

/* ---- paged KV pool -------------------------------------------------------------------------
 * The pool divides `dev_mem` into blocks of `block_tokens` positions (all layers, K and V).
 * A sequence (ax_kv) is a list of block ids plus a length; blocks are reference counted so
 * that sequences sharing a prefix share its blocks (prefix caching: the cache of a common
 * prefix is valid for every continuation, Sec. 2.3).  Device layout, element type = dtype:
 *   K: [layer][kv_head][block][token in block][head_dim]
 *   V: [layer][kv_head][block][head_dim][token in block]      (token-minor)
 * Block bookkeeping is host only and never touches or waits for the device.              */

/* Bytes one block occupies = 2 * n_layers * n_kv_heads * head_dim * block_tokens * itemsize. */
size_t ax_pool_block_bytes(const ax_model_config *cfg, int block_tokens);

/* `dev_mem` need not be initialised: slots past the end of a sequence are never used, whatever
 * they hold.  It may be NULL only for host-side bookkeeping tests (no ax_extend on such a pool).
 * block_tokens must be 16.  The pool holds floor(bytes / block_bytes) blocks (>= 1).      */
ax_status ax_pool_create(const ax_model_config *cfg, void *dev_mem, size_t bytes,
                         int block_tokens, ax_pool **out);
/* AX_ERR_STATE (and nothing destroyed) while sequences of the pool are alive. */
ax_status ax_pool_destroy(ax_pool *p);
/* Free blocks / total blocks / live sequences; any pointer may be NULL. */
ax_status ax_pool_stats(const ax_pool *p, int64_t *free_blocks, int64_t *total_blocks,
                        int64_t *live_seqs);

/* New empty sequence. */
ax_status ax_kv_alloc(ax_pool *p, ax_kv **out);
/* New sequence holding the first n_tokens positions of src (-1 = all of them) by sharing its
 * blocks (refcount + 1 each); no data moves.  A later append into a shared, partly filled
 * last block copies that block first (copy on write).  Errors: INVALID (n_tokens > len). */
ax_status ax_kv_fork(const ax_kv *src, int64_t n_tokens, ax_kv **out);
/* Cut the sequence back to new_len <= len positions and release blocks wholly beyond it:
 * rollback of rejected drafts (Sec. 2.3), or removal of the mismatched tail of a cached
 * prompt (Sec. 4.2).  Device memory is not touched; stale slots are overwritten later. */
ax_status ax_kv_truncate(ax_kv *kv, int64_t new_len);
/* Length in tokens, or -1 for a bad handle. */
int64_t ax_kv_len(const ax_kv *kv);
/* Drop the sequence: refcount - 1 on each of its blocks, blocks reaching 0 return to the pool. */
ax_status ax_kv_free(ax_kv *kv);
/* Introspection for tests: copies up to cap block ids to ids (host), returns the block count
 * (or -1); refcount of one block of a pool (or -1). */
int64_t ax_kv_blocks(const ax_kv *kv, int32_t *ids, int64_t cap);
int ax_pool_refcount(const ax_pool *p, int64_t block);
/* Host half of an append, exposed so block logic can be tested without a GPU: reserves room
 * for n more positions (allocating blocks, and replacing a shared partly filled last block by
 * a private one), advances the length and reports the copy-on-write copy it would have
 * launched as (*cow_src, *cow_dst), -1/-1 if none.  Errors: OOM with nothing changed. */
ax_status ax_kv_reserve_host(ax_kv *kv, int64_t n, int32_t *cow_src, int32_t *cow_dst);

/* ---- forward -------------------------------------------------------------------------------
 * Runs tokens[0..T) (host, int32) at positions P..P+T-1 where P = ax_kv_len(kv), appends their
 * K/V to kv (length becomes P + T) and writes what out_mode asks for to `out` (device).  Row i
 * attends to positions 0..P+i.  kv must belong to a pool created with the same config as
 * `model`.  Asynchronous on hip_stream.
 * Errors: INVALID (T <= 0, T > max_tokens, P + T > max_pos, token outside [0, vocab), NULL out
 * for a mode that writes), OOM (no free KV block; kv unchanged), DEVICE. */
ax_status ax_extend(ax_model *model, ax_kv *kv, const int32_t *tokens, int T,
                    int out_mode, void *out, void *hip_stream);

/* The same for n sequences in one pass (weights are read once for all sum(T_each) rows).
 * tokens_concat holds the sequences' tokens back to back; outputs are in the same order.
 * The sequences must be distinct and live in one pool. */
ax_status ax_extend_batch(ax_model *model, int n, ax_kv *const *kvs, const int32_t *tokens_concat,
                          const int *T_each, int out_mode, void *out, void *hip_stream);

/* One speculative round (Sec. 2.3 verification phase with greedy exact-match acceptance, as a
 * lookup-table drafter has no logits of its own, Sec. 4.3).  kv holds everything before
 * `pending`.  Runs [pending, drafts[0..k)] in one forward, takes the greedy token g_i after
 * each row, accepts the longest prefix with drafts[i] == g_i, writes *accepted = a in 0..k
 * and *next_token = g_a (host), and cuts kv back to P + 1 + a (prefix, pending, accepted
 * drafts).  The round emits drafts[0..a) then *next_token, which becomes the next pending
 * token and is not yet in kv.  k = 0 is plain one-token decoding (the fallback of Sec. 4.3).
 * Waits for the result.  Errors as ax_extend; kv is unchanged on error. */
ax_status ax_verify(ax_model *model, ax_kv *kv, int32_t pending, const int32_t *drafts, int k,
                    int *accepted, int32_t *next_token, void *hip_stream);

/* ax_verify over n sequences of one pool in a single forward (the round itself is that of Sec. 2.3
 * and Sec. 4.3; running several agent sessions through one forward is this library's addition, the
 * paper evaluates one session at a time): sequence s contributes the rows
 * [pending[s], its k_each[s] drafts] (drafts_concat holds the drafts back to back; host memory),
 * the weights are streamed once for all sum(1 + k_s) rows, acceptance and rollback are per
 * sequence.  accepted[s], next_token[s] (host) as in ax_verify.  All or nothing on errors. */
ax_status ax_verify_batch(ax_model *model, int n, ax_kv *const *kvs, const int32_t *pending,
                          const int32_t *drafts_concat, const int *k_each, int *accepted,
                          int32_t *next_token, void *hip_stream);

/* ---- KV images: precomputed prefixes kept outside the pool (paper Sec. 4.2, Sec. 5: the KV of
 * the static prefix and of the selected cluster combinations is computed offline, kept on
 * storage and loaded on demand).  An image is a 64-byte header (magic "AXKV", version, layers,
 * KV heads, head_dim, dtype, block size, token count, payload size) followed by the sequence's
 * blocks in logical order, each exactly as it lies in the pool; it depends on the cached values
 * only (not on block ids; the unused slots of the last block are zero).  `image` must be memory
 * the GPU can address - pinned host memory (hipHostMalloc, a pinned torch tensor: the staging
 * buffer of a file read or write) or device memory - because a kernel gathers / scatters the
 * blocks directly; other pointers are rejected with AX_ERR_INVALID.  The model lends its
 * descriptor ring; pool and model geometry must match. */
int64_t ax_kv_image_bytes(const ax_pool *p, int64_t n_tokens);          /* -1 on bad arguments */
/* Writes the image of the first n_tokens (-1 = all) of kv; returns after the image is complete. */
ax_status ax_kv_export(ax_model *model, const ax_kv *kv, int64_t n_tokens, void *image,
                       int64_t image_bytes, void *hip_stream);
/* ax_kv_export for callers that cannot allocate or wait: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same image, byte for byte, but no model is needed (the
 * block-id list the gather kernel walks is staged in a fixed 64 KiB device array of the library's
 * own instead of a model's workspace) and nothing is allocated, copied through host staging or
 * waited for: the call enqueues a few kernels on hip_stream and returns; the image is complete once
 * the stream has passed them.  The pool's memory must live on the current device.  Limit: 16 384
 * blocks (262 144 tokens), AX_ERR_UNSUPPORTED beyond.  `image` must be 4-byte aligned.
 * All calls on one GPU share that GPU's array: calls on one stream are ordered, calls that overlap
 * on different streams race on it.  Nothing in it has to start out as zero - every id a call reads
 * it has staged itself. */
ax_status ax_kv_export_static(const ax_kv *kv, int64_t n_tokens, void *image, int64_t image_bytes,
                              void *hip_stream);
/* Creates a sequence in `pool` holding the image's tokens.  Only enqueues: the image must stay
 * valid and unchanged until the stream has passed the copy; later calls on the same stream see
 * the imported values.  AX_ERR_OOM (nothing changed) if the pool lacks the blocks. */
ax_status ax_kv_import(ax_model *model, ax_pool *pool, const void *image, int64_t image_bytes,
                       ax_kv **out, void *hip_stream);

/* ---- automatic prefix reuse (paper Sec. 2.3, "Prefix caching": KV is reused for all tokens before
 * the first one that differs; Sec. 4.2: a cached "1-3-2" serves a prompt that activates "1-3" by cutting the
 * tail).  An index remembers which token sequence each registered KV holds.  Host only.
 * The index keeps its own reference (a fork) to every registered sequence, so the blocks stay
 * alive after the caller frees its handle; destroy the index before its pool. */
typedef struct ax_index ax_index;
ax_status ax_index_create(ax_pool *pool, ax_index **out);
void ax_index_destroy(ax_index *index);
int64_t ax_index_entries(const ax_index *index);                        /* -1 for a bad handle */
/* Registers that the first n positions of kv cache `tokens` (host).  n <= length of kv. */
ax_status ax_index_insert(ax_index *index, const ax_kv *kv, const int32_t *tokens, int64_t n);
/* New sequence sharing the blocks of the registered sequence with the longest common prefix with
 * `prompt` (token granular; the first registered among equals), cut to that prefix and to at most
 * max_reuse tokens (-1 = no limit; pass n - 1 to keep one token to run).  *matched = reused
 * tokens; with no match *out is an empty sequence.  The caller extends *out with
 * prompt[matched..n) - a shared, partly filled last block is copied on that write - and frees it. */
ax_status ax_index_match(ax_index *index, const int32_t *prompt, int64_t n, int64_t max_reuse,
                         ax_kv **out, int64_t *matched);

/* ---- offline selection of the cluster combinations to precompute (paper Sec. 4.2, Algorithm 1).
 * A sample is the ordered list of clusters it activates (sample i has sample_len[i] ids, all
 * samples back to back in samples_concat).  `budget` rounds; each adds the prefix - a single
 * cluster, or a chosen prefix extended by one cluster - whose addition raises the coverage (sum
 * over samples of the number of leading clusters found in the chosen set) most; equal gains go to
 * the smallest prefix in lexicographic order of cluster ids.  Stops early when no candidate is
 * left.  Outputs: the chosen prefixes back to back in chosen_concat (capacity chosen_cap ids),
 * their lengths, the coverage after each round (optional), and their number.  Host only. */
ax_status ax_select_combinations(const int32_t *samples_concat, const int32_t *sample_len,
                                 int64_t n_samples, int budget, int32_t *chosen_concat,
                                 int64_t chosen_cap, int32_t *chosen_len, int64_t *coverage_after,
                                 int *n_chosen);
/* Coverage of a cached set as defined above; -1 on bad arguments. */
int64_t ax_coverage(const int32_t *samples_concat, const int32_t *sample_len, int64_t n_samples,
                    const int32_t *cached_concat, const int32_t *cached_len, int64_t n_cached);

/* ---- example-based drafter and decode loop (paper Sec. 4.3) -------------------------------------
 * A per-query n-gram lookup table: a window of n tokens slides over `stream` (the few-shot
 * examples followed by the user query; host memory) one token at a time; the first n-1 tokens
 * are the key, the value is the next token seen most often with that key (ties: the one
 * recorded first).  Host only, O(n_tokens).  n >= 1, vocab > 0, tokens in [0, vocab). */
typedef struct ax_lut ax_lut;
ax_status ax_lut_build(const int32_t *stream, int64_t n_tokens, int n, int vocab, ax_lut **out);
void ax_lut_free(ax_lut *lut);
/* Number of keys, or -1 for a bad handle. */
int64_t ax_lut_size(const ax_lut *lut);
/* Drafts after `context` (host, most recent token last): the table's answer to the last n-1
 * tokens, appended to the context, k times.  selective != 0: if the first lookup misses, no draft
 * is produced (the caller decodes one token normally).  A miss after a first hit - or any miss
 * when selective == 0 - yields splitmix64(seed + stream_pos + i) % vocab for draft i: a guess that
 * verification will reject.  Writes the drafts to drafts[0..k) and returns how many (0 or k),
 * -1 on bad arguments; *hits (optional) = drafts that came from the table. */
int ax_lut_draft(const ax_lut *lut, const int32_t *context, int64_t n_context, int k, int selective,
                 uint64_t seed, int64_t stream_pos, int32_t *drafts, int *hits);

typedef struct {
    int64_t rounds;      /* verification forwards run                                   */
    int64_t fallbacks;   /* rounds decoded without speculation (first lookup missed)    */
    int64_t drafted;     /* draft tokens generated                                      */
    int64_t accepted;    /* draft tokens accepted; accuracy = accepted / drafted        */
} ax_exspec_stats;

/* The decode loop: repeat { draft from the table (context = history, pending, everything emitted
 * so far); ax_verify } until max_new tokens follow `pending`.  kv holds everything before
 * `pending`; `history` (host, may be NULL) are the tokens before `pending` the drafter may use as
 * context.  Never drafts past max_new.  out_tokens[0..max_new) (host) receives the tokens; they
 * equal one-token-at-a-time greedy decoding whatever the table holds.  On return kv holds
 * everything except the last emitted token (the next pending one).  Errors as ax_verify. */
ax_status ax_exspec_generate(ax_model *model, ax_kv *kv, const ax_lut *lut, const int32_t *history,
                             int64_t n_history, int32_t pending, int max_new, int k, int selective,
                             uint64_t seed, int32_t *out_tokens, ax_exspec_stats *stats, void *hip_stream);

/* Text for the last failing call on this thread (static storage, never NULL). */
const char *ax_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* AGENTX_H */

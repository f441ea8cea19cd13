/*
 * dllm.h -- C ABI of the MI355X (gfx950) denoise-step library for masked-diffusion LLM decoding.
 *
 * The calls follow the decoding problem as the d3LLM paper (arxiv 2601.07568) states it in
 * Section 3.2: a block of query tokens, some of them the special mask id, is run through a
 * bidirectional transformer against a cache of the key/value states of the prompt and of the
 * completed blocks ("KV-Cache and KV-Refresh Mechanism"); for every masked position the model's
 * distribution over the vocabulary is reduced to a candidate token and a confidence, and the
 * positions that are confident enough, but never fewer than a floor, are unmasked in parallel
 * ("Entropy-Based Multi-Block Parallel Decoding").  From time to time a forward pass that does
 * not use the cache recomputes the cached states.
 *
 * General rules
 *   - Every pointer named "dev" is DEVICE memory owned by the caller (e.g. a PyTorch-ROCm
 *     tensor's data_ptr()).  The library allocates no device memory and frees none.  Pointers in
 *     dllm_weights, the KV pool and the workspace are borrowed for the life of the context; all
 *     other pointers for the duration of the call (the call is asynchronous: "duration" ends
 *     when the work enqueued on the stream has run).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue; they never synchronise and read no device value on the host, so a sequence of
 *     calls can be captured into a HIP graph.
 *   - Return value: DLLM_OK or a negative DLLM_E* code.  Arguments are validated on the host
 *     before anything is launched; on error nothing has been enqueued.  Values that live in
 *     device memory (token ids, block-table entries, lengths) are bounds-checked by the kernels:
 *     an offending access is skipped and a bit is set in the context's device status word
 *     (dllm_read_status).  Nothing aborts, throws or prints.
 *   - Calls on one context must not overlap in time (they share the workspace).
 *
 * Data layout
 *   - dtype DLLM_F32: weights, KV pool and inter-kernel activations are float.  DLLM_BF16: they
 *     are bfloat16 (the residual stream, softmax statistics and all accumulators stay float).
 *   - Linear weights are [out_features, in_features] row-major, no biases; norm gains [d_model];
 *     tok_emb and lm_head are [vocab, d_model] (untied).
 *   - KV pool: 2 * n_layers slabs of n_pages * n_kv_heads * page_tokens * head_dim elements, slab
 *     2l = K of layer l, slab 2l+1 = V of layer l.  Within a slab, (page p, kv head h, slot s,
 *     channel c) is at ((p * n_kv_heads + h) * page_tokens + s) * head_dim + c for K, and at
 *     ((p * n_kv_heads + h) * head_dim + c) * page_tokens + s for V (V is stored transposed, the
 *     slots of one channel contiguous, which is the operand layout of the P*V matrix
 *     instruction).  K is stored after the rotary embedding.  Position j of sequence b lives in
 *     page block_table[b * max_pages_per_seq + j / page_tokens], slot j % page_tokens.
 *   - Rounding points of a DLLM_BF16 model (everything else is float): the gain-scaled input of a
 *     normalised product, bf16(x * gain) - the row factor 1/sqrt(mean(x^2) + eps) stays float and
 *     multiplies the product's float sums -, q and k after the rotary embedding, v, the attention
 *     output, silu(gate) * up.
 *   - Rotary embedding: half-split pairing (c, c + head_dim/2), angle = position * rope_base^(-2c/head_dim),
 *     positions counted from the start of the sequence.
 */
#ifndef DLLM_H
#define DLLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DLLM_OK        0
#define DLLM_EINVAL   (-1)  /* null pointer, negative or inconsistent argument                  */
#define DLLM_ESHAPE   (-2)  /* shape not supported (see dllm_create) or above the configured max */
#define DLLM_ENOSPACE (-3)  /* workspace or KV pool smaller than required                        */
#define DLLM_EHIP     (-4)  /* a launch failed; dllm_last_hip_error() has the runtime's text     */

#define DLLM_F32  0
#define DLLM_BF16 1

/* bits of the device status word */
#define DLLM_STATUS_BAD_TOKEN 1  /* a token id outside [0, vocab) was read (row 0 was used)       */
#define DLLM_STATUS_BAD_PAGE  2  /* a block-table entry outside [0, n_pages), or a position beyond
                                    max_pages_per_seq * page_tokens (access skipped)              */
#define DLLM_STATUS_ROWS_CAP  4  /* more masked rows than max_batch * max_q in a refresh call      */
#define DLLM_STATUS_BAD_LENGTH 8 /* a device-resident length disagrees with the host value that sized the
                                    launch: prefix_len[b] outside [0, max_prefix_len], a sequence longer than
                                    max_seqlen, cu_seqlens[0] != 0 or cu_seqlens[B] != total_tokens (the
                                    length was clamped; rows left without a sequence are skipped)          */

typedef struct dllm_ctx dllm_ctx; /* opaque, host memory; holds descriptors only */

typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ff, vocab, mask_id;
  float   rms_eps, rope_base;
  int32_t dtype;             /* DLLM_F32 or DLLM_BF16                                             */
  int32_t page_tokens;       /* tokens per KV page, >= 1                                          */
  int32_t max_pages_per_seq; /* row length of every block table                                   */
  int32_t n_pages;           /* pages in the pool                                                 */
  int32_t max_batch;         /* largest B of any call                                             */
  int32_t max_q;             /* largest Q of a denoise step                                       */
  int32_t max_tokens;        /* largest total token count of a prefill / refresh call (0: unused) */
} dllm_config;

typedef struct {
  const void *attn_norm, *wq, *wk, *wv, *wo, *mlp_norm, *w_gate, *w_up, *w_down;
} dllm_layer_w;

typedef struct {
  const void *tok_emb, *final_norm, *lm_head; /* dev */
  const dllm_layer_w *layers;                 /* HOST array of n_layers records of dev pointers; copied by dllm_create */
} dllm_weights;

/* Bytes of workspace / KV pool a context with this configuration needs; 0 if the configuration
 * is invalid. */
size_t dllm_workspace_bytes(const dllm_config *cfg);
size_t dllm_kv_pool_bytes(const dllm_config *cfg);

/* Creates a context.  Supported: head_dim in {64, 128}; n_q_heads a multiple of n_kv_heads;
 * for DLLM_BF16 d_model, d_ff and n_*_heads * head_dim must be multiples of 8; mask_id in
 * [0, vocab).  kv_pool (dev) holds dllm_kv_pool_bytes, workspace (dev, 256-byte aligned) holds
 * dllm_workspace_bytes; the workspace's status word must be cleared once with
 * dllm_reset_status before the first call.  Performs no HIP call. */
int dllm_create(dllm_ctx **out, const dllm_config *cfg, const dllm_weights *w,
                void *kv_pool, size_t kv_pool_bytes, void *workspace, size_t workspace_bytes);
void dllm_destroy(dllm_ctx *ctx);

/* Weight packing for the matrix-core path of DLLM_BF16 models.  Batch-1 denoise steps are bound by
 * reading every weight once from HBM (the forward of Section 3.2 is run once per step on a 32-token
 * block); the kernels reach HBM speed only if a wavefront's loads are contiguous, so the linear
 * weights are re-ordered once into the operand order of the matrix instruction: 16-byte unit
 * ((rt * ceil(K/128) + kb) * 4 + j) * 64 + g*16 + c of a matrix holds row rt*16 + c, columns
 * kb*128 + j*32 + g*8 .. +7 (rows padded to 16, columns to 128, with zeros).
 * dllm_pack_weights enqueues the re-ordering of all projection matrices and of the LM head into
 * `packed` (dev, 256-byte aligned, dllm_packed_weight_bytes, borrowed for the life of the context).
 * The original weights stay in use (prefill, refresh and steps of more than 64 rows read them).
 * Until this call has been made, bfloat16 denoise steps run on the generic kernels. */
size_t dllm_packed_weight_bytes(const dllm_config *cfg);
int dllm_pack_weights(dllm_ctx *ctx, void *stream, void *packed, size_t packed_bytes);

/* Prefill (Section 3.2, "KV-Cache"): one bidirectional forward without cache over B packed
 * sequences -- sequence b is tokens[cu_seqlens[b] .. cu_seqlens[b+1]), every token attends to every
 * token of its sequence -- and stores the K/V states of its first n_cache[b] positions (all of
 * them if n_cache is NULL) of every layer into the pages block_table maps.  No LM head.
 *   tokens      dev int32 [total_tokens]      cu_seqlens  dev int32 [B+1], cu_seqlens[0] = 0
 *   n_cache     dev int32 [B] or NULL         block_table dev int32 [B, max_pages_per_seq]
 *   total_tokens = cu_seqlens[B] and max_seqlen >= every sequence length are passed by value
 *   (host), they size the launches. */
int dllm_prefill_kv(dllm_ctx *ctx, void *stream, int B, int total_tokens, int max_seqlen,
                    const int32_t *tokens, const int32_t *cu_seqlens, const int32_t *n_cache,
                    const int32_t *block_table);

/* One denoising forward (Section 3.2): for each sequence b, Q query tokens at positions
 * prefix_len[b] .. prefix_len[b]+Q-1 attend, without any mask, to the cached prefix
 * [0, prefix_len[b]) and to one another.  Their K/V are written into the pages the block table
 * maps for those positions (in-flight pages; nothing below prefix_len[b] is written).  For
 * every row whose token is mask_id the distribution over the vocabulary (mask_id column
 * excluded) is reduced on the fly -- the logits are never stored --
 * to cand_token = arg max (lowest id on ties), conf = its softmax probability, and optionally
 * entropy (nats).  Rows that are not masked get cand_token = their own token, conf = 1,
 * entropy = 0.
 *   q_tokens dev int32 [B, Q]    prefix_len dev int32 [B]    block_table dev int32 [B, max_pages_per_seq]
 *   cand_token dev int32 [B, Q]  conf dev float [B, Q]       entropy dev float [B, Q] or NULL
 *   max_prefix_len (host) >= every prefix_len[b]; it only sizes the launch. */
int dllm_denoise_step(dllm_ctx *ctx, void *stream, int B, int Q, int max_prefix_len,
                      const int32_t *q_tokens, const int32_t *prefix_len,
                      const int32_t *block_table, int32_t *cand_token, float *conf,
                      float *entropy);

/* dllm_denoise_step for callers that cannot allocate device memory or bring a workspace of their own
 * into the call: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same kernels and same results as dllm_denoise_step, but every intermediate of the
 * step lives in a device array inside the library (DLLM_STATIC_SCRATCH_BYTES = 64 MiB, held by every GPU
 * the library runs on until the process ends) instead of the context's workspace; the call allocates
 * nothing and frees nothing.  The context must be one whose dllm_workspace_bytes fits the array
 * (a batch-1 step of 32 rows at the 8B shape needs 54 MiB), otherwise DLLM_ENOSPACE is returned and
 * nothing is enqueued.  Status bits raised by the step are merged into the context's status word.
 * All calls on one GPU share the one array, whatever their context: calls that overlap in time on
 * a GPU race.  The array keeps the last call's contents; the call clears what it needs cleared. */
#define DLLM_STATIC_SCRATCH_BYTES (64u << 20)
size_t dllm_static_scratch_bytes(void);
int dllm_denoise_step_static(dllm_ctx *ctx, void *stream, int B, int Q, int max_prefix_len,
                             const int32_t *q_tokens, const int32_t *prefix_len,
                             const int32_t *block_table, int32_t *cand_token, float *conf,
                             float *entropy);

/* Threshold-based parallel unmasking with a floor (Section 3.2: tokens that pass the threshold
 * are decoded, and at least a minimum number per forward regardless of the threshold; with
 * threshold > 1 and min_unmask = 1 this is the one-token-per-step rule of Section 3.1).
 * The Q positions of each sequence are treated as Q / block_len independent blocks.  Within a
 * block, every masked position with conf >= threshold is unmasked, and so are the
 * min(min_unmask, #masked) masked positions that come first when ordered by confidence
 * descending, index ascending (NaN confidences come last).  Unmasking position i sets
 * q_tokens[i] = cand_token[i]; other positions are left untouched.
 *   q_tokens dev int32 [B, Q] in/out    n_unmasked, n_remaining dev int32 [B, Q / block_len] or NULL
 *   Requires Q % block_len == 0, 1 <= block_len <= 1024, min_unmask >= 0 (0 = threshold only, the
 *   conservative strategy Section 3.2 gives a newly activated block). */
int dllm_unmask(dllm_ctx *ctx, void *stream, int B, int Q, int block_len, int32_t *q_tokens,
                const int32_t *cand_token, const float *conf, float threshold, int min_unmask,
                int32_t *n_unmasked, int32_t *n_remaining);

/* The same selection on the entropy of the predictive distribution (Section 3.2, "Entropy-Based
 * Multi-Block Parallel Decoding": positions that meet the entropy threshold are decoded, lower
 * entropy first; Appendix, inference settings: thresholds of 0.4 to 0.5).  Within a block every
 * masked position with entropy <= theta is unmasked, and so are the min(min_unmask, #masked)
 * masked positions that come first when ordered by entropy ascending, index ascending (NaN
 * entropies come last).  entropy is the array dllm_denoise_step / dllm_refresh_cache write (nats).
 * Arguments, layouts and limits as for dllm_unmask. */
int dllm_unmask_entropy(dllm_ctx *ctx, void *stream, int B, int Q, int block_len, int32_t *q_tokens,
                        const int32_t *cand_token, const float *entropy, float theta, int min_unmask,
                        int32_t *n_unmasked, int32_t *n_remaining);

/* The selection with a floor per block (Section 3.2: a newly activated block decodes only what meets
 * the threshold, a fully activated one at least one position per forward).  stat is the confidence
 * (by_entropy = 0: positions with stat >= threshold pass, highest first) or the entropy (by_entropy
 * != 0: positions with stat <= threshold pass, lowest first).  floor[b, k] >= 0 is the floor of block k
 * of sequence b; a negative entry leaves that block untouched (its counts are still reported).
 *   floor dev int32 [B, Q / block_len]; everything else as for dllm_unmask. */
int dllm_unmask_blocks(dllm_ctx *ctx, void *stream, int B, int Q, int block_len, int32_t *q_tokens,
                       const int32_t *cand_token, const float *stat, float threshold, int by_entropy,
                       const int32_t *floor, int32_t *n_unmasked, int32_t *n_remaining);

/* Block states of multi-block decoding (Section 3.2: Inactive, Activated, Fully-Activated, Completed
 * but Stabilizing, Completed) and their transitions after a round, evaluated on the device from the
 * generation tokens themselves.  In block order, with filled = unmasked positions of a block and
 * prev = filled of the block before it (the first block's predecessor counts as complete):
 *   Stabilizing: counter -= 1 if the round's forward did not use the cache (nocache_round != 0);
 *                becomes Completed once counter <= 0 and the block before it is Completed;
 *   Activated / Fully-Activated: becomes Stabilizing with counter = delay when filled == block_len;
 *                an Activated block becomes Fully-Activated when prev / block_len >= full_at;
 *   the first Inactive block: becomes Activated when the block before it is not Inactive and
 *                prev / block_len >= add_at (Fully-Activated at once if also >= full_at).
 * Appendix, inference settings: add_at 0.1, full_at 0.95, delay 1 or 2.  The ratios are compared in
 * double precision on the host side of the call (converted to counts).
 *   gen_tokens dev int32 [B, n_blocks * block_len]   the generation part of each sequence
 *   state, counter dev int32 [B, n_blocks] in/out    state values DLLM_BLOCK_*
 *   floor_next dev int32 [B, n_blocks] or NULL       floors for dllm_unmask_blocks in the next round:
 *                                                    1 Fully-Activated, 0 Activated, -1 otherwise
 *   summary dev int32 [B, 4] or NULL                 first and last active block (-1 if none), whether a
 *                                                    block is Stabilizing (the next forward must not use
 *                                                    the cache), number of Completed blocks
 *   Requires 1 <= n_blocks <= DLLM_FSM_MAX_BLOCKS, delay >= 0. */
#define DLLM_BLOCK_INACTIVE 0
#define DLLM_BLOCK_ACTIVATED 1
#define DLLM_BLOCK_FULLY_ACTIVATED 2
#define DLLM_BLOCK_STABILIZING 3
#define DLLM_BLOCK_COMPLETED 4
#define DLLM_FSM_MAX_BLOCKS 256
int dllm_fsm_update(dllm_ctx *ctx, void *stream, int B, int n_blocks, int block_len, const int32_t *gen_tokens,
                    int32_t *state, int32_t *counter, double add_at, double full_at, int delay, int nocache_round,
                    int32_t *floor_next, int32_t *summary);
/* nocache_round < 0: derived per sequence - the round skipped the cache iff one of the sequence's blocks was
 * Stabilizing in the incoming state (the rule by which the forward of a round is chosen).  The library only
 * counts: running that forward (dllm_refresh_cache with the step outputs) for those sequences before this call
 * is the caller's part. */

/* The plan of the next round of multi-block decoding, per sequence, from the block states dllm_fsm_update has left
 * (Section 3.2: forward passes without the cache while a block is Completed but Stabilizing, which refresh the previous
 * caches, and a periodic refresh that updates the cache every few rounds).  On entry nocache[b] tells whether the
 * round just done ran without the cache (0 before the first round); rounds_since[b] counts the cached rounds since
 * the last forward without cache and is updated.  On exit nocache[b] = 1 if the next forward must not use the cache:
 * a block is Stabilizing, or refresh_every > 0 and rounds_since[b] >= refresh_every.  n_commit_next[b] = base_len[b]
 * + block_len * (blocks that are Completed when the transitions of such a round are done: the Completed ones and the
 * Stabilizing ones behind them whose count-down ends with it) - the n_commit of the dllm_refresh_cache call of that
 * round, whose tokens are base_len[b] + (last active block + 1) * block_len long.
 *   state, counter dev int32 [B, n_blocks]; base_len dev int32 [B] or NULL (0); rounds_since, nocache dev int32 [B]
 *   in/out; n_commit_next dev int32 [B]; refresh_every >= 0 (0: no periodic refresh). */
int dllm_fsm_plan(dllm_ctx *ctx, void *stream, int B, int n_blocks, int block_len, const int32_t *state,
                  const int32_t *counter, const int32_t *base_len, int refresh_every, int32_t *rounds_since,
                  int32_t *nocache, int32_t *n_commit_next);

/* A denoise step whose sequences have different numbers of query rows (multi-block decoding: the windows of
 * the sequences of a batch differ): as dllm_denoise_step, but rows j >= q_valid[b] of sequence b are padding.
 * Padding rows are no keys for the other rows (sequence b attends to prefix_len[b] + q_valid[b] keys), get no
 * LM-head row, report their own token with confidence 1 and write nothing to the cache (only positions up
 * to prefix_len[b] + q_valid[b] - 1 need to be mapped by the block table).
 *   q_valid dev int32 [B], 0 <= q_valid[b] <= Q (clamped) */
int dllm_denoise_step_var(dllm_ctx *ctx, void *stream, int B, int Q, int max_prefix_len, const int32_t *q_tokens,
                          const int32_t *prefix_len, const int32_t *q_valid, const int32_t *block_table,
                          int32_t *cand_token, float *conf, float *entropy);

/* The window of a cached round of multi-block decoding, per sequence, from the block states: the run of
 * Activated / Fully-Activated blocks, at most W of them, copied out of the generation tokens into
 * win_tokens (padded with pad_token), with the floors of those blocks (-1 for padding blocks), the prefix
 * length base_len[b] + first_block * block_len and the valid-row count - the arguments of
 * dllm_denoise_step_var (Q = W * block_len) and dllm_unmask_blocks.  A sequence with a Stabilizing block
 * (its round must not use the cache) or without an active block gets an empty window (q_valid 0, floors
 * -1).  dllm_fsm_scatter writes the valid rows of the windows back into the generation tokens.
 *   gen_tokens dev int32 [B, n_blocks * block_len]; state dev int32 [B, n_blocks]; base_len dev int32 [B]
 *   win_tokens dev int32 [B, W * block_len]; win_floor dev int32 [B, W]; prefix_len, q_valid, win_lo dev int32 [B]
 *   pad_token: any token id other than the mask id. */
int dllm_fsm_window(dllm_ctx *ctx, void *stream, int B, int n_blocks, int block_len, int W, const int32_t *gen_tokens,
                    const int32_t *state, const int32_t *base_len, int32_t pad_token, int32_t *win_tokens,
                    int32_t *win_floor, int32_t *prefix_len, int32_t *q_valid, int32_t *win_lo);
int dllm_fsm_scatter(dllm_ctx *ctx, void *stream, int B, int n_blocks, int block_len, int W, const int32_t *win_tokens,
                     const int32_t *win_lo, const int32_t *q_valid, int32_t *gen_tokens);

/* A whole round of multi-block decoding without a host read (Section 3.2, multi-block paragraph): the plan of
 * dllm_fsm_plan decides on the device which sequences of the batch run the cached step and which the forward without
 * cache; every launch is sized by host capacities, so the same sequence of calls serves every round (and replays as
 * a captured graph):
 *   dllm_fsm_round_windows  windows as dllm_fsm_window, but for every sequence that has an active block, whatever its
 *                           forward; q_valid_cached[b] = q_valid[b] for the sequences of the cached step, 0 for those
 *                           with nocache[b] != 0 (they take no part in dllm_denoise_step_var);
 *   dllm_fsm_pack           the packed batch of the forward without cache: sequence b contributes, iff nocache[b] != 0
 *                           and it has an active block, its prompt (prompt_tokens[b, 0 .. base_len[b])) followed by
 *                           its generation up to the end of its window; cu_seqlens[b+1] - cu_seqlens[b] is that
 *                           length or 0, n_commit[b] = n_commit_plan[b] (dllm_fsm_plan) or 0, rows of `tokens` behind
 *                           the last sequence hold pad_token.  A sequence longer than max_seqlen, or one that does
 *                           not fit token_capacity any more, is left out and DLLM_STATUS_BAD_LENGTH is set;
 *   dllm_refresh_cache_dev  dllm_refresh_cache whose total is device-resident: token_capacity (a host value, at most
 *                           max_tokens) sizes the launches, cu_seqlens[B] <= token_capacity rows are sequences, the
 *                           rest is padding (no position, nothing cached, no LM-head row; GEMMs that tile over rows
 *                           skip them); cu_seqlens[B] = 0 is legal: the call then does nothing but launch;
 *   dllm_fsm_unpack         the step outputs of that forward (indexed by packed row) into the window layout [B, Q] of
 *                           the sequences that took part: row j < q_valid[b] of sequence b is packed row
 *                           cu_seqlens[b] + prefix_len[b] + j; the other sequences' entries are left as the cached
 *                           step wrote them.
 * Followed by dllm_unmask_blocks, dllm_fsm_scatter, dllm_fsm_update (nocache_round < 0) and dllm_fsm_plan.
 *   prompt_tokens dev int32 [B, max_prompt]; nocache, n_commit_plan dev int32 [B] (dllm_fsm_plan);
 *   tokens dev int32 [token_capacity]; cu_seqlens dev int32 [B + 1]; n_commit dev int32 [B];
 *   packed_cand / packed_conf / packed_entropy dev [token_capacity] (packed_entropy and entropy may be NULL);
 *   other arguments as for dllm_fsm_window / dllm_refresh_cache. */
int dllm_fsm_round_windows(dllm_ctx *ctx, void *stream, int B, int n_blocks, int block_len, int W,
                           const int32_t *gen_tokens, const int32_t *state, const int32_t *base_len,
                           const int32_t *nocache, int32_t pad_token, int32_t *win_tokens, int32_t *win_floor,
                           int32_t *prefix_len, int32_t *q_valid, int32_t *q_valid_cached, int32_t *win_lo);
int dllm_fsm_pack(dllm_ctx *ctx, void *stream, int B, int n_blocks, int block_len, int W, int max_prompt,
                  int token_capacity, int max_seqlen, const int32_t *prompt_tokens, const int32_t *gen_tokens,
                  const int32_t *state, const int32_t *base_len, const int32_t *nocache, const int32_t *n_commit_plan,
                  int32_t pad_token, int32_t *tokens, int32_t *cu_seqlens, int32_t *n_commit);
int dllm_refresh_cache_dev(dllm_ctx *ctx, void *stream, int B, int token_capacity, int max_seqlen,
                           const int32_t *tokens, const int32_t *cu_seqlens, const int32_t *n_commit,
                           const int32_t *block_table, int32_t *cand_token, float *conf, float *entropy);
int dllm_fsm_unpack(dllm_ctx *ctx, void *stream, int B, int Q, int token_capacity, const int32_t *cu_seqlens,
                    const int32_t *prefix_len, const int32_t *q_valid, const int32_t *nocache,
                    const int32_t *packed_cand, const float *packed_conf, const float *packed_entropy,
                    int32_t *cand_token, float *conf, float *entropy);

/* The selection of dllm_unmask / dllm_unmask_entropy that also records the decoding order (Section 3.1:
 * the teacher's pseudo-trajectory is the order in which its tokens are decoded, one per step, for the
 * full output length): order[b, i] = step_index for every position this call unmasks, other entries are
 * left as they are.  With threshold above 1 (by_entropy = 0) and min_unmask = 1 exactly one position per
 * block is decoded per call; trajectory state T_j then has position i decoded iff order[b, i] <= j.
 *   order dev int32 [B, Q] in/out; other arguments as for dllm_unmask_blocks / dllm_unmask. */
int dllm_unmask_traced(dllm_ctx *ctx, void *stream, int B, int Q, int block_len, int32_t *q_tokens,
                       const int32_t *cand_token, const float *stat, float threshold, int by_entropy, int min_unmask,
                       int32_t step_index, int32_t *order, int32_t *n_unmasked, int32_t *n_remaining);

/* Noisy sequence of pseudo-trajectory distillation (Section 3.1, the displayed case formula): given the
 * ground-truth response y, the teacher's decoding order, a decoding window {s, ..., s + k} and a ratio t,
 * position i (1-based, as in the paper; array index i - 1) of the output is y_i if i <= s, [MASK] if
 * i > s + k, and inside the window y_i iff order_i <= s + ceil(k t) (decoded in trajectory state
 * T_{s + ceil(k t)}), else [MASK].  Where the two printed cases overlap the window bounds decide.
 *   y, order dev int32 [B, n]; window_start dev int32 [B] (s per sequence); out dev int32 [B, n]
 *   Requires 0 <= t <= 1, k >= 0, B <= 65535. */
int dllm_noisy_sequence(dllm_ctx *ctx, void *stream, int B, int n, const int32_t *y, const int32_t *order,
                        const int32_t *window_start, int k, double t, int32_t *out);

/* Early stopping (Section 3.2, "Early Stopping on EOS Token"): a sequence is finished once an
 * end-of-sequence token has been decoded and no [MASK] is left before it; the caller stops issuing
 * forwards for it.  finished[b] = 1/0, first_eos[b] = index of that token or -1.  active_index lists,
 * in order, the sequences that are not finished (entries past n_active[0] are -1), for the caller to
 * gather the next call's batch from.
 *   gen_tokens dev int32 [B, n]; finished dev int32 [B]; first_eos dev int32 [B] or NULL;
 *   active_index dev int32 [B] and n_active dev int32 [1], both or neither. */
int dllm_eos_scan(dllm_ctx *ctx, void *stream, int B, int n, const int32_t *gen_tokens, int32_t eos_id,
                  int32_t *finished, int32_t *first_eos, int32_t *active_index, int32_t *n_active);

/* Ragged batch after early stopping (Section 3.2, "Early Stopping on EOS Token": a finished sequence takes part in no
 * further forward).  dllm_gather_rows moves the live sequences' rows to the front of a batch array, in the order of the
 * list dllm_eos_scan writes: dst[i] = src[index[i]] for i < n_index[0], every other row of dst = fill; rows are row_len
 * int32 values (generation tokens, prefix lengths with row_len 1, block-table rows, block states, ...).
 * dllm_scatter_rows is the way back: dst[index[i]] = src[i] for i < n_index[0], other rows of dst untouched.  An index
 * outside [0, B) addresses nothing (gather: that row is filled).
 *   index dev int32 [B]; n_index dev int32 [1] (clamped to [0, B]); src, dst dev int32 [B, row_len], distinct buffers. */
int dllm_gather_rows(dllm_ctx *ctx, void *stream, int B, int row_len, const int32_t *index, const int32_t *n_index,
                     const int32_t *src, int32_t *dst, int32_t fill);
int dllm_scatter_rows(dllm_ctx *ctx, void *stream, int B, int row_len, const int32_t *index, const int32_t *n_index,
                      const int32_t *src, int32_t *dst);

/* The denoise step over the live sequences of a compacted batch: as dllm_denoise_step_var (q_valid may be NULL: every
 * row valid), but only sequences b < n_live[0] take part.  The others cost no attention and no cache write, get no
 * LM-head row and report their own tokens with confidence 1; on the paths that tile over rows (more than 64 rows in
 * the call) the rows past the live sequences are skipped by the GEMMs as well, so a finished sequence stops consuming
 * work although B, which sizes the launches, stays a host value.
 *   n_live dev int32 [1], clamped to [0, B] (n_active of dllm_eos_scan after dllm_gather_rows). */
int dllm_denoise_step_live(dllm_ctx *ctx, void *stream, int B, int Q, int max_prefix_len, const int32_t *q_tokens,
                           const int32_t *prefix_len, const int32_t *q_valid, const int32_t *n_live,
                           const int32_t *block_table, int32_t *cand_token, float *conf, float *entropy);

/* KV refresh (Section 3.2, "KV-Refresh"; the forward passes of the "Completed but Stabilizing"
 * state): the same no-cache forward as dllm_prefill_kv over the committed tokens, optionally
 * followed by in-flight ones, overwriting the cached K/V of positions [0, n_commit[b]) (all if
 * NULL).  If cand_token is not NULL the rows at positions >= n_commit[b] are treated as a
 * denoise step without cache: cand_token / conf / entropy (dev, [total_tokens], entropy may be
 * NULL) are written for them as in dllm_denoise_step; rows below n_commit[b] are left
 * untouched.  At most max_batch * max_q masked rows are reduced per call. */
int dllm_refresh_cache(dllm_ctx *ctx, void *stream, int B, int total_tokens, int max_seqlen,
                       const int32_t *tokens, const int32_t *cu_seqlens, const int32_t *n_commit,
                       const int32_t *block_table, int32_t *cand_token, float *conf,
                       float *entropy);

/* Test hooks.  dllm_debug_logits runs the same forward as dllm_denoise_step and stores the raw
 * logits (mask_id column included) of all B*Q rows as float [B, Q, vocab].  dllm_debug_hidden
 * stops after n_layers_run layers and stores the residual stream as float [B, Q, d_model]. */
int dllm_debug_logits(dllm_ctx *ctx, void *stream, int B, int Q, int max_prefix_len,
                      const int32_t *q_tokens, const int32_t *prefix_len,
                      const int32_t *block_table, float *logits);
int dllm_debug_hidden(dllm_ctx *ctx, void *stream, int B, int Q, int max_prefix_len,
                      const int32_t *q_tokens, const int32_t *prefix_len,
                      const int32_t *block_table, int n_layers_run, float *hidden);

/* Device status word: reset enqueues a clear; read enqueues a copy to *host_out and waits for
 * the stream (the only call here that synchronises). */
int dllm_reset_status(dllm_ctx *ctx, void *stream);
int dllm_read_status(dllm_ctx *ctx, void *stream, int32_t *host_out);

/* Selects kernels: 0 = automatic (MFMA kernels where the shape allows), 1 = force the generic
 * scalar-FMA kernels (test aid). */
int dllm_set_kernel_mode(dllm_ctx *ctx, int mode);

/* Per-kernel timing for benchmarks.  While enabled, every launch of the weight-streaming GEMMs
 * and of the attention kernel inside dllm_denoise_step is bracketed by HIP events on the call's
 * stream (this perturbs end-to-end time; do not enable it in a timed region or under graph
 * capture).  dllm_profile_read waits for the stream and returns, for kernel class `cls`
 * (0 = q/k/v projection, 1 = output projection, 2 = gate/up projection, 3 = down projection,
 * 4 = LM head, 5 = attention), the number of launches since enabling, the sum of their
 * event-to-event durations in milliseconds and the sum of their algorithmic bytes (weights, or
 * K/V, read once).  At most 8192 launches are recorded; later ones are not bracketed. */
int dllm_profile_enable(dllm_ctx *ctx, int on);
int dllm_profile_read(dllm_ctx *ctx, void *stream, int cls, int32_t *n_launches, double *total_ms,
                      double *total_bytes);

/* Probes for benchmarks: the rates this chip sustains, measured with the library's own launch machinery in the same
 * run as the kernels that are held against them.  dllm_probe_hbm_read enqueues one plain streaming read of `bytes`
 * bytes at buf (dev, 16-byte aligned; every lane keeps eight 16-byte loads in flight; nothing is written but, at
 * most, one word of sink).  dllm_probe_mfma enqueues a kernel of nothing but 32x32x16 bfloat16 matrix instructions
 * on register operands (one wave per SIMD, sixteen independent accumulators) and returns the floating-point
 * operations of that launch in *flops (host); random_bits != 0 gives the operands random signs, mantissas and
 * exponents (the switching activity of real data; the rate the chip sustains depends on it), 0 values that share
 * sign and exponent.  The caller times them with events on `stream`.
 *   sink dev, at least 4 bytes. */
int dllm_probe_hbm_read(dllm_ctx *ctx, void *stream, const void *buf, size_t bytes, void *sink);
int dllm_probe_mfma(dllm_ctx *ctx, void *stream, int iters, int random_bits, void *sink, double *flops);

const char *dllm_strerror(int code);
const char *dllm_last_hip_error(const dllm_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* DLLM_H */

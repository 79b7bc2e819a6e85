/*
 * space.h -- C ABI of the SPACE auto-correct decoding step on one MI355X (gfx950).
 *
 * The operation is one iteration of the auto-correct decoding algorithm of arxiv 2402.11809
 * (Methods, "Auto-Correct Decoding Algorithm", Algorithm 1) in the greedy setting:
 *   1. a single decoder forward over the rows that are not cached yet -- the last committed
 *      token x_l, the k candidates of the previous iteration and k+1 groups of k mask tokens
 *      (Eq. 2) -- under the semi-autoregressive attention mask (Eq. 3) with position ids equal
 *      to the number of visible keys minus one (sentence after Eq. 3), against a KV cache that
 *      holds x_1..x_{l-1};
 *   2. greedy verification: candidate c_i is accepted iff it equals the argmax of the logits of
 *      the previous accepted row; the first mismatch stops the scan (Algorithm 1, the for loop);
 *      one extra token comes from the last accepted row; the k new candidates are the argmax
 *      of the mask rows that follow it (Algorithm 1, last two lines of the loop body);
 *   3. the K/V of x_l and of the accepted candidates become part of the cache, every other row
 *      of the block is dropped (commit), or the cache is shortened (rollback).
 *
 * Conventions
 *   - every pointer is marked HOST or DEVICE; device pointers are plain hipMalloc-style
 *     addresses on the current device, owned by the caller unless stated otherwise;
 *   - all matrices are bf16, row-major [out_features, in_features]; activations travel between
 *     kernels in fp32 and reach the matrix units as two bf16 planes (hi + lo, about 16 mantissa
 *     bits); the only rounding to plain bf16 is the KV cache (k after rotary, v);
 *   - every call returns SPACE_OK (0) or a negative space_status; nothing aborts or throws;
 *     space_last_error() returns the text of the last failure;
 *   - calls that take a stream only enqueue work on it (a hipStream_t passed as void*; NULL is
 *     the default stream); none of them synchronises, reads device memory on the host or
 *     allocates, so a step + commit sequence can be captured into a HIP graph;
 *   - a context may be used from one host thread at a time.
 */
#ifndef SPACE_H_
#define SPACE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum space_status {
    SPACE_OK = 0,
    SPACE_EINVAL = -1,    /* null pointer, negative size, malformed layout */
    SPACE_ESHAPE = -2,    /* a dimension the kernels do not support */
    SPACE_ECAPACITY = -3, /* block does not fit the KV cache / a buffer sized at init */
    SPACE_EHIP = -4,      /* a HIP runtime call failed */
    SPACE_ENOMEM = -5     /* device allocation failed at init */
} space_status;

typedef struct space_ctx space_ctx;       /* opaque: packed weights + scratch of one model */
typedef struct space_layout space_layout; /* opaque: which rows of a block are mask rows */

/* Model and limits.  The decoder is LLaMA-shaped (the family the paper fine-tunes, Experimental
 * Settings): pre-norm, RMSNorm with eps inside the root, rotary embedding with half-split pairing
 * (element i rotates with i + head_dim/2 by pos * rope_base^(-2i/head_dim)), SwiGLU FFN, softmax
 * scale 1/sqrt(head_dim), no biases, untied LM head.
 * Supported: head_dim 64 or 128; d_model, n_heads*head_dim multiples of 32; any ffn and vocab;
 * n_kv_heads (below; written H_kv in the layouts) dividing n_heads. */
typedef struct space_config {
    int32_t n_layers;
    int32_t d_model;
    int32_t n_heads;
    int32_t head_dim;
    int32_t ffn;
    int32_t vocab;      /* LM-head rows; the embedding table has vocab + 1 rows, the last one is the
                           mask token (Experimental Settings: the mask token is a new special token) */
    int32_t max_batch;  /* largest number of sequences in one step */
    int32_t max_rows;   /* largest number of block rows per sequence in one call, <= 1024; space_step
                           verifies blocks of at most 96 rows, longer ones are prompt chunks
                           (space_prefill) */
    int32_t max_ctx;    /* largest KV-cache capacity (positions) this context will be used with */
    float rms_eps;
    float rope_base;
    int32_t n_kv_heads; /* key/value heads: 0 or n_heads = one per query head; a divisor of n_heads =
                           grouped-query attention (query head h reads key/value head
                           h / (n_heads / n_kv_heads)), as in the 70B member of the family */
} space_config;

/* DEVICE pointers to the canonical bf16 tensors of one layer, each [out, in] row-major. */
typedef struct space_layer_weights {
    const void *attn_norm; /* [d_model] */
    const void *wq;        /* [n_heads*head_dim, d_model] */
    const void *wk;        /* [H_kv*head_dim, d_model] */
    const void *wv;        /* [H_kv*head_dim, d_model] */
    const void *wo;        /* [d_model, n_heads*head_dim] */
    const void *ffn_norm;  /* [d_model] */
    const void *w_gate;    /* [ffn, d_model] */
    const void *w_up;      /* [ffn, d_model] */
    const void *w_down;    /* [d_model, ffn] */
} space_layer_weights;

typedef struct space_weights {
    const void *embed;                 /* DEVICE [vocab + 1, d_model] */
    const void *final_norm;            /* DEVICE [d_model] */
    const void *lm_head;               /* DEVICE [vocab, d_model] */
    const space_layer_weights *layers; /* HOST array [n_layers] of DEVICE pointers */
} space_weights;

/* KV cache of `batch` sequences, memory owned by the caller (space_kv_bytes() each for k and v).
 *   k:   DEVICE bf16 [n_layers][batch][H_kv][capacity][head_dim]
 *   v:   DEVICE bf16 [n_layers][batch][H_kv][capacity/32][head_dim][32]  (each run of 32 slots
 *        is stored transposed so that a tile of V feeds the matrix unit without a shuffle)
 *   len: DEVICE int32 [batch], number of committed positions (x_1..x_{l-1} of Algorithm 1)
 * capacity is a multiple of 32.  The memory must be cleared once with space_kv_reset(); slots
 * at or beyond len hold scratch.  host_len_bound is a HOST-side upper bound of every len[b],
 * kept by the library (reset: 0; commit: += rows committed, or += the number of groups of the
 * last block when the counts live on the device); the caller may lower it to the true maximum
 * whenever it knows it.  It is what the capacity check of space_step uses.
 *
 * Paged form (block_table != NULL), for serving loops that admit and retire sequences: k and v
 * are pools of n_pages pages of 32 positions shared by all sequences,
 *   k:   DEVICE bf16 [n_layers][n_pages][H_kv][32][head_dim]
 *   v:   DEVICE bf16 [n_layers][n_pages][H_kv][head_dim][32]
 * (space_kv_pool_bytes() each), and position p of sequence b lives in page
 * block_table[b * table_stride + p / 32], slot p % 32.  capacity must be table_stride * 32.  The
 * caller owns the table (DEVICE int32) and must have filled the entries that cover positions
 * 0 .. host_len_bound + G - 1 before a step over a layout of G groups; entries outside
 * 0 .. n_pages-1 are clamped and counted by space_device_faults().  Pages never move: a view of
 * other sequences (another len / block_table / batch over the same pools) is a valid space_kv, as
 * long as a block is committed through the view (the same len pointer) that staged it.  The
 * kernels read a page as they read a 32-position run of the contiguous form, so both forms give
 * the same results bit for bit. */
typedef struct space_kv {
    void *k;
    void *v;
    int32_t *len;
    int32_t batch;
    int32_t capacity;
    int32_t host_len_bound;
    const int32_t *block_table; /* NULL: contiguous form */
    int32_t table_stride;       /* entries per sequence */
    int32_t n_pages;
} space_kv;

/* Outputs of one step; all DEVICE, caller-owned, any of them may be NULL (then not written).
 * B = batch, L = rows of the layout, G = groups of the layout. */
typedef struct space_step_out {
    float *logits;         /* [B, L, vocab]  raw logits of every block row (Algorithm 1: P)      */
    int32_t *argmax;       /* [B, L]         argmax of every row, lowest id on ties              */
    int32_t *accepted_len; /* [B]            i*: accepted candidates, 0 .. G-1                   */
    int32_t *bonus;        /* [B]            the extra token from the last accepted row          */
    int32_t *new_cands;    /* [B, max_cands] argmax of the mask rows after the last accepted row;
                                             entries beyond that group's mask count are -1       */
    int32_t max_cands;     /* row stride of new_cands                                            */
    int32_t *next_tokens;  /* [B, L_next]    tokens of the next block, laid out by `next_layout`:
                                             bonus, new candidates, mask id on mask rows         */
    int32_t *emit;         /* [B, emit_cap]  generated tokens, appended at emit_len[b]           */
    int32_t *emit_len;     /* [B]            += i* + 1 per step (never beyond emit_cap)          */
    int32_t emit_cap;
    int32_t eos_id;        /* end-of-sequence token (Algorithm 1, the check after the extra token):
                              < 0 = none.  When the tokens of a step contain it, only the tokens in
                              front of it are appended (O[:eos_index]) and finished[b] becomes 1;
                              a finished sequence appends nothing more.  Needs emit and finished. */
    int32_t *finished;     /* [B]            0 / 1, sticky; the caller clears it for a new sequence */
} space_step_out;

/* Text of the last failure on this context (or of the last failed space_init when ctx is NULL).
 * The pointer stays valid until the next failing call. */
const char *space_last_error(const space_ctx *ctx);

/* Validates `cfg`, re-packs the canonical weights into the streaming order of the projection
 * kernel (library-owned device copies: the caller may free its tensors after the call returns),
 * allocates the scratch for max_batch * max_rows rows.  Synchronous.  *out is NULL on failure.
 * Layers may be left out here (all nine pointers NULL) and handed over with space_load_layer. */
int space_init(const space_config *cfg, const space_weights *weights, space_ctx **out);

/* Hands over one layer after space_init: a layer whose nine pointers were all NULL in
 * space_init's `weights->layers` is packed here instead (same tensors, same layouts), so that a
 * model whose canonical and packed copies do not fit the device together can be loaded layer by
 * layer, the caller freeing each canonical layer when the call returns.  Synchronous.  space_step
 * fails with SPACE_EINVAL while a layer is missing.  SPACE_EINVAL: null pointer, bad index, or a
 * layer that was loaded before. */
int space_load_layer(space_ctx *ctx, int32_t layer, const space_layer_weights *weights);

/* Frees everything space_init allocated and every layout created on ctx.  NULL is a no-op. */
void space_destroy(space_ctx *ctx);

/* Describes a block of L rows per sequence (Eq. 2 restricted to the rows that are not cached).
 *   is_mask HOST uint8 [L]: 1 for a mask row.
 *   group   HOST int32 [L]: 0-based group of the row.  Rows are ordered by group; each group is
 *           one non-mask row (x_l for group 0, candidate c_g for group g) followed by its mask rows.
 * The paper's block for k masks is k+1 groups of 1+k rows; a prompt chunk is L groups of one
 * row; the first iteration (no candidates yet) is one group.  From this the library derives,
 * per row, the in-block visibility of Eq. 3 (a non-mask key is visible to every later row, a
 * mask key only to later mask rows of its own group) and the position offset
 * (#visible in-block keys - 1), which is added to len[b].
 * Returns SPACE_EINVAL for a malformed layout, SPACE_ECAPACITY if L > max_rows. */
int space_layout_create(space_ctx *ctx, int32_t n_rows, const uint8_t *is_mask, const int32_t *group,
                        space_layout **out);
void space_layout_destroy(space_ctx *ctx, space_layout *layout);

/* Bytes of each of kv.k and kv.v for this model; 0 if capacity is not a positive multiple of 32. */
size_t space_kv_bytes(const space_config *cfg, int32_t batch, int32_t capacity);

/* Bytes of each of the k and v pools of the paged form; 0 if n_pages < 1. */
size_t space_kv_pool_bytes(const space_config *cfg, int32_t n_pages);

/* Clears k, v and len of a cache (fill kernels on `stream`), sets host_len_bound = 0.  Paged form:
 * clears the whole pools and the len entries of this view. */
int space_kv_reset(space_ctx *ctx, space_kv *kv, void *stream);

/* One model invocation + verification (steps 1 and 2 above) for kv->batch sequences.
 *   tokens      DEVICE int32 [B, L]; ids in [0, vocab]; the id on mask rows is ignored (the mask
 *               embedding, row `vocab`, is used).  May alias out->next_tokens.
 *   layout      rows of this block; next_layout (may be NULL) shapes out->next_tokens.
 * K/V of every block row are staged inside ctx; K/V of non-mask row g are also written to cache
 * slot len[b] + g, which is where a later commit makes them visible.  len is not changed.
 * Errors: SPACE_EINVAL (null), SPACE_ECAPACITY (B > max_batch, capacity > max_ctx, B * L >
 * max_batch * max_rows, or host_len_bound + G > capacity), SPACE_ESHAPE (L > 96).
 * A token id outside [0, vocab] or a write beyond capacity detected on the device is clamped /
 * skipped and recorded; space_device_faults() reports it. */
int space_step(space_ctx *ctx, const int32_t *tokens, const space_layout *layout,
               const space_layout *next_layout, space_kv *kv, const space_step_out *out, void *stream);

/* The same forward without the LM head and the verification: what Algorithm 1 needs of the prompt
 * x_1 .. x_{l-1} is only their keys and values.  Any layout is allowed (a prompt chunk is L groups
 * of one row), L up to max_rows (B * L <= max_batch * max_rows); the last layer stops after its
 * keys and values are stored.  The block is staged as by space_step: commit it with
 * space_kv_commit(ctx, kv, NULL, G - 1, stream).  Errors as space_step. */
int space_prefill(space_ctx *ctx, const int32_t *tokens, const space_layout *layout, space_kv *kv, void *stream);

/* Step 3, commit: len[b] += accepted + 1, i.e. x_l and the accepted candidates of the block staged
 * by the last space_step on this cache become visible; everything else is dropped.
 *   accepted_len DEVICE int32 [B] (values are clamped to 0 .. G-1), or NULL to commit
 *   `accepted_all` candidates (0 .. G-1) for every sequence, e.g. L-1 for a prompt chunk.
 * O(1): the rows were written in place by the step.  SPACE_EINVAL without a staged block. */
int space_kv_commit(space_ctx *ctx, space_kv *kv, const int32_t *accepted_len, int32_t accepted_all,
                    void *stream);

/* Step 3, rollback: drops the staged block and shortens the cache, len[b] = max(0, len[b] - n[b]).
 *   n DEVICE int32 [B], or NULL to remove `n_all` (>= 0) positions from every sequence. */
int space_kv_rollback(space_ctx *ctx, space_kv *kv, const int32_t *n, int32_t n_all, void *stream);

/* Verification by rejection sampling: lines 6-22 of Algorithm 1 as printed, on the logits a
 * space_step wrote (step_out.logits), with the warping of the appendix "Random Sampling"
 * (top-k, then top-p over the softmax of the kept logits; the paper's runs use 10 and 0.95).
 * All arithmetic is float32 in a fixed order; the random numbers are inputs.  For a layout with
 * G groups (candidates c_1 .. c_{G-1} are the non-mask rows of groups 1 .. G-1):
 *   Q = warp(row of x_l); for i = 1 .. G-1: accept c_i iff uniforms[i-1] <= Q(c_i) / p_c[i-1], then
 *   Q = warp(row of c_i); stop at the first rejection.  extra ~ Q with uniforms[G-1] (inverse CDF
 *   over the kept tokens in descending probability, ties by lowest id).  The new candidates are
 *   drawn from the warped mask rows behind the last accepted row with uniforms[G+j]; new_pc holds
 *   their probabilities (the next step's p_c).
 * residual != 0 replaces the extra token's distribution after a rejection of slot i by
 * norm(max(0, Q - D_i)), D_i being the distribution c_i was drawn from (draft_ids / draft_probs,
 * i.e. the previous call's new_ids / new_probs): the rule of the speculative-sampling papers the
 * paper cites, which makes the output law equal the model's. */
#define SPACE_MAX_TOP_K 64
typedef struct space_sample_params {
    int32_t top_k;    /* 1 .. SPACE_MAX_TOP_K */
    float top_p;      /* (0, 1] */
    int32_t residual; /* 0: extra ~ Q as printed in Algorithm 1 */
} space_sample_params;

/* All pointers DEVICE and caller-owned.  B = batch, L / G = rows / groups of `layout`.
 * Inputs: logits, tokens, p_c, uniforms are required; draft_* only when residual != 0.
 * Outputs may be NULL (then not written) except accepted_len, extra, new_cands, new_pc. */
typedef struct space_sample_io {
    const float *logits;      /* [B, L, vocab] */
    const int32_t *tokens;    /* [B, L]  the block that produced the logits                       */
    const float *p_c;         /* [B, max_cands]  P_c of the candidates; +inf rejects (first step) */
    const float *uniforms;    /* [B, G + max_cands]  numbers in [0, 1), order as above            */
    const int32_t *draft_ids; /* [B, max_cands, top_k]  kept ids of each draft distribution, -1 pads */
    const float *draft_probs; /* [B, max_cands, top_k] */
    int32_t *accepted_len;    /* [B] */
    int32_t *extra;           /* [B] */
    int32_t *new_cands;       /* [B, max_cands]  -1 beyond the group's mask count */
    float *new_pc;            /* [B, max_cands] */
    int32_t max_cands;
    int32_t *new_ids;         /* [B, max_cands, top_k]  distributions the new candidates were drawn from */
    float *new_probs;         /* [B, max_cands, top_k] */
    int32_t *next_tokens;     /* [B, L_next]  as in space_step_out (needs next_layout)            */
    int32_t *emit;            /* [B, emit_cap] */
    int32_t *emit_len;        /* [B] */
    int32_t emit_cap;
    float *ratios;            /* [B, G-1]  quotient of every test made, -1 for tests not reached   */
    int32_t eos_id;           /* as in space_step_out; < 0 = none */
    int32_t *finished;        /* [B] */
} space_sample_io;

/* Asynchronous on `stream`; no allocation, no host synchronisation.  Pass io->accepted_len to the
 * following space_kv_commit, as after a greedy step.  Errors: SPACE_EINVAL (null / missing buffer, top_k or top_p out of range, residual
 * without draft buffers, max_cands < the largest mask group), SPACE_ECAPACITY (batch * L beyond
 * max_batch * max_rows). */
int space_sample_verify(space_ctx *ctx, int32_t batch, const space_layout *layout, const space_layout *next_layout,
                        const space_sample_params *params, const space_sample_io *io, void *stream);

/* The same verification for callers that cannot allocate or depend on allocations: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Identical arguments, checks
 * and results (bit for bit) as space_sample_verify, but the per-row lists the two kernels exchange
 * live in a fixed array inside the library's device image instead of in memory space_init allocated;
 * the call itself allocates nothing and frees nothing, on the host or on the device.
 * Limit: batch * L <= SPACE_STATIC_MAX_ROWS (532 KB of device memory per GPU, held until the process
 * ends); beyond it the call returns SPACE_ECAPACITY and launches nothing.  The array keeps the
 * last call's contents; every entry a call reads is written by that call first, so nothing has to be
 * cleared.  All calls on one GPU (from any context or stream) share the array: two calls that
 * overlap in time on one GPU race, so keep them on one stream or order them with events. */
#define SPACE_STATIC_MAX_ROWS 1024
int space_sample_verify_static(space_ctx *ctx, int32_t batch, const space_layout *layout,
                               const space_layout *next_layout, const space_sample_params *params,
                               const space_sample_io *io, void *stream);

/* Synchronises `stream` and returns the number of device-side faults recorded since the last
 * call (token id out of range, cache slot beyond capacity), or a negative space_status. */
int space_device_faults(space_ctx *ctx, void *stream);

/* Training half of the method (Methods, "Semi-Autoregressive Finetuning").
 *
 * space_sar_transform is the modified dataloader, on the HOST: `tokens` holds a prompt of n_prompt
 * tokens followed by an answer y_1 .. y_N of n_answer tokens.  With u_keep < p_ar the sample stays as it
 * is (input_ids = labels = tokens, *m = 0: the autoregressive loss L_AR applies).  Otherwise the position
 * m = 1 + floor(u_pos * (N - k)), i.e. uniform over 1 .. N-k for a uniform u_pos in [0, 1), is taken and
 *   input_ids = prompt ++ y_1 .. y_{m-1} ++ k times mask_id      (the y^k_<m of the section),
 *   labels    = prompt ++ y_1 .. y_{m+k}                         (the original tokens, cut behind y_{m+k}),
 * so that in one causal forward over input_ids row i predicts labels[i + 1]: the last real token
 * predicts y_m and the j-th mask token y_{m+j} -- the k + 1 terms of the second sum of L_SAR.
 * input_ids and labels are HOST arrays with room for n_prompt + n_answer entries; the lengths and m come
 * back through n_input, n_labels and m.  (The text draws m from {0..N-k}; the equations need y_{m-1} or
 * the prompt in front of the masks and y_{m+k} behind them, which leaves 1..N-k.)
 * Errors: SPACE_EINVAL (null, n_prompt < 1, n_answer < 1, k < 0), SPACE_ESHAPE (N <= k). */
int space_sar_transform(const int32_t *tokens, int32_t n_prompt, int32_t n_answer, int32_t k, int32_t mask_id,
                        float p_ar, float u_keep, float u_pos, int32_t *input_ids, int32_t *labels,
                        int32_t *n_input, int32_t *n_labels, int32_t *m);

/* The losses of that section are sums of terms -log softmax(logits[r])[labels[r]]: L_AR over the rows in
 * front of every answer token, L_SAR over those in front of y_1 .. y_{m-1} plus the row of the last real
 * token and the k mask rows (for which space_step's logits of the one-group block [y_{m-1}, M^k] are
 * exactly the rows needed).  This call reduces any such selection:
 *   logits   DEVICE float32 [rows, vocab]   (e.g. space_step_out.logits)
 *   labels   DEVICE int32 [rows]            token the row has to predict; negative = row does not count
 *   row_loss DEVICE float32 [rows] or NULL  the terms themselves (0 on rows that do not count)
 *   loss_sum DEVICE float32 [1]             their sum, added up in row order
 *   n_terms  DEVICE int32 [1] or NULL       number of rows that count
 * float32 throughout, fixed summation order (the same inputs give the same bits).  Asynchronous on
 * `stream`.  Errors: SPACE_EINVAL (null, rows < 1), SPACE_ECAPACITY (row_loss NULL and rows beyond
 * max_batch * max_rows).  A label >= vocab is skipped and counted by space_device_faults(). */
int space_sar_loss(space_ctx *ctx, const float *logits, const int32_t *labels, int32_t rows, float *row_loss,
                   float *loss_sum, int32_t *n_terms, void *stream);

/* Tuning hook (not part of the method).  space_init reads the environment variable SPACE_TUNE once, a
 * comma-separated list of overrides of what it would otherwise pick by itself:
 *   qkv=R:S, o=R:S, gu=R:S, dn=R:S, lm=R:S   tiling of one projection: R weight tiles per wave (2, 4, 6, 8)
 *                                             and S partial sums over the contraction (1..8; gu and lm: 1);
 *   attn=N   longest context, in 32-key chunks, that the one-launch attention kernel handles
 *            (0: always split over the key axis; 1000000 and more: always the one-launch kernel, also
 *            where a batch would put more than two of its workgroups on a compute unit);
 *   wide=N   fewest rows for the many-row projection kernel (default 193; 97 for QKV), widemask=M which projections
 *            may use it (bit 0 QKV, 1 O, 2 gate/up, 3 down, 4 LM head);
 *   widecut=A:B:C:D:O   forces how that kernel cuts the rows of every launch whose rows make up exactly
 *            4A + 3B + 2C + D groups of 32 rows: A pieces of 128 rows, B of 96, C of 64, D of 32, launched
 *            weight group by weight group (O = 0) or all pieces of a size before any smaller one (O = 1).
 *   wideks=N   that kernel sums the contraction in N parts (1, 2 or 4; plain-sum projections only) instead of
 *            what its cost model or space_tune_rows picked.
 * Results do not depend on it beyond the order of floating-point sums; the tests use it to force every
 * kernel variant.  Malformed entries are ignored. */

/* Tuning call for callers that run blocks or prompt chunks of hundreds of rows (batches, prefill), where
 * the projections are bound by the matrix unit and what a launch costs is the work of its busiest
 * compute unit.  Measures, for every projection that uses the many-row kernel at `rows` rows (batch x
 * rows of the layout), a handful of ways to cut the rows into workgroups of 128, 96, 64 or 32 rows on the
 * context's own scratch buffers and the loaded layers' weights in turn -- and, for the projections whose
 * output is a plain sum (QKV, O, down), in how many parts the contraction is summed (1, 2 or 4) -- and
 * remembers the fastest for later space_step / space_prefill calls with that row count.  The cut of the rows
 * changes no result (every output element is computed by the same instructions in the same order); the
 * number of partial sums changes the order of the fp32 additions, i.e. results of a tuned context can
 * differ from an untuned one's in the last bits, as they do between any two tilings.  Unlike the other calls it waits for the
 * stream (a few tens of milliseconds) and must not be called on a stream that is being captured
 * (SPACE_EINVAL).  rows: 1..max_batch*max_rows, else SPACE_ESHAPE.  Row counts below the many-row kernel's
 * switch points and contexts without a loaded layer return SPACE_OK without doing anything. */
int space_tune_rows(space_ctx *ctx, int32_t rows, void *stream);

/* Measurement hook.  Kernel classes of a step, in launch order within a layer. */
typedef enum space_kernel_class {
    SPACE_K_EMBED = 0,   /* embedding gather + position ids + rotary table */
    SPACE_K_NORM = 1,    /* residual add + RMSNorm */
    SPACE_K_QKV = 2,     /* projection W_qkv */
    SPACE_K_ROPE = 3,    /* rotary + K/V store */
    SPACE_K_ATTN = 4,    /* masked block attention + merge of the key splits */
    SPACE_K_O = 5,       /* projection W_o */
    SPACE_K_GATE_UP = 6, /* projection W_gate, W_up + SwiGLU */
    SPACE_K_DOWN = 7,    /* projection W_down */
    SPACE_K_LM_HEAD = 8, /* LM head + per-workgroup argmax */
    SPACE_K_VERIFY = 9,  /* final argmax + acceptance scan + next block */
    SPACE_K_COUNT = 10
} space_kernel_class;

/* While a class bit (1u << class) is set in `class_mask`, every launch of that class inside
 * space_step is bracketed by a pair of HIP events on the step's stream; up to `max_records`
 * launches are kept between two reads.  class_mask == 0 switches timing off and frees the events.
 * What an empty bracket measures (median of nine, taken here) is subtracted from every record.
 * Synchronises the device.  Not for use under graph capture. */
int space_timing_enable(space_ctx *ctx, uint32_t class_mask, int32_t max_records);

/* Synchronises `stream`, adds up the recorded launches per class and clears the records.
 * total_ms and launches are HOST arrays of SPACE_K_COUNT entries. */
int space_timing_read(space_ctx *ctx, void *stream, double *total_ms, int64_t *launches);

/* Test hook: DEVICE address and size in bytes of one scratch buffer of ctx, as the last
 * space_step left it (with several layers: the last layer's contents).  Names:
 *   "x"        fp32 residual stream [rows, d_model];
 *   "xn", "attn_out", "h"  the operands of the projections (normalised rows; attention output,
 *              n_heads*head_dim columns; SwiGLU product, ffn columns) as split-bf16 planes in tile
 *              order: [column tiles of 32][row tiles of 16][hi, lo][64 lanes][8], lane l holding
 *              row l%16 and columns 8*(l/16)..+8 of the tile; the last row tile keeps only its c
 *              real rows, [hi, lo][4 column groups][c][8]; value = hi + lo;
 *   "q"        rotated queries, bf16 [hi, lo][max_batch][n_heads][L of the call][head_dim]
 *              (written only when the block has more than 48 rows);
 *   "pos"      int32 position id of every row.
 * SPACE_EINVAL for an unknown name.  The memory stays owned by ctx. */
int space_debug_buffer(space_ctx *ctx, const char *name, void **ptr, size_t *bytes);

#ifdef __cplusplus
}
#endif
#endif /* SPACE_H_ */

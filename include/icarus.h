/*
 * icarus.h -- C ABI of the ICaRus shared-KV layer step for MI355X (gfx950).
 *
 * One transformer layer of the paper's multi-model decode/prefill path: a frozen
 * logical encoder (the base weights) is the only writer of a paged KV cache
 * (Eq. 4); M task-specific logical decoders (the same base weights plus one LoRA
 * adapter each) only issue queries against that cache (Eq. 5).  At decode the
 * encoder row and the decoder rows of every sequence run side by side in one
 * batched pass (Sec. 3.3, Alg. 2 and Alg. 3).
 *
 * Conventions
 *  - Every call returns an icarus_status (0 = OK), never throws, never aborts;
 *    icarus_last_error() gives the message of the last failure on that context
 *    (or of the last failed icarus_create when ctx is NULL).
 *  - The CALLER owns all device memory (weights, KV pool, block tables,
 *    activations, workspace).  The library allocates no device memory, frees
 *    nothing of the caller's, and enqueues all work on the caller's stream
 *    without synchronising that stream.  Per-call metadata goes through a ring
 *    of 16 pinned HOST staging buffers per context: a buffer is allocated
 *    (hipHostMalloc) the first time its turn comes or when a call needs a
 *    larger one, and a call that finds its buffer still in use by the call
 *    made 16 calls earlier blocks the HOST until that call's metadata copy has
 *    run (back-pressure: at most 16 calls of one context are in flight).
 *    icarus_attn_shared_kv_static uses neither the ring nor a workspace.
 *  - "host" / "device" after a pointer says where the memory lives.
 *  - Small integer metadata (lengths, row lists) is passed as HOST arrays so it
 *    can be validated; block tables are DEVICE int32 [S, max_blocks].
 *  - dtype selects the storage type of weights, activations and cache:
 *    ICARUS_BF16 (2 bytes, arithmetic on bf16 MFMA with fp32 accumulation) or
 *    ICARUS_F32 (4 bytes, fp32 vector arithmetic).
 *  - Base weights W_p are [out_p, in_p] row-major.  LoRA A_p is
 *    [n_models, r, in_p], B_p is [n_models, out_p, r]; the adapter delta is
 *    lora_scale * B (A x) on the layer INPUT x (Alg. 2, read as standard LoRA).
 *    Adapters for K and V may be supplied but are never read: K and V come from
 *    the encoder row with base weights only (Alg. 3; App. C).
 *  - All pointers must be 16-byte aligned; head_dim must be even.
 *
 * KV pool layout (part of the ABI): element type = dtype,
 *     pool[num_blocks][n_kv_heads][2][block_size * head_dim]
 *   plane 0 holds K of the block as [block_size][head_dim] (token-major),
 *   plane 1 holds V of the block TRANSPOSED as [head_dim][block_size],
 * so that one (block, kv-head) is one contiguous run of 2*block_size*head_dim
 * elements and both planes load straight into matrix-core operand registers.
 * K is stored after RoPE (and after QK-RMSNorm when enabled).
 * Logical position p of sequence s lives in block block_table[s][p / block_size]
 * at in-block offset p % block_size; its "slot" is block * block_size + offset.
 */
#ifndef ICARUS_H
#define ICARUS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum icarus_status {
    ICARUS_OK = 0,
    ICARUS_ERR_INVALID_ARG = 1, /* null pointer, negative size, bad enum */
    ICARUS_ERR_SHAPE = 2,       /* config fields inconsistent (heads, dims, rank) */
    ICARUS_ERR_ALIGNMENT = 3,   /* a pointer is not 16-byte aligned */
    ICARUS_ERR_MODEL_ID = 4,    /* model id out of range or duplicated in a sequence */
    ICARUS_ERR_ROW_ORDER = 5,   /* rows not grouped by sequence / encoder row missing or not first */
    ICARUS_ERR_CAPACITY = 6,    /* block table, max_position or workspace too small */
    ICARUS_ERR_UNSUPPORTED = 7, /* shape outside what the kernels cover */
    ICARUS_ERR_HIP = 8          /* a HIP runtime call failed (message has the HIP error) */
} icarus_status;

enum { ICARUS_F32 = 0, ICARUS_BF16 = 1 };

/* Projection indices for the weight arrays and for lora_target_mask bits. */
enum { ICARUS_PROJ_Q = 0, ICARUS_PROJ_K, ICARUS_PROJ_V, ICARUS_PROJ_O,
       ICARUS_PROJ_GATE, ICARUS_PROJ_UP, ICARUS_PROJ_DOWN, ICARUS_NPROJ };

typedef struct icarus_layer_config {
    int32_t d_model, n_q_heads, n_kv_heads, head_dim, d_ffn;
    int32_t block_size;       /* tokens per KV block (16 in every benchmark config) */
    int32_t num_blocks;       /* blocks in the pool; block ids are 0..num_blocks-1 */
    int32_t n_models;         /* M: adapters loaded (0 = base model only) */
    int32_t lora_rank;        /* r */
    int32_t lora_target_mask; /* bit p set: projection p carries an adapter (K, V bits ignored) */
    int32_t dtype;            /* ICARUS_F32 or ICARUS_BF16 */
    int32_t qk_norm;          /* 1: per-head RMSNorm on q and k before RoPE */
    int32_t max_position;     /* largest position + 1 any call may touch */
    int32_t kv_dtype;         /* ICARUS_KV_SAME: cache elements have `dtype`; ICARUS_KV_FP8_E4M3: 1-byte codes */
    double rope_theta;        /* RoPE base; rotate-half pairing (i, i + head_dim/2) */
    double rms_eps;
    double lora_scale;        /* s = alpha / r */
    double k_scale, v_scale;  /* ICARUS_KV_FP8_E4M3 only, > 0: cached value = code * k_scale (K) or * v_scale (V) */
} icarus_layer_config;

/* Quantised shared cache (the paper names KV quantisation as orthogonal prior work, Sec. 1; the scheme is that of
 * the serving stacks it builds on: one static scale for all K and one for all V of a layer, calibrated by the
 * caller).  Codes are OCP FP8 E4M3 (bias 7, largest finite value 448, no infinities): on append
 * code = round-to-nearest-even(clamp(x / scale, -448, 448)); on read value = code * scale.  The pool has the same
 * shape with 1-byte elements: pool[num_blocks][n_kv_heads][2][block_size * head_dim] bytes.  K is quantised after
 * RoPE.  Activations and weights keep `dtype`. */
enum { ICARUS_KV_SAME = 0, ICARUS_KV_FP8_E4M3 = 1 };

typedef struct icarus_base_weights { /* all DEVICE, dtype elements */
    const void *w[ICARUS_NPROJ];       /* W_q [Hq*D, d], W_k, W_v [Hkv*D, d], W_o [d, Hq*D],
                                          W_gate, W_up [F, d], W_down [d, F] */
    const void *norm_attn, *norm_ffn;  /* [d] RMSNorm weights before attention / before the FFN */
    const void *q_norm, *k_norm;       /* [D], read only when qk_norm */
} icarus_base_weights;

typedef struct icarus_lora_weights { /* all DEVICE, dtype elements; NULL where not targeted */
    const void *A[ICARUS_NPROJ];       /* [n_models, r, in_p]  */
    const void *B[ICARUS_NPROJ];       /* [n_models, out_p, r] */
} icarus_lora_weights;

/* Decoders with private weights instead of adapters (Sec. 3.2: the logical decoder may as well be trained by
 * full fine-tuning or by an adapter that is merged into the weights, e.g. DoRA; at inference each such decoder
 * is a full matrix of its own per projection).  All DEVICE, dtype elements: w[p] = [n_models][out_p][in_p] for
 * p in {Q, O, GATE, UP, DOWN}; the K and V entries are ignored (K/V come from the encoder row with the base
 * weights, Alg. 3).  The arrays must outlive the context. */
typedef struct icarus_full_weights {
    const void *w[ICARUS_NPROJ];
} icarus_full_weights;

typedef struct icarus_ctx icarus_ctx;

/* Create a layer context: validates the configuration and keeps the (caller-owned)
 * weight pointers.  Host work only; no device is touched.  lora may be NULL when
 * n_models == 0.  On failure *out = NULL and icarus_last_error(NULL) has the reason. */
icarus_status icarus_create(const icarus_layer_config *cfg, const icarus_base_weights *base,
                            const icarus_lora_weights *lora, icarus_ctx **out);
void icarus_destroy(icarus_ctx *ctx);
const char *icarus_last_error(const icarus_ctx *ctx);

/* Device workspace, in bytes, sufficient for any call with at most max_rows rows
 * (decode: R; prefill: sum of chunk lengths), max_seqs sequences, and contexts of
 * at most max_ctx tokens (after the call's appends).  0 on invalid arguments. */
size_t icarus_workspace_bytes(const icarus_ctx *ctx, int32_t max_rows, int32_t max_seqs, int32_t max_ctx);

/* Host-only checks of a decode batch (what icarus_decode_step checks before it
 * launches anything): rows grouped by sequence in increasing sequence order, exactly
 * one encoder row (model -1) first in each group, decoder model ids in range and not
 * repeated within a sequence, every sequence's block table long enough for position
 * ctx_lens[s], positions below max_position. */
icarus_status icarus_validate_decode(icarus_ctx *ctx, int32_t max_blocks, int32_t S,
                                     const int32_t *ctx_lens /*host [S]*/, int32_t R,
                                     const int32_t *row_seq /*host [R]*/,
                                     const int32_t *row_model /*host [R]*/);

/* Host-only check of a HOST copy of the block tables (the device table itself is never read back): the
 * kernels index the pool with the ids they find in the table, so an id outside the pool is an out-of-bounds
 * device access.  For each sequence s the entries that a call with ctx_lens[s] cached tokens and extra[s] new
 * tokens touches -- the first ceil((ctx_lens[s] + extra[s]) / block_size) of its row -- must lie in
 * 0..num_blocks-1 (ICARUS_ERR_CAPACITY otherwise, also when the row is too short), and no block may receive the
 * new tokens of two different sequences (ICARUS_ERR_INVALID_ARG: the appends would overwrite each other; blocks
 * that are only read may be shared, as with a common cached prefix).  extra = NULL means one new token per
 * sequence (a decode step).  Meant for debugging and for callers that build tables from untrusted input; the
 * entry points themselves trust the device table (Alg. 1 / Alg. 3: the block table is the serving layer's).
 *   tables            host int32 [S, max_blocks], the same contents as the device table
 *   ctx_lens, extra   host int32 [S] */
icarus_status icarus_validate_block_tables(icarus_ctx *ctx, const int32_t *tables /*host*/, int32_t max_blocks,
                                           int32_t S, const int32_t *ctx_lens /*host*/,
                                           const int32_t *extra /*host or NULL*/);

/* Prefill of the logical encoder (Alg. 1; Sec. 3.3: prefill uses the encoder only).
 * Sequence s appends chunk_lens[s] new rows at positions ctx_lens[s] .. ctx_lens[s] +
 * chunk_lens[s] - 1 of its (possibly non-empty) paged prefix.  K (after RoPE) and V
 * of every new row are written to the pool with base weights only; the row at chunk
 * offset i attends to positions 0 .. ctx_lens[s] + i; then W_o, the residual and the
 * SwiGLU FFN give x_out.  Rows of x_in / x_out / slot_out are ordered by sequence,
 * then by chunk offset.
 *   kv_pool           device, mutated only at the new slots
 *   block_tables      device int32 [S, max_blocks]
 *   x_in              device [sum T, d_model]
 *   x_out             device [sum T, d_model], or NULL to write the cache only
 *   slot_out          device int64 [sum T] or NULL: slot written for each row
 *   workspace         device, >= icarus_workspace_bytes(ctx, sum T, S, max(ctx+chunk)) */
icarus_status icarus_prefill_kv(icarus_ctx *ctx, void *kv_pool, const int32_t *block_tables,
                                int32_t max_blocks, int32_t S, const int32_t *ctx_lens /*host*/,
                                const int32_t *chunk_lens /*host*/, const void *x_in, void *x_out,
                                int64_t *slot_out, void *workspace, size_t workspace_bytes,
                                void *stream /* hipStream_t */);

/* One decode step of one layer (Alg. 3 with ICaRusLinear, Alg. 2), one token per row.
 * Rows are grouped by sequence; the first row of a group is the logical encoder
 * (row_model -1), followed by that sequence's active decoders (row_model 0..M-1,
 * distinct; none is legal and gives a plain base-model step).  For sequence s, with
 * p = ctx_lens[s] tokens already cached: the encoder row's K, V (base weights) are
 * appended at position p; every row's query (base + its adapter) attends once to
 * positions 0..p of the shared cache; then W_o, residual, SwiGLU FFN, residual, each an
 * ICaRusLinear.  x_in is not modified.
 *   slot_out          device int64 [S] or NULL: slot written for each sequence      */
icarus_status icarus_decode_step(icarus_ctx *ctx, void *kv_pool, const int32_t *block_tables,
                                 int32_t max_blocks, int32_t S, const int32_t *ctx_lens /*host*/,
                                 int32_t R, const int32_t *row_seq /*host*/,
                                 const int32_t *row_model /*host*/, const void *x_in /*[R,d]*/,
                                 void *x_out /*[R,d]*/, int64_t *slot_out, void *workspace,
                                 size_t workspace_bytes, void *stream);

/* Shared-KV attention alone (the GQA line of Alg. 3; Sec. 3.3: the streams' queries are
 * concatenated on the head axis so that the cache is read once).  q [R, Hq, D] is
 * already normed and rotated; rows are grouped by sequence (any number >= 1 per
 * sequence, row_seq non-decreasing); kv_lens[s] INCLUDES the current token.  Head h of
 * every row uses kv-head h / (Hq/Hkv).  out [R, Hq, D] = softmax(q K^T / sqrt(D)) V. */
icarus_status icarus_attn_shared_kv(icarus_ctx *ctx, const void *q, const void *kv_pool,
                                    const int32_t *block_tables, int32_t max_blocks, int32_t S,
                                    const int32_t *kv_lens /*host*/, int32_t R,
                                    const int32_t *row_seq /*host*/, void *out, void *workspace,
                                    size_t workspace_bytes, void *stream);

/* The same attention for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  It takes no workspace and allocates nothing, on the device or pinned: what
 * icarus_attn_shared_kv keeps in the caller's workspace (row arrays, the attention plan, the partial results of
 * sequences cut into several pieces) lives in a 32 MiB array inside the library's code object, one copy per GPU,
 * held until the process ends; the per-call metadata reaches it as kernel arguments.  Same arguments, checks and
 * results as icarus_attn_shared_kv.  A call whose plan needs more than the array holds returns
 * ICARUS_ERR_CAPACITY (need = 16 R + 4 (plan ints) + pieces * n_kv_heads * largest stacked group * (head_dim + 2)
 * * 4 bytes; the benchmark decode batches need 10-16 MiB).  Every call on a GPU shares that GPU's array:
 * calls that may overlap on one GPU (different streams, different contexts) race and must be ordered by the
 * caller.  Nothing in the array has to start at zero: a call writes every entry it later reads. */
icarus_status icarus_attn_shared_kv_static(icarus_ctx *ctx, const void *q, const void *kv_pool,
                                           const int32_t *block_tables, int32_t max_blocks, int32_t S,
                                           const int32_t *kv_lens /*host*/, int32_t R,
                                           const int32_t *row_seq /*host*/, void *out, void *stream);

/* Kernel selection for tests and measurements: 0 = automatic (matrix-core kernels
 * where the shape allows, default), 1 = force the generic vector kernels. */
icarus_status icarus_set_kernel_mode(icarus_ctx *ctx, int32_t mode);

/* For tests and measurements: the longest piece, in tokens, that the decode attention's plan may give one
 * workgroup (rounded down to a multiple of 32, at least 32); 0 = automatic (default: up to 16384).  A small
 * limit cuts even short sequences into several pieces, which exercises the partial-result merge at sizes an
 * oracle finishes in seconds.  Changes the workspace a call needs: query icarus_workspace_bytes afterwards. */
icarus_status icarus_set_attn_piece_limit(icarus_ctx *ctx, int32_t tokens);

/* Per-phase kernel timing for measurements.  While enabled, every kernel launch of the entry
 * points above is bracketed by HIP events recorded on the caller's stream (this costs a few
 * microseconds per launch: leave it off when timing whole steps).  icarus_timing_read waits
 * for the recorded events, returns the accumulated milliseconds and launch counts per phase
 * (host arrays of ICARUS_NPHASE entries) and resets the accumulators. */
enum { ICARUS_PH_NORM = 0, ICARUS_PH_LORA, ICARUS_PH_GEMM_QKV, ICARUS_PH_ROPE_APPEND, ICARUS_PH_ATTN,
       ICARUS_PH_ATTN_MERGE, ICARUS_PH_GEMM_O, ICARUS_PH_GEMM_GATEUP, ICARUS_PH_GEMM_DOWN,
       ICARUS_PH_ELEMWISE, ICARUS_NPHASE };
icarus_status icarus_timing_enable(icarus_ctx *ctx, int32_t on);
icarus_status icarus_timing_read(icarus_ctx *ctx, double *ms /*host*/, int32_t *launches /*host*/);

/* Plain device-to-device copy of `bytes` bytes (a multiple of 16; src, dst device, 16-byte aligned) by a
 * grid-stride kernel named k_bench_copy.  For measurements only: a kernel that moves a known number of
 * bytes, against which the profiler's HBM traffic counters are calibrated. */
icarus_status icarus_bench_copy(const void *src, void *dst, size_t bytes, void *stream);

/* Streaming read of `bytes` bytes (a multiple of 8192; src device, 16-byte aligned) by kernel k_bench_read: every
 * wave reads whole 8 KB chunks -- the size of one (block, kv-head) of the cache -- with 16-byte loads, sixteen in
 * flight per lane, and stores nothing (out: one device word, written only if the fold of the data hits one value).
 * For measurements only: the read rate this GPU's HBM sustains, beside the published peak (use a buffer well
 * beyond the 256 MB memory-side cache). */
icarus_status icarus_bench_read(const void *src, size_t bytes, uint32_t *out, void *stream);

/* Register-resident matrix-core loop (kernel k_bench_mfma): `waves` wavefronts (a multiple of 4) each issue
 * `iters` rounds of 8 independent 32x32x16 bf16 MFMAs on operands that never leave the registers, then write
 * one float each to out (device, `waves` * 64 floats).  2 * 32*32*16 * 8 * iters * waves flops in all.  For
 * measurements only: the bf16 MFMA rate this GPU sustains, beside the published peak. */
icarus_status icarus_bench_mfma(float *out, int32_t waves, int32_t iters, void *stream);

/* Switch the context's decoders to private full weights (fw != NULL) or back to its LoRA adapters (NULL).
 * With private weights icarus_decode_step (and icarus_stack_decode) run every projection once per group of
 * rows -- the encoder rows with the base weights, the rows of model j with w[p][j] -- i.e. M + 1 grouped
 * GEMMs over row lists instead of one stacked GEMM: the weights are no longer shared, only the cache is.
 * Needs the matrix-core path (ICARUS_BF16 shapes it supports), n_models >= 1, 16-byte aligned arrays;
 * ICARUS_ERR_UNSUPPORTED otherwise.  Prefill is unaffected (encoder only). */
icarus_status icarus_set_full_decoders(icarus_ctx *ctx, const icarus_full_weights *fw);

/* ---- Layer stack: the outer loop of Alg. 3 and, for the prompt, Alg. 1 --------------------------------------
 * n_layers layer contexts of identical configuration, each with its own KV pool (all pools share the block
 * tables), a token embedding, the final RMSNorm and the LM head (base weights: shared by all streams).
 * A token step embeds each sequence's current token into all of its rows (the streams differ from layer 1
 * on), runs the rows through every layer, applies final norm + LM head to every row and takes the greedy
 * token (first index of the largest logit).  The prompt runs through the frozen encoder of every layer; the
 * first generated token comes from the base model (Alg. 1, y_prefill).
 * The stack borrows the layer contexts (they must outlive it and must not be used concurrently with it) and
 * the device arrays embed [vocab, d_model], final_norm [d_model], lm_head [vocab, d_model] (storage dtype). */
typedef struct icarus_stack icarus_stack;
typedef struct icarus_stack_config {
    int32_t n_layers;            /* >= 1 */
    int32_t vocab;               /* a multiple of 8 */
    icarus_ctx *const *layers;   /* host array [n_layers] */
    const void *embed, *final_norm, *lm_head; /* device */
} icarus_stack_config;

/* All layers must share one configuration; a row of d_model elements must hold at least 256 bytes
 * (ICARUS_ERR_UNSUPPORTED otherwise: the greedy token's partial results reuse a row buffer). */
icarus_status icarus_stack_create(const icarus_stack_config *cfg, icarus_stack **out);
void icarus_stack_destroy(icarus_stack *st);
const char *icarus_stack_last_error(const icarus_stack *st);
/* Workspace for calls of at most max_rows rows, max_seqs sequences, max_ctx context tokens, of which at most
 * max_logit_rows rows go through the LM head (decode: every row; prefill: one per sequence). */
size_t icarus_stack_workspace_bytes(const icarus_stack *st, int32_t max_rows, int32_t max_seqs, int32_t max_ctx,
                                    int32_t max_logit_rows);

/* Prompt chunks (Alg. 1): as icarus_prefill_kv on every layer, rows = embeddings of `tokens` (host, [sum of
 * chunk_lens]); kv_pools: host array of n_layers device pools.  next_token (device int32 [S]): greedy token
 * of the base model after each sequence's last chunk token; logits (device float [S, vocab]) optional. */
icarus_status icarus_stack_prefill(icarus_stack *st, void *const *kv_pools, const int32_t *block_tables, int32_t max_blocks,
                                   int32_t S, const int32_t *ctx_lens, const int32_t *chunk_lens, const int32_t *tokens,
                                   int32_t *next_token, float *logits, void *workspace, size_t workspace_bytes, void *stream);

/* One token step (Alg. 3): as icarus_decode_step on every layer.  seq_token (device int32 [S]): the token
 * each sequence decodes now.  row_next (device int32 [R]): greedy token of every row (an encoder row gives
 * the base model's); seq_next (device int32 [S], optional): row_next of each sequence's last row -- with one
 * decoder per sequence, the pair of the paper, the decoder's token; logits (device float [R, vocab]) optional.
 * seq_next may alias seq_token. */
icarus_status icarus_stack_decode(icarus_stack *st, void *const *kv_pools, const int32_t *block_tables, int32_t max_blocks,
                                  int32_t S, const int32_t *ctx_lens, int32_t R, const int32_t *row_seq,
                                  const int32_t *row_model, const int32_t *seq_token, int32_t *row_next, int32_t *seq_next,
                                  float *logits, void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ICARUS_H */

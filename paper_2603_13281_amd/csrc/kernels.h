// Internal launch interface between the C-ABI host layer and the gfx950 kernels.
// Every launcher enqueues on `st` and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace icarus {

typedef uint16_t bf16_raw;  // raw bfloat16 bits

struct Dims {
    int d, Hq, Hkv, D, F, Bk, M, r;
    int bf16;      // storage type: 1 = bfloat16, 0 = float32
    int kv8;       // 1: the KV pool holds FP8 E4M3 codes, value = code * k_scale (K plane) or v_scale (V plane)
    float k_scale, v_scale;
    int qk_norm;
    double theta;
    float eps, lora_scale;
};

// Per-call row metadata, device int32 arrays.
struct RowMeta {
    const int32_t *row_seq;    // [R] sequence of each row
    const int32_t *row_model;  // [R] -1 = logical encoder row, else adapter id
    const int32_t *row_pos;    // [R] position of the row's token
    const int32_t *row_kvlen;  // [R] cache positions the row attends to (0..kvlen-1)
};

// ---- generic vector kernels (any shape; fp32 accumulation) -------------------------------
// y[r,:] = x[r,:] * rsqrt(mean(x^2)+eps) * w        (storage type in and out)
hipError_t launch_rmsnorm(const Dims &dm, const void *x, const void *w, void *y, int R, int n, hipStream_t st);
// Y[m, n] (fp32, ld = ldy) = sum_k X[m,k] W[n,k];  X, W storage type
hipError_t launch_gemm_generic(const Dims &dm, const void *X, int ldx, const void *W, int M, int N, int K,
                               float *Y, int ldy, hipStream_t st);
// t[row, 0..r) (fp32) = lora_scale * A[model(row)] x[row]   for decoder rows (model >= 0)
hipError_t launch_lora_shrink_generic(const Dims &dm, const void *X, int ldx, const void *A, int K,
                                      const int32_t *row_model, float *t, int R, hipStream_t st);
// Y[row, n] += sum_k B[model(row)][n,k] t[row,k]           for decoder rows
hipError_t launch_lora_expand_generic(const Dims &dm, const float *t, const void *B, int N,
                                      const int32_t *row_model, float *Y, int ldy, int R, hipStream_t st);
// out[r, n] (storage) = resid[r, n] (storage) + acc[r, n] (fp32)
hipError_t launch_resid_store(const Dims &dm, const void *resid, const float *acc, void *out, int R, int n, hipStream_t st);
// h[r, n] (storage) = silu(gate[r,n]) * up[r,n]     (fp32 in)
hipError_t launch_silu_mul(const Dims &dm, const float *gate, const float *up, void *h, int R, int n, hipStream_t st);
// QK-RMSNorm (optional) + RoPE on q (all rows) and k (encoder rows), q -> q_out (storage, [R,Hq,D]),
// k, v of encoder rows -> paged cache; slot_out[slot_by_row ? row : seq] = slot.
// qkv: fp32 [R, ldq] with q at column 0, k at Hq*D, v at (Hq+Hkv)*D, given as `splits` slices that are
// summed (`slice` floats apart; splits = 1: the plain array).
hipError_t launch_rope_append(const Dims &dm, const float *qkv, int ldq, int splits, size_t slice, const RowMeta &rm,
                              const int32_t *bt, int max_blocks, void *pool, void *q_out, int64_t *slot_out, int slot_by_row,
                              const void *q_norm, const void *k_norm, int R, hipStream_t st, const int32_t *row_map = nullptr);
// out[row, h, :] = softmax(q[row,h,:] K^T / sqrt(D)) V over positions 0..row_kvlen[row]-1 of row_seq[row]
hipError_t launch_attn_generic(const Dims &dm, const void *q, const void *pool, const int32_t *bt, int max_blocks,
                               const RowMeta &rm, void *out, int R, hipStream_t st);

// plain grid-stride copy of `bytes` bytes (multiple of 16), kernel k_bench_copy: profiler calibration
hipError_t launch_bench_copy(const void *src, void *dst, size_t bytes, hipStream_t st);
// streaming read of `bytes` bytes (whole 8 KB chunks) by kernel k_bench_read: the read rate HBM sustains; out: one word
hipError_t launch_bench_read(const void *src, size_t bytes, uint32_t *out, hipStream_t st);
// register-resident MFMA loop, kernel k_bench_mfma: waves (multiple of 4) x iters x 8 MFMAs 32x32x16 bf16
hipError_t launch_bench_mfma(float *out, int waves, int iters, hipStream_t st);

// ---- matrix-core kernels (bf16 storage) ------------------------------------------------------
// Host-built plan of the attention kernels.  All arrays are device int32.
// Decode (causal = 0): the call's work -- the cached tokens of every sequence -- is laid on one line
// and cut into n_wgs equal shares; share b is walked by Hkv workgroups (one per kv-head), each over
// the pieces [wg_first[b], wg_first[b+1]), a piece being a token range of one sequence.  Piece
// boundaries are multiples of 32 tokens.  A sequence cut into several pieces leaves one partial
// result per piece and kv-head.
// Prefill (causal = 1): one piece per token group (x kv-heads in the launch), never split.
struct AttnPlan {
    const int32_t *item_seq;     // [n_items] plan sequence of the piece
    const int32_t *item_begin;   // [n_items] first token of the piece (decode)
    const int32_t *item_len;     // [n_items] tokens of the piece (decode)
    const int32_t *item_part;    // [n_items] partial-result slot of the piece (decode)
    const int32_t *item_direct;  // [n_items] 1: the piece is its whole sequence: write the final output (decode)
    const int32_t *wg_first;     // [n_wgs + 1] first piece of each share (decode)
    const int32_t *seq_kvlen;    // [S] tokens to attend to
    const int32_t *seq_row0;     // [S] first row of the sequence
    const int32_t *seq_rows;     // [S] rows (stacked streams) of the sequence
    const int32_t *seq_part0;    // [S] first partial slot (decode)
    const int32_t *seq_nparts;   // [S] number of pieces (decode)
    const int32_t *seq_bt;       // [S] row of the block table the sequence reads
    int n_items, n_wgs, chunk, g_max;  // n_wgs: shares; chunk: longest piece; g_max: largest stacked group (rows * Hq/Hkv)
    int causal;                  // 1: row t of a sequence attends to kv_len - (rows - 1 - t) tokens (prefill)
};
// ICaRusLinear GEMM on matrix cores.  Y = X W^T (+ T Bcat^T), see gemm_mfma.hip.
enum { GEMM_PLAIN = 0, GEMM_DUAL = 1 };          // DUAL: W[0] = gate, W[1] = up, Y = silu(gate) * up
enum { EPI_F32 = 0, EPI_BF16_RESID = 1 };        // plain epilogues (DUAL always stores bf16)
struct GemmArgs {
    const bf16_raw *X; int ldx; int R; int K;    // activations [R, K] (row stride ldx)
    const bf16_raw *W[3]; int n_seg[3]; int nseg; // weight segments stacked along N, each [n_seg, K]
    const bf16_raw *T; int ldt;                  // masked shrink result [R, ldt] or null
    const bf16_raw *B[2]; int r; int M_models;   // adapter B [M, n_seg[0], r] of segment 0 (DUAL: gate, up)
    int mode, epi;
    void *Y; int ldy;                            // EPI_F32: float [splits][R][ldy]; else bf16 [R][ldy]
    const bf16_raw *resid; int ldr;              // EPI_BF16_RESID: added to the result
    int splits;                                  // split-K slices (EPI_F32 without adapters only)
    int tile;                                    // tile kind, 0 = chosen by the launcher
    // filled by the launcher
    int tiles_seg[3]; int m_tiles, n_tiles, K_ext, k_per_split;
    int run, panel_m, panel_n, panels_m, n_panels;  // tile order: panels of panel_m x panel_n <= run tiles
    int slabs_per_split;                            // decode kernel: 64-wide K slabs per split-K slice
};
bool gemm_mfma_supported(const Dims &dm, int K);
hipError_t launch_gemm_mfma(GemmArgs g, hipStream_t st);
int gemm_mfma_tiles(const GemmArgs &g);  // workgroups of one K slice
int gemm_mfma_max_splits(const GemmArgs &g);  // most split-K slices worth launching (each keeps a pipeline's worth of K)
// The same contraction for decode-sized batches (gemm_decode.hip): both operands loaded coalesced, parked in registers
// two slabs ahead and staged through LDS by register stores; launch_gemm_mfma takes this path when gemm_uses_decode.
bool gemm_uses_decode(const GemmArgs &g);
bool gemm_decode_supported(const GemmArgs &g);
int gemm_decode_tiles(const GemmArgs &g);
int gemm_decode_slabs(const GemmArgs &g);
hipError_t launch_gemm_decode(GemmArgs g, hipStream_t st);
// Sum split-K partials P[splits][R][N] (fp32) and apply the epilogue `epi` into Y.
hipError_t launch_splitk_reduce(const float *P, int splits, int R, int N, int epi, void *Y, int ldy, const void *resid,
                                int ldr, hipStream_t st);
// Row-wise kernels (bf16 storage).  T [R, targets*M*r] (bf16) is the masked LoRA shrink the GEMM reads
// as extra K columns: T[row, t*M*r + j*r + i] = lora_scale * (A_t[j] x_row)_i for j = row_model[row], zero
// in every other column (encoder rows: all zero).  A: [M][r][K].
bool row_shrink_supported(int r, int targets);
// y = rmsnorm(x) * wn for R rows of K, and (A0 != null) the shrink of y for one or two targets that
// share y; also sets zero[0..n_zero) = 0.
hipError_t launch_norm_shrink(const Dims &dm, const void *x, const void *wn, void *y, int R, int K, const void *A0, const void *A1,
                              const int32_t *row_model, void *T, int *zero, int n_zero, hipStream_t st);
// the same on rows that are still in pieces: xsum = resid + sum of `splits` fp32 slices [R, K] (`slice` floats
// apart, the split-K partials of the projection before the norm) is formed, rounded, stored, and normalised
hipError_t launch_sum_norm_shrink(const Dims &dm, const float *part, int splits, size_t slice, const void *resid, void *xsum,
                                  const void *wn, void *y, int R, int K, const void *A0, const void *A1, const int32_t *row_model,
                                  void *T, hipStream_t st);
// the shrink alone, of x [R, K] (row stride ldx)
hipError_t launch_row_shrink(const Dims &dm, const void *x, int ldx, int R, int K, const void *A0, const int32_t *row_model, void *T,
                             hipStream_t st);

bool attn_decode_mfma_supported(const Dims &dm, int g_max);
// Merge of the attention partials of cut sequences (as launch_attn_merge) and, with A0, the shrink of the O projection
// on the merged rows, in one kernel: attn [R][Hq*D] is completed in place, T as for launch_row_shrink.
hipError_t launch_merge_shrink(const Dims &dm, const float *part_o, const float *part_ml, const struct AttnPlan &pl,
                               const int32_t *row_pseq, void *attn, int R, const void *A0, const int32_t *row_model, void *T,
                               hipStream_t st);
// Causal attention of prefill chunks: each plan sequence is a group of consecutive chunk tokens with at
// most attn_prefill_group_queries() stacked queries (tokens x Hq/Hkv); never split, writes `out` directly.
int attn_prefill_group_queries();
bool attn_prefill_mfma_supported(const Dims &dm, int g_max);
hipError_t launch_attn_prefill_mfma(const Dims &dm, const void *q, const void *pool, const int32_t *bt, int max_blocks,
                                    const AttnPlan &pl, void *out, hipStream_t st);
// part_o: fp32 [slots, Hkv, g_max, D]; part_ml: fp32 [slots, Hkv, g_max, 2] (max in log2 units, sum)
hipError_t launch_attn_decode_mfma(const Dims &dm, const void *q, const void *pool, const int32_t *bt, int max_blocks,
                                   const AttnPlan &pl, void *out, float *part_o, float *part_ml, hipStream_t st);
hipError_t launch_attn_merge(const Dims &dm, const float *part_o, const float *part_ml, const AttnPlan &pl,
                             const int32_t *row_seq, void *out, int R, hipStream_t st);

// ---- layer stack helpers (index work) ----------------------------------------------------------
// x[row, :] = embed[tok[idx ? idx[row] : row], :]   (rows of row_bytes bytes, a multiple of 16)
hipError_t launch_embed_rows(const void *embed, const int32_t *tok, const int32_t *idx, void *x, int R, int row_bytes, hipStream_t st);
// out[i, :] = x[rows[i], :]
hipError_t launch_gather_rows(const void *x, const int32_t *rows, void *out, int n, int row_bytes, hipStream_t st);
// token[row] = first index of the largest of logits[row, 0..V)
// scratch: argmax_scratch_bytes(R) bytes of device memory, 8-byte aligned (partial results)
size_t argmax_scratch_bytes(int R);
hipError_t launch_argmax(const float *logits, int R, int V, int32_t *token, void *scratch, hipStream_t st);
// seq_next[s] = row_next[last_row[s]]
hipError_t launch_pick_rows(const int32_t *row_next, const int32_t *last_row, int32_t *seq_next, int S, hipStream_t st);

}  // namespace icarus

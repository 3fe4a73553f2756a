// Host side of the C ABI: context, validation, per-call metadata staging, workspace
// layout and the launch sequence of one layer step.  No arithmetic of the method
// happens here; every step runs in the kernels.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/icarus.h"
#include "kernels.h"

using namespace icarus;

// ---- device scratch of the entry point that allocates nothing ------------------------------------------
// icarus_attn_shared_kv_static keeps what icarus_attn_shared_kv keeps in the caller's workspace -- row arrays,
// the attention plan, the partial results of cut sequences -- in this array.  Every GPU the library runs on holds
// its own copy until the process ends.  In host code the array's name is only a stand-in: the address that
// kernels and copies take is the one hipGetSymbolAddress returns for the current device (static_scratch()).
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Per-call metadata of that entry point travels to the device as kernel arguments (no pinned host buffer to
// allocate, nothing for the host to wait on): kStageInts ints per launch.
constexpr int kStageInts = 960;
struct StageChunk { int32_t v[kStageInts]; };
__global__ void __launch_bounds__(256) k_stage_ints(StageChunk c, int32_t *__restrict__ dst, int n) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = c.v[i];
}

namespace {

constexpr int kSlots = 16;  // pinned staging ring depth
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {nullptr};  // device address of `scratch` on each GPU, once looked up
std::mutex g_scratch_mu;

struct StageSlot {
    void *host = nullptr;
    size_t cap = 0;
    hipEvent_t ev = nullptr;
    bool in_flight = false;
};

char g_create_err[512] = "";

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

struct PhaseTimer {
    bool on = false;
    struct Span { int phase; hipEvent_t a, b; };
    std::vector<Span> pending;
    std::vector<hipEvent_t> pool;
    double ms[ICARUS_NPHASE] = {0};
    int32_t launches[ICARUS_NPHASE] = {0};
    hipEvent_t get() {
        if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        (void)hipEventCreate(&e);
        return e;
    }
};

struct icarus_ctx {
    icarus_layer_config cfg;
    icarus_base_weights base;
    icarus_lora_weights lora;
    Dims dm;
    icarus_full_weights full{};   // private decoder weights (full_set), instead of the adapters
    bool full_set = false;
    int mode = 0;
    int attn_chunk_override = 0;  // longest attention piece in tokens; 0 = automatic (icarus_set_attn_piece_limit)
    int attn_wgs = 256;           // workgroups of the decode attention: Hkv per equal share of the work
    // cost model of the decode attention plan, from per-workgroup timings: a cached token costs
    // attn_weight_base + attn_weight_tile * (16-query tiles of its sequence), a piece as much as
    // attn_piece_tokens tokens on top
    int attn_weight_base = 128, attn_weight_tile = 7, attn_piece_tokens = 768;
    char err[512];
    StageSlot slots[kSlots];
    int next_slot = 0;
    PhaseTimer timer;
    std::mutex mu;
};

struct icarus_stack {
    std::vector<icarus_ctx *> layers;
    int vocab = 0;
    const void *embed = nullptr, *final_norm = nullptr, *lm_head = nullptr;
    char err[512];
    std::mutex mu;
};

namespace {

icarus_status fail(icarus_ctx *ctx, icarus_status st, const char *fmt, ...) {
    char *dst = ctx ? ctx->err : g_create_err;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 512, fmt, ap);
    va_end(ap);
    return st;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int proj_in(const icarus_layer_config &c, int p) {
    switch (p) {
    case ICARUS_PROJ_O: return c.n_q_heads * c.head_dim;
    case ICARUS_PROJ_DOWN: return c.d_ffn;
    default: return c.d_model;
    }
}
int proj_out(const icarus_layer_config &c, int p) {
    switch (p) {
    case ICARUS_PROJ_Q: return c.n_q_heads * c.head_dim;
    case ICARUS_PROJ_K: case ICARUS_PROJ_V: return c.n_kv_heads * c.head_dim;
    case ICARUS_PROJ_GATE: case ICARUS_PROJ_UP: return c.d_ffn;
    default: return c.d_model;
    }
}

bool has_lora(const icarus_ctx *ctx, int p) {
    if (p == ICARUS_PROJ_K || p == ICARUS_PROJ_V) return false;  // the decoder writes no KV: never read
    return ctx->cfg.n_models > 0 && ctx->cfg.lora_rank > 0 && ((ctx->cfg.lora_target_mask >> p) & 1);
}

// ---- workspace layout ---------------------------------------------------------------
struct WsLayout {
    size_t meta, xn, qkv, q, attn, z, h, f32a, f32b, t, part_o, part_ml, lora_t, xg, ag, yg, total;
    size_t meta_ints, max_items, gemm_part, gemm_part_bytes;
};

// Rows regrouped for decoders with private weights: group 0 = encoder rows, group 1 + j = rows of model j.
struct FullPlan {
    const int32_t *perm = nullptr;  // device [R]: grouped position -> row of the call
    const int32_t *inv = nullptr;   // device [R]: row of the call -> grouped position
    std::vector<int32_t> off;       // host [n_models + 2]: first grouped position of each group
};

constexpr int kAttnTargetWgs = 1280;  // decode attention: sizing bound for pieces and partial results
constexpr int kAttnMaxChunk = 16384;  // tokens per attention chunk, at most (block ids of a chunk sit in LDS)
constexpr int kAttnGMax = 80;         // largest stacked query group the MFMA attention covers
constexpr int kGemmMaxSplits = 12;    // split-K slices of a narrow ICaRusLinear GEMM

// Upper bounds used for sizing: chunks (= partial slots) of a call and its largest stacked group.
size_t attn_max_items(const icarus_ctx *ctx, size_t seqs, size_t max_ctx) {
    // pieces of the decode plan: one per share, one more per sequence, and the cuts forced by the
    // longest allowed piece
    size_t cap = ctx->attn_chunk_override > 0 ? (size_t)std::max(32, ctx->attn_chunk_override / 32 * 32) : (size_t)kAttnMaxChunk;
    return std::max<size_t>(4 * kAttnTargetWgs / ctx->cfg.n_kv_heads, (size_t)ctx->attn_wgs) + seqs * (2 + max_ctx / cap) + 1;
}

WsLayout ws_layout(const icarus_ctx *ctx, size_t rows, size_t seqs, size_t max_ctx) {
    const icarus_layer_config &c = ctx->cfg;
    size_t es = c.dtype == ICARUS_BF16 ? 2 : 4;
    size_t qd = (size_t)c.n_q_heads * c.head_dim, kvd = (size_t)c.n_kv_heads * c.head_dim;
    WsLayout w{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    w.max_items = attn_max_items(ctx, seqs, max_ctx);
    // metadata: 4 row arrays and the attention plan (5 arrays per piece, the shares' first pieces, 6 arrays
    // per plan sequence); a prefill call has up to `rows` plan sequences of one piece each
    w.meta_ints = 4 * rows + 5 * std::max(rows, w.max_items) + (size_t)ctx->attn_wgs + 6 * std::max(rows, seqs) + 64 +
                  rows + seqs +  // + what a layer stack stages with the call: prompt tokens, last row of each sequence
                  2 * rows;      // + the regrouping of rows for decoders with private weights
    w.meta = take(w.meta_ints * 4);
    {
        size_t g = (size_t)c.n_q_heads / c.n_kv_heads;
        size_t g_bound = std::min<size_t>(kAttnGMax, rows * g);
        size_t pj = w.max_items * c.n_kv_heads * g_bound;
        w.part_o = take(pj * c.head_dim * 4);
        w.part_ml = take(pj * 2 * 4);
    }
    w.xn = take(rows * c.d_model * es);
    w.qkv = take(rows * (qd + 2 * kvd) * 4);
    w.q = take(rows * qd * es);
    w.attn = take(rows * qd * es);
    w.z = take(rows * c.d_model * es);
    w.h = take(rows * c.d_ffn * es);
    w.f32a = take(rows * std::max<size_t>(c.d_ffn, c.d_model) * 4);
    w.f32b = take(rows * c.d_ffn * 4);
    w.t = take(rows * std::max(1, c.lora_rank) * 4 * 2);
    w.lora_t = take(rows * 2 * std::max(1, c.n_models) * std::max(1, c.lora_rank) * 2);  // gate + up share a shrink
    // split-K partials of a narrow GEMM: only calls of a few hundred rows are split
    w.gemm_part_bytes = (size_t)kGemmMaxSplits * std::min<size_t>(rows, 512) * std::max(qd + 2 * kvd, (size_t)c.d_model) * 4;
    w.gemm_part = take(w.gemm_part_bytes);
    // rows regrouped by model (decoders with private weights): input, attention output, layer output
    w.xg = take(rows * c.d_model * es);
    w.ag = take(rows * qd * es);
    w.yg = take(rows * c.d_model * es);
    w.total = off;
    return w;
}

// ---- pinned staging of per-call metadata -----------------------------------------------
// Returns a host buffer of at least `bytes`; the caller fills it, then calls stage_commit to
// enqueue the copy to the device and mark the slot busy until that copy has run.
icarus_status stage_acquire(icarus_ctx *ctx, size_t bytes, StageSlot **out) {
    StageSlot &s = ctx->slots[ctx->next_slot];
    ctx->next_slot = (ctx->next_slot + 1) % kSlots;
    hipError_t e;
    if (s.in_flight) {
        e = hipEventSynchronize(s.ev);
        if (e != hipSuccess) return fail(ctx, ICARUS_ERR_HIP, "hipEventSynchronize: %s", hipGetErrorString(e));
        s.in_flight = false;
    }
    if (!s.ev) {
        e = hipEventCreateWithFlags(&s.ev, hipEventDisableTiming);
        if (e != hipSuccess) return fail(ctx, ICARUS_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(e));
    }
    if (s.cap < bytes) {
        if (s.host) (void)hipHostFree(s.host);
        s.host = nullptr;
        s.cap = 0;
        size_t cap = align_up(std::max<size_t>(bytes, 1 << 16), 4096);
        e = hipHostMalloc(&s.host, cap, hipHostMallocDefault);
        if (e != hipSuccess) return fail(ctx, ICARUS_ERR_HIP, "hipHostMalloc(%zu): %s", cap, hipGetErrorString(e));
        s.cap = cap;
    }
    *out = &s;
    return ICARUS_OK;
}

icarus_status stage_commit(icarus_ctx *ctx, StageSlot *s, void *dev, size_t bytes, hipStream_t st) {
    hipError_t e = hipMemcpyAsync(dev, s->host, bytes, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) return fail(ctx, ICARUS_ERR_HIP, "hipMemcpyAsync(meta): %s", hipGetErrorString(e));
    e = hipEventRecord(s->ev, st);
    if (e != hipSuccess) return fail(ctx, ICARUS_ERR_HIP, "hipEventRecord: %s", hipGetErrorString(e));
    s->in_flight = true;
    return ICARUS_OK;
}

#define HIP_TRY(ctx, expr)                                                                         \
    do {                                                                                           \
        hipError_t e__ = (expr);                                                                   \
        if (e__ != hipSuccess) return fail(ctx, ICARUS_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e__)); \
    } while (0)

// Device address of the static scratch array on the current GPU (looked up once per device).
icarus_status static_scratch(icarus_ctx *ctx, char **out) {
    int dev = -1;
    HIP_TRY(ctx, hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(ctx, ICARUS_ERR_UNSUPPORTED, "device %d: at most %d devices", dev, kMaxDevices);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIP_TRY(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(ctx, ICARUS_ERR_HIP, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = p;
    }
    *out = (char *)g_scratch_ptr[dev];
    return ICARUS_OK;
}

// Copy n host ints to device memory through kernel arguments.
icarus_status stage_by_kernarg(icarus_ctx *ctx, const int32_t *src, size_t n, int32_t *dst, hipStream_t st) {
    for (size_t at = 0; at < n; at += kStageInts) {
        StageChunk c;
        const int k = (int)std::min<size_t>(kStageInts, n - at);
        memcpy(c.v, src + at, (size_t)k * 4);
        hipLaunchKernelGGL(k_stage_ints, dim3((k + 255) / 256), dim3(256), 0, st, c, dst + at, k);
        HIP_TRY(ctx, hipGetLastError());
    }
    return ICARUS_OK;
}

// Run one launch; with phase timing on, bracket it with events on the launch stream.
#define PHASE(ctx, st, phase, expr)                                                 \
    do {                                                                            \
        PhaseTimer &tm__ = (ctx)->timer;                                            \
        hipEvent_t a__ = nullptr, b__ = nullptr;                                    \
        if (tm__.on) { a__ = tm__.get(); b__ = tm__.get(); (void)hipEventRecord(a__, st); } \
        HIP_TRY(ctx, expr);                                                         \
        if (tm__.on) { (void)hipEventRecord(b__, st); tm__.pending.push_back({phase, a__, b__}); } \
    } while (0)

// ---- validation ----------------------------------------------------------------------
icarus_status check_decode_rows(icarus_ctx *ctx, int32_t max_blocks, int32_t S, const int32_t *ctx_lens, int32_t R,
                                const int32_t *row_seq, const int32_t *row_model) {
    const icarus_layer_config &c = ctx->cfg;
    if (S < 0 || R < 0 || max_blocks < 0) return fail(ctx, ICARUS_ERR_INVALID_ARG, "negative size");
    if (S == 0 && R == 0) return ICARUS_OK;
    if (!ctx_lens || !row_seq || !row_model) return fail(ctx, ICARUS_ERR_INVALID_ARG, "null metadata array");
    if (R > 65535) return fail(ctx, ICARUS_ERR_UNSUPPORTED, "at most 65535 rows per call (got %d)", R);
    int r = 0;
    std::vector<char> seen((size_t)std::max(1, c.n_models));
    for (int s = 0; s < S; ++s) {
        if (ctx_lens[s] < 0) return fail(ctx, ICARUS_ERR_INVALID_ARG, "ctx_lens[%d] = %d is negative", s, ctx_lens[s]);
        if (ctx_lens[s] + 1 > c.max_position)
            return fail(ctx, ICARUS_ERR_CAPACITY, "sequence %d: position %d >= max_position %d", s, ctx_lens[s], c.max_position);
        if ((int64_t)ctx_lens[s] / c.block_size + 1 > max_blocks)
            return fail(ctx, ICARUS_ERR_CAPACITY, "sequence %d: position %d needs %d blocks, table has %d", s, ctx_lens[s],
                        ctx_lens[s] / c.block_size + 1, max_blocks);
        if (r >= R || row_seq[r] != s)
            return fail(ctx, ICARUS_ERR_ROW_ORDER, "sequence %d has no rows at row %d (rows must be grouped by sequence, in order)", s, r);
        if (row_model[r] != -1)
            return fail(ctx, ICARUS_ERR_ROW_ORDER, "row %d: the first row of sequence %d must be the encoder row (model -1)", r, s);
        ++r;
        std::fill(seen.begin(), seen.end(), 0);
        while (r < R && row_seq[r] == s) {
            int j = row_model[r];
            if (j == -1) return fail(ctx, ICARUS_ERR_ROW_ORDER, "row %d: second encoder row in sequence %d", r, s);
            if (j < 0 || j >= c.n_models) return fail(ctx, ICARUS_ERR_MODEL_ID, "row %d: model id %d outside 0..%d", r, j, c.n_models - 1);
            if (seen[j]) return fail(ctx, ICARUS_ERR_MODEL_ID, "row %d: model id %d repeated in sequence %d", r, j, s);
            seen[j] = 1;
            ++r;
        }
    }
    if (r != R) {
        if (row_seq[r] < 0 || row_seq[r] >= S) return fail(ctx, ICARUS_ERR_INVALID_ARG, "row %d: sequence id %d outside 0..%d", r, row_seq[r], S - 1);
        return fail(ctx, ICARUS_ERR_ROW_ORDER, "row %d: sequence %d appears out of order", r, row_seq[r]);
    }
    return ICARUS_OK;
}

icarus_status check_common_ptrs(icarus_ctx *ctx, const void *pool, const void *bt, const void *ws, size_t ws_bytes, size_t need) {
    if (!pool || !bt) return fail(ctx, ICARUS_ERR_INVALID_ARG, "kv_pool / block_tables is null");
    if (!ws) return fail(ctx, ICARUS_ERR_INVALID_ARG, "workspace is null");
    if (!aligned16(pool) || !aligned16(bt) || !aligned16(ws)) return fail(ctx, ICARUS_ERR_ALIGNMENT, "kv_pool, block_tables and workspace must be 16-byte aligned");
    if (ws_bytes < need) return fail(ctx, ICARUS_ERR_CAPACITY, "workspace has %zu bytes, this call needs %zu", ws_bytes, need);
    return ICARUS_OK;
}

// ---- decode-attention split plan --------------------------------------------------------
// Builds the attention plan of a call into the host staging buffer `m` starting at int offset `at`;
// `dmeta` is the device address the buffer will be copied to.  seq_row0 / seq_rows: rows of each
// plan sequence.  hp->valid stays false if the matrix-core attention does not cover this call (then
// the generic kernel runs).
struct HostPlan {
    AttnPlan pl;
    bool valid = false, has_split = false;
    size_t ints = 0;
};

// Decode: the cached tokens of all sequences are laid on one line (weighted by a per-token cost that
// grows mildly with the stacked group) and cut into equal shares, one per group of Hkv workgroups
// (a workgroup per kv-head), so that every workgroup finishes at about the same time whatever the
// mix of context lengths; pieces are multiples of 32 tokens and at most kAttnMaxChunk long.
// Prefill (causal): seq_bt gives the block-table row of each plan sequence (a group of consecutive
// chunk tokens; row t attends to kv_len - (rows-1-t) tokens); never split, so the call is covered
// only if every kv_len fits one piece.
void build_attn_plan(const icarus_ctx *ctx, int32_t *m, size_t at, const int32_t *dmeta, int S, const int32_t *kv_lens,
                     const int32_t *seq_row0, const int32_t *seq_rows, const int32_t *seq_bt, bool causal, size_t max_items,
                     HostPlan *hp) {
    AttnPlan *pl = &hp->pl;
    *pl = AttnPlan{};
    hp->valid = false;
    hp->has_split = false;
    hp->ints = 0;
    const icarus_layer_config &c = ctx->cfg;
    if (ctx->mode != 0) return;
    const int g = c.n_q_heads / c.n_kv_heads, Hkv = c.n_kv_heads;
    int g_max = 0;
    for (int s = 0; s < S; ++s) {
        if (seq_rows[s] > 0 && kv_lens[s] <= 0) return;  // empty context: generic kernel writes zeros
        if (causal && kv_lens[s] > kAttnMaxChunk) return;
        g_max = std::max(g_max, seq_rows[s] * g);
    }
    if (causal ? !attn_prefill_mfma_supported(ctx->dm, g_max) : (!attn_decode_mfma_supported(ctx->dm, g_max) || g_max > kAttnGMax)) return;
    const int32_t *d = dmeta + at;
    if (causal) {
        // One piece per token group (x kv-heads in the launch).  The launch maps kv-head c of piece i to workgroup
        // i * Hkv + c, so with Hkv = 8 every XCD runs one kv-head and takes the pieces in this order, about 32 at a
        // time: the token groups of one sequence are kept next to each other, so that they walk the sequence's
        // cached prefix at the same time and all but the first find it in that XCD's L2 (sorted by length alone,
        // the groups of a sequence were rounds apart and each one fetched the prefix from HBM again).  Sequences
        // with the longest contexts go first, and within a sequence the longest group.
        std::vector<int32_t> order;
        int n_bt = 0;
        for (int s = 0; s < S; ++s) {
            if (seq_rows[s] > 0) order.push_back(s);
            n_bt = std::max(n_bt, (seq_bt ? seq_bt[s] : s) + 1);
        }
        std::vector<int32_t> longest((size_t)n_bt, 0);  // per block-table row (= sequence of the call)
        for (int s : order) {
            int32_t &l = longest[seq_bt ? seq_bt[s] : s];
            l = std::max(l, kv_lens[s]);
        }
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
            const int ra = seq_bt ? seq_bt[a] : a, rb = seq_bt ? seq_bt[b] : b;
            if (longest[ra] != longest[rb]) return longest[ra] > longest[rb];
            if (ra != rb) return ra < rb;
            return kv_lens[a] > kv_lens[b];
        });
        const size_t n_items = order.size();
        int32_t *item_seq = m + at, *seq_kvlen = item_seq + n_items, *row0 = seq_kvlen + S, *rows = row0 + S, *sbt = rows + S;
        for (size_t i = 0; i < n_items; ++i) item_seq[i] = order[i];
        for (int s = 0; s < S; ++s) {
            seq_kvlen[s] = kv_lens[s];
            row0[s] = seq_row0[s];
            rows[s] = seq_rows[s];
            sbt[s] = seq_bt ? seq_bt[s] : s;
        }
        pl->item_seq = d;
        pl->seq_kvlen = d + n_items;
        pl->seq_row0 = pl->seq_kvlen + S;
        pl->seq_rows = pl->seq_row0 + S;
        pl->seq_bt = pl->seq_rows + S;
        pl->n_items = (int)n_items;
        pl->chunk = kAttnMaxChunk;
        pl->g_max = g_max;
        pl->causal = 1;
        hp->ints = n_items + 4 * (size_t)S;
        hp->valid = n_items > 0;
        return;
    }
    // ---- decode: equal shares of the weighted work line
    auto weight = [&](int s) {  // cost of one cached token
        return (int64_t)(ctx->attn_weight_base + ctx->attn_weight_tile * ((seq_rows[s] * g + 15) / 16));
    };
    auto piece_cost = [&](int s) { return (int64_t)ctx->attn_piece_tokens * weight(s); };  // fixed cost of starting a piece
    int64_t total = 0, tokens = 0;
    for (int s = 0; s < S; ++s)
        if (seq_rows[s] > 0) {
            total += (int64_t)kv_lens[s] * weight(s) + piece_cost(s);
            tokens += kv_lens[s];
        }
    if (tokens == 0) return;
    const int cap = ctx->attn_chunk_override > 0 ? std::max(32, ctx->attn_chunk_override / 32 * 32) : kAttnMaxChunk;  // longest piece
    const int max_wgs = (int)std::max<int64_t>(1, std::min<int64_t>(std::max(1, ctx->attn_wgs / Hkv), tokens / 256));
    struct Piece { int32_t s, begin, len, wg; };
    std::vector<Piece> pieces;
    // Shares are filled in order up to a target cost T (tokens x weight + a fixed cost per piece); a share closes when
    // what is left of its target would not pay for another piece.  T is the smallest target with which max_wgs shares
    // take everything (bisection: the fill is monotone in T), so that no share, the last included, exceeds it.
    const int min_piece = std::max(64, ctx->attn_piece_tokens);  // a shorter piece is not worth its fixed cost
    auto fill = [&](int64_t T, bool emit) {
        int wg = 0;
        int64_t room = T;
        for (int s = 0; s < S; ++s) {
            if (seq_rows[s] <= 0) continue;
            const int64_t wt = weight(s), pc = piece_cost(s);
            int begin = 0;
            while (begin < kv_lens[s]) {
                const int left = kv_lens[s] - begin;
                if (room < pc + (int64_t)std::min(left, min_piece) * wt && room < T) {  // a fresh share always takes something
                    ++wg;
                    room = T;
                }
                int64_t fit = std::max<int64_t>(room - pc, 0) / wt;
                int len = (int)std::min<int64_t>({(int64_t)left, (int64_t)cap, std::max<int64_t>(32, fit / 32 * 32)});
                if (len < left) len = std::max(32, len / 32 * 32);  // inner boundaries on whole 32-token groups
                if (emit) pieces.push_back({s, begin, len, wg});
                begin += len;
                room -= pc + (int64_t)len * wt;
            }
        }
        return wg + 1;
    };
    int64_t lo = total / max_wgs, hi = 2 * total + 1;  // fill(hi) is a single share (cuts forced by the longest piece cost far less than total)
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (fill(mid, false) <= max_wgs) hi = mid; else lo = mid + 1;
    }
    int n_wgs = fill(lo, true);
    const size_t n_items = pieces.size();
    if (n_items > max_items) return;
    int32_t *item_seq = m + at, *item_begin = item_seq + n_items, *item_len = item_begin + n_items,
            *item_part = item_len + n_items, *item_direct = item_part + n_items, *wg_first = item_direct + n_items,
            *seq_kvlen = wg_first + n_wgs + 1, *row0 = seq_kvlen + S, *rows = row0 + S, *sbt = rows + S, *part0 = sbt + S,
            *nparts = part0 + S;
    for (int s = 0; s < S; ++s) {
        seq_kvlen[s] = kv_lens[s];
        row0[s] = seq_row0[s];
        rows[s] = seq_rows[s];
        sbt[s] = seq_bt ? seq_bt[s] : s;
        part0[s] = 0;
        nparts[s] = 0;
    }
    int max_len = 0;
    for (size_t i = 0; i < n_items; ++i) {  // pieces of one sequence are consecutive
        const Piece &e = pieces[i];
        if (nparts[e.s] == 0) part0[e.s] = (int32_t)i;
        ++nparts[e.s];
        item_seq[i] = e.s;
        item_begin[i] = e.begin;
        item_len[i] = e.len;
        item_part[i] = (int32_t)i;
        max_len = std::max(max_len, (int)e.len);
    }
    for (size_t i = 0; i < n_items; ++i) {
        item_direct[i] = nparts[pieces[i].s] == 1;
        if (nparts[pieces[i].s] > 1) hp->has_split = true;
    }
    {   // first piece of each share (pieces are in share order)
        size_t i = 0;
        for (int b = 0; b <= n_wgs; ++b) {
            while (i < n_items && pieces[i].wg < b) ++i;
            wg_first[b] = (int32_t)i;
        }
    }
    pl->item_seq = d;
    pl->item_begin = d + n_items;
    pl->item_len = d + 2 * n_items;
    pl->item_part = d + 3 * n_items;
    pl->item_direct = d + 4 * n_items;
    pl->wg_first = d + 5 * n_items;
    pl->seq_kvlen = pl->wg_first + n_wgs + 1;
    pl->seq_row0 = pl->seq_kvlen + S;
    pl->seq_rows = pl->seq_row0 + S;
    pl->seq_bt = pl->seq_rows + S;
    pl->seq_part0 = pl->seq_bt + S;
    pl->seq_nparts = pl->seq_part0 + S;
    pl->n_items = (int)n_items;
    pl->n_wgs = n_wgs;
    pl->chunk = max_len;
    pl->g_max = g_max;
    pl->causal = 0;
    hp->ints = 5 * n_items + (size_t)n_wgs + 1 + 6 * (size_t)S;
    hp->valid = n_items > 0;
}

// Attention of decode rows: matrix-core kernel + merge when a plan exists, else the generic kernel.
icarus_status run_decode_attention(icarus_ctx *ctx, char *ws, const WsLayout &L, const RowMeta &rm, const HostPlan *hp,
                                   const void *q, const void *pool, const int32_t *bt, int max_blocks, void *out, int R,
                                   hipStream_t st, bool *merge_left = nullptr) {
    if (merge_left) *merge_left = false;
    if (!hp || !hp->valid) {
        PHASE(ctx, st, ICARUS_PH_ATTN, launch_attn_generic(ctx->dm, q, pool, bt, max_blocks, rm, out, R, st));
        return ICARUS_OK;
    }
    if (hp->pl.causal) {
        PHASE(ctx, st, ICARUS_PH_ATTN, launch_attn_prefill_mfma(ctx->dm, q, pool, bt, max_blocks, hp->pl, out, st));
        return ICARUS_OK;
    }
    float *part_o = (float *)(ws + L.part_o), *part_ml = (float *)(ws + L.part_ml);
    PHASE(ctx, st, ICARUS_PH_ATTN, launch_attn_decode_mfma(ctx->dm, q, pool, bt, max_blocks, hp->pl, out, part_o, part_ml, st));
    if (hp->has_split && merge_left) {  // the caller merges the partials in its next row kernel
        *merge_left = true;
        return ICARUS_OK;
    }
    if (hp->has_split) PHASE(ctx, st, ICARUS_PH_ATTN_MERGE, launch_attn_merge(ctx->dm, part_o, part_ml, hp->pl, rm.row_seq, out, R, st));
    return ICARUS_OK;
}

#define LORA_TRY(call) do { icarus_status rc__ = (call); if (rc__) return rc__; } while (0)

// ---- the layer on matrix cores (bf16 storage) -----------------------------------------
bool layer_mfma_supported(const icarus_ctx *ctx) {
    const icarus_layer_config &c = ctx->cfg;
    bool shrink_ok = c.n_models == 0 || c.lora_rank == 0 || row_shrink_supported(c.lora_rank, 2);
    return ctx->mode == 0 && gemm_mfma_supported(ctx->dm, c.d_model) && gemm_mfma_supported(ctx->dm, c.n_q_heads * c.head_dim) &&
           gemm_mfma_supported(ctx->dm, c.d_ffn) && shrink_ok;
}

// One plain ICaRusLinear GEMM.  When its grid would leave most of the chip idle (few rows and a
// narrow output), K is split over several workgroups into fp32 partials [splits][R][N]; a second
// small kernel sums them and applies the epilogue, unless the caller takes the slices as they are
// (deferred_splits: set to the number of slices left in the workspace, 0 if the output is final).
icarus_status run_gemm(icarus_ctx *ctx, char *ws, const WsLayout &L, int phase, GemmArgs g, hipStream_t st,
                       int *deferred_splits = nullptr) {
    int tiles = gemm_mfma_tiles(g);
    int n_total = 0;
    for (int s = 0; s < g.nseg; ++s) n_total += g.n_seg[s];
    int splits = 1;
    if (tiles < 160) splits = std::max(1, std::min({kGemmMaxSplits, 256 / tiles, gemm_mfma_max_splits(g)}));
    splits = (int)std::max<size_t>(1, std::min<size_t>(splits, L.gemm_part_bytes / ((size_t)g.R * n_total * 4)));
    if (deferred_splits) *deferred_splits = 0;
    if (splits == 1) {
        g.splits = 1;
        PHASE(ctx, st, phase, launch_gemm_mfma(g, st));
        return ICARUS_OK;
    }
    GemmArgs p = g;
    p.epi = EPI_F32; p.Y = ws + L.gemm_part; p.ldy = n_total; p.splits = splits;
    PHASE(ctx, st, phase, launch_gemm_mfma(p, st));
    if (deferred_splits && n_total == g.ldy) {  // the consumer sums the slices [splits][R][n_total] itself
        *deferred_splits = splits;
        return ICARUS_OK;
    }
    PHASE(ctx, st, phase, launch_splitk_reduce((const float *)(ws + L.gemm_part), splits, g.R, n_total, g.epi, g.Y, g.ldy, g.resid,
                                               g.ldr, st));
    return ICARUS_OK;
}

icarus_status run_layer_mfma(icarus_ctx *ctx, char *ws, const WsLayout &L, const RowMeta &rm, const HostPlan *hp, int R,
                             bool use_lora, bool kv_only, int slot_by_row, void *pool, const int32_t *bt, int max_blocks,
                             const void *x_in, void *x_out, int64_t *slot_out, hipStream_t st, int in_splits = 0,
                             int *out_splits = nullptr) {
    // in_splits > 0 (layer stack): the input rows are still in pieces -- the previous layer's down projection left
    // `in_splits` split-K slices in the workspace and its residual in z -- and are formed (and stored to x_in) by
    // this layer's first row kernel.  out_splits != null: this layer may leave its own output the same way.
    const icarus_layer_config &c = ctx->cfg;
    const Dims &dm = ctx->dm;
    int d = c.d_model, qd = c.n_q_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim, F = c.d_ffn;
    int ldq = qd + 2 * kvd, mr = c.n_models * c.lora_rank;
    bf16_raw *xn = (bf16_raw *)(ws + L.xn), *q = (bf16_raw *)(ws + L.q), *attn = (bf16_raw *)(ws + L.attn),
             *z = (bf16_raw *)(ws + L.z), *h = (bf16_raw *)(ws + L.h), *T = (bf16_raw *)(ws + L.lora_t);
    float *qkv = (float *)(ws + L.qkv);
    auto W = [&](int p) { return (const bf16_raw *)ctx->base.w[p]; };
    auto lo = [&](int p) { return use_lora && has_lora(ctx, p); };
    auto Bw = [&](int p) { return (const bf16_raw *)ctx->lora.B[p]; };

    auto Aw = [&](int p) { return ctx->lora.A[p]; };
    const bool lq = !kv_only && lo(ICARUS_PROJ_Q);
    // RMSNorm, with the shrink of the Q adapters on the normalised rows
    if (in_splits > 0) {
        PHASE(ctx, st, ICARUS_PH_NORM, launch_sum_norm_shrink(dm, (const float *)(ws + L.gemm_part), in_splits, (size_t)R * d, z,
                                                              const_cast<void *>(x_in), ctx->base.norm_attn, xn, R, d,
                                                              lq ? Aw(ICARUS_PROJ_Q) : nullptr, nullptr, rm.row_model, T, st));
    } else {
        PHASE(ctx, st, ICARUS_PH_NORM, launch_norm_shrink(dm, x_in, ctx->base.norm_attn, xn, R, d, lq ? Aw(ICARUS_PROJ_Q) : nullptr,
                                                          nullptr, rm.row_model, T, nullptr, 0, st));
    }
    int qkv_splits = 0, o_splits = 0;
    {   // Q (ICaRusLinear) and the encoder's K, V in one GEMM over [W_q; W_k; W_v]
        GemmArgs g{};
        g.X = xn; g.ldx = d; g.R = R; g.K = d;
        g.mode = GEMM_PLAIN; g.epi = EPI_F32; g.splits = 1; g.r = c.lora_rank; g.M_models = c.n_models;
        if (kv_only) {
            g.W[0] = W(ICARUS_PROJ_K); g.n_seg[0] = kvd; g.W[1] = W(ICARUS_PROJ_V); g.n_seg[1] = kvd; g.nseg = 2;
            g.Y = qkv + qd; g.ldy = ldq;
        } else {
            if (lq) { g.T = T; g.ldt = mr; g.B[0] = Bw(ICARUS_PROJ_Q); }
            g.W[0] = W(ICARUS_PROJ_Q); g.n_seg[0] = qd; g.W[1] = W(ICARUS_PROJ_K); g.n_seg[1] = kvd;
            g.W[2] = W(ICARUS_PROJ_V); g.n_seg[2] = kvd; g.nseg = 3;
            g.Y = qkv; g.ldy = ldq;
        }
        LORA_TRY(run_gemm(ctx, ws, L, ICARUS_PH_GEMM_QKV, g, st, &qkv_splits));
    }
    {   // split-K slices of the projection, if any were left, are summed by the RoPE kernel
        const float *src = qkv_splits ? (const float *)(ws + L.gemm_part) : qkv;
        PHASE(ctx, st, ICARUS_PH_ROPE_APPEND, launch_rope_append(dm, src, ldq, std::max(1, qkv_splits), (size_t)R * ldq, rm, bt, max_blocks,
                                                                 pool, q, slot_out, slot_by_row, ctx->base.q_norm, ctx->base.k_norm, R, st));
    }
    if (kv_only) return ICARUS_OK;
    bool merge_left = false;
    LORA_TRY(run_decode_attention(ctx, ws, L, rm, hp, q, pool, bt, max_blocks, attn, R, st, &merge_left));
    {   // O projection (ICaRusLinear) + residual; its shrink also merges the attention partials of cut sequences
        GemmArgs g{};
        g.X = attn; g.ldx = qd; g.R = R; g.K = qd;
        g.W[0] = W(ICARUS_PROJ_O); g.n_seg[0] = d; g.nseg = 1;
        g.mode = GEMM_PLAIN; g.epi = EPI_BF16_RESID; g.splits = 1; g.r = c.lora_rank; g.M_models = c.n_models;
        const bool l_o = lo(ICARUS_PROJ_O);
        if (merge_left)
            PHASE(ctx, st, ICARUS_PH_ATTN_MERGE,
                  launch_merge_shrink(dm, (const float *)(ws + L.part_o), (const float *)(ws + L.part_ml), hp->pl, rm.row_seq, attn, R,
                                      l_o ? Aw(ICARUS_PROJ_O) : nullptr, rm.row_model, T, st));
        else if (l_o)
            PHASE(ctx, st, ICARUS_PH_LORA, launch_row_shrink(dm, attn, qd, R, qd, Aw(ICARUS_PROJ_O), rm.row_model, T, st));
        if (l_o) { g.T = T; g.ldt = mr; g.B[0] = Bw(ICARUS_PROJ_O); }
        g.Y = z; g.ldy = d; g.resid = (const bf16_raw *)x_in; g.ldr = d;
        LORA_TRY(run_gemm(ctx, ws, L, ICARUS_PH_GEMM_O, g, st, &o_splits));
    }
    const bool lg = lo(ICARUS_PROJ_GATE), lu = lo(ICARUS_PROJ_UP);
    if (lg != lu) return fail(ctx, ICARUS_ERR_UNSUPPORTED, "adapters on only one of gate/up need the generic kernels (set kernel mode 1)");
    // RMSNorm with the shrink of the gate/up adapters; if the O projection left split-K slices, the
    // same kernel first forms z = x + their sum
    if (o_splits)
        PHASE(ctx, st, ICARUS_PH_NORM, launch_sum_norm_shrink(dm, (const float *)(ws + L.gemm_part), o_splits, (size_t)R * d, x_in, z,
                                                              ctx->base.norm_ffn, xn, R, d, lg ? Aw(ICARUS_PROJ_GATE) : nullptr,
                                                              lg ? Aw(ICARUS_PROJ_UP) : nullptr, rm.row_model, T, st));
    else
        PHASE(ctx, st, ICARUS_PH_NORM, launch_norm_shrink(dm, z, ctx->base.norm_ffn, xn, R, d, lg ? Aw(ICARUS_PROJ_GATE) : nullptr,
                                                          lg ? Aw(ICARUS_PROJ_UP) : nullptr, rm.row_model, T, nullptr, 0, st));
    {   // gate and up (ICaRusLinear x 2) with the SwiGLU product in the epilogue
        GemmArgs g{};
        g.X = xn; g.ldx = d; g.R = R; g.K = d;
        g.W[0] = W(ICARUS_PROJ_GATE); g.W[1] = W(ICARUS_PROJ_UP); g.n_seg[0] = F; g.nseg = 1;
        g.mode = GEMM_DUAL; g.splits = 1; g.r = c.lora_rank; g.M_models = c.n_models;
        if (lg) { g.T = T; g.ldt = 2 * mr; g.B[0] = Bw(ICARUS_PROJ_GATE); g.B[1] = Bw(ICARUS_PROJ_UP); }
        g.Y = h; g.ldy = F;
        PHASE(ctx, st, ICARUS_PH_GEMM_GATEUP, launch_gemm_mfma(g, st));
    }
    {   // down projection (ICaRusLinear) + residual
        GemmArgs g{};
        g.X = h; g.ldx = F; g.R = R; g.K = F;
        g.W[0] = W(ICARUS_PROJ_DOWN); g.n_seg[0] = d; g.nseg = 1;
        g.mode = GEMM_PLAIN; g.epi = EPI_BF16_RESID; g.splits = 1; g.r = c.lora_rank; g.M_models = c.n_models;
        if (lo(ICARUS_PROJ_DOWN)) {
            PHASE(ctx, st, ICARUS_PH_LORA, launch_row_shrink(dm, h, F, R, F, Aw(ICARUS_PROJ_DOWN), rm.row_model, T, st));
            g.T = T; g.ldt = mr; g.B[0] = Bw(ICARUS_PROJ_DOWN);
        }
        g.Y = x_out; g.ldy = d; g.resid = z; g.ldr = d;
        LORA_TRY(run_gemm(ctx, ws, L, ICARUS_PH_GEMM_DOWN, g, st, out_splits));
    }
    return ICARUS_OK;
}

// ---- decode step with private decoder weights -----------------------------------------
// The rows are regrouped (encoder rows, then the rows of model 0, 1, ...) for everything but attention, and every
// projection runs once per group with that group's weights; q is written back in call order by the RoPE kernel
// (row map), the attention output is regrouped by a gather, the result returned to call order by another.
icarus_status run_layer_full(icarus_ctx *ctx, char *ws, const WsLayout &L, const RowMeta &rm, const HostPlan *hp, const FullPlan &fp,
                             int R, int slot_by_row, void *pool, const int32_t *bt, int max_blocks, const void *x_in, void *x_out,
                             int64_t *slot_out, hipStream_t st) {
    const icarus_layer_config &c = ctx->cfg;
    const Dims &dm = ctx->dm;
    if (!fp.perm || fp.off.size() != (size_t)c.n_models + 2) return fail(ctx, ICARUS_ERR_UNSUPPORTED, "rows were not regrouped for private decoder weights");
    const int d = c.d_model, qd = c.n_q_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim, F = c.d_ffn;
    const int ldq = qd + 2 * kvd;
    bf16_raw *xn = (bf16_raw *)(ws + L.xn), *q = (bf16_raw *)(ws + L.q), *attn = (bf16_raw *)(ws + L.attn),
             *z = (bf16_raw *)(ws + L.z), *h = (bf16_raw *)(ws + L.h);
    bf16_raw *xg = (bf16_raw *)(ws + L.xg), *ag = (bf16_raw *)(ws + L.ag), *yg = (bf16_raw *)(ws + L.yg);
    float *qkv = (float *)(ws + L.qkv);
    auto Wg = [&](int p, int grp) {  // weight of projection p for group grp
        if (grp == 0) return (const bf16_raw *)ctx->base.w[p];
        return (const bf16_raw *)ctx->full.w[p] + (size_t)(grp - 1) * proj_out(c, p) * proj_in(c, p);
    };
    const int n_groups = c.n_models + 1;
    PHASE(ctx, st, ICARUS_PH_ELEMWISE, launch_gather_rows(x_in, fp.perm, xg, R, d * 2, st));
    PHASE(ctx, st, ICARUS_PH_NORM, launch_norm_shrink(dm, xg, ctx->base.norm_attn, xn, R, d, nullptr, nullptr, nullptr, nullptr, nullptr, 0, st));
    for (int grp = 0; grp < n_groups; ++grp) {  // Q per group; K, V of the encoder rows
        const int o0 = fp.off[grp], n = fp.off[grp + 1] - o0;
        if (n <= 0) continue;
        GemmArgs g{};
        g.X = xn + (size_t)o0 * d; g.ldx = d; g.R = n; g.K = d;
        g.mode = GEMM_PLAIN; g.epi = EPI_F32; g.splits = 1;
        g.W[0] = Wg(ICARUS_PROJ_Q, grp); g.n_seg[0] = qd; g.nseg = 1;
        if (grp == 0) { g.W[1] = Wg(ICARUS_PROJ_K, 0); g.n_seg[1] = kvd; g.W[2] = Wg(ICARUS_PROJ_V, 0); g.n_seg[2] = kvd; g.nseg = 3; }
        g.Y = qkv + (size_t)o0 * ldq; g.ldy = ldq;
        LORA_TRY(run_gemm(ctx, ws, L, ICARUS_PH_GEMM_QKV, g, st));
    }
    PHASE(ctx, st, ICARUS_PH_ROPE_APPEND, launch_rope_append(dm, qkv, ldq, 1, 0, rm, bt, max_blocks, pool, q, slot_out, slot_by_row,
                                                             ctx->base.q_norm, ctx->base.k_norm, R, st, fp.perm));
    LORA_TRY(run_decode_attention(ctx, ws, L, rm, hp, q, pool, bt, max_blocks, attn, R, st));
    PHASE(ctx, st, ICARUS_PH_ELEMWISE, launch_gather_rows(attn, fp.perm, ag, R, qd * 2, st));
    for (int grp = 0; grp < n_groups; ++grp) {  // O projection + residual
        const int o0 = fp.off[grp], n = fp.off[grp + 1] - o0;
        if (n <= 0) continue;
        GemmArgs g{};
        g.X = ag + (size_t)o0 * qd; g.ldx = qd; g.R = n; g.K = qd;
        g.W[0] = Wg(ICARUS_PROJ_O, grp); g.n_seg[0] = d; g.nseg = 1;
        g.mode = GEMM_PLAIN; g.epi = EPI_BF16_RESID; g.splits = 1;
        g.Y = z + (size_t)o0 * d; g.ldy = d; g.resid = xg + (size_t)o0 * d; g.ldr = d;
        LORA_TRY(run_gemm(ctx, ws, L, ICARUS_PH_GEMM_O, g, st));
    }
    PHASE(ctx, st, ICARUS_PH_NORM, launch_norm_shrink(dm, z, ctx->base.norm_ffn, xn, R, d, nullptr, nullptr, nullptr, nullptr, nullptr, 0, st));
    for (int grp = 0; grp < n_groups; ++grp) {  // gate, up, SwiGLU
        const int o0 = fp.off[grp], n = fp.off[grp + 1] - o0;
        if (n <= 0) continue;
        GemmArgs g{};
        g.X = xn + (size_t)o0 * d; g.ldx = d; g.R = n; g.K = d;
        g.W[0] = Wg(ICARUS_PROJ_GATE, grp); g.W[1] = Wg(ICARUS_PROJ_UP, grp); g.n_seg[0] = F; g.nseg = 1;
        g.mode = GEMM_DUAL; g.splits = 1;
        g.Y = h + (size_t)o0 * F; g.ldy = F;
        PHASE(ctx, st, ICARUS_PH_GEMM_GATEUP, launch_gemm_mfma(g, st));
    }
    for (int grp = 0; grp < n_groups; ++grp) {  // down projection + residual
        const int o0 = fp.off[grp], n = fp.off[grp + 1] - o0;
        if (n <= 0) continue;
        GemmArgs g{};
        g.X = h + (size_t)o0 * F; g.ldx = F; g.R = n; g.K = F;
        g.W[0] = Wg(ICARUS_PROJ_DOWN, grp); g.n_seg[0] = d; g.nseg = 1;
        g.mode = GEMM_PLAIN; g.epi = EPI_BF16_RESID; g.splits = 1;
        g.Y = yg + (size_t)o0 * d; g.ldy = d; g.resid = z + (size_t)o0 * d; g.ldr = d;
        LORA_TRY(run_gemm(ctx, ws, L, ICARUS_PH_GEMM_DOWN, g, st));
    }
    PHASE(ctx, st, ICARUS_PH_ELEMWISE, launch_gather_rows(yg, fp.inv, x_out, R, d * 2, st));
    return ICARUS_OK;
}

// Whether run_layer would take rows that are still in pieces (split-K slices + residual) as its input: only the
// matrix-core path forms its rows in its first row kernel.
bool layer_takes_slices(icarus_ctx *ctx, bool use_lora) {
    if (use_lora && ctx->full_set) return false;
    if (!layer_mfma_supported(ctx)) return false;
    return (use_lora && has_lora(ctx, ICARUS_PROJ_GATE)) == (use_lora && has_lora(ctx, ICARUS_PROJ_UP));
}

// ---- the layer, after metadata is on the device ---------------------------------------
// rows: x_in [R, d].  use_lora: decoder rows get adapter deltas.  kv_only: stop after the append.
icarus_status run_layer(icarus_ctx *ctx, char *ws, const WsLayout &L, const RowMeta &rm, const HostPlan *hp, int R, bool use_lora, bool kv_only,
                        int slot_by_row, void *pool, const int32_t *bt, int max_blocks, const void *x_in, void *x_out,
                        int64_t *slot_out, hipStream_t st, const FullPlan *fp = nullptr, int in_splits = 0, int *out_splits = nullptr) {
    if (out_splits) *out_splits = 0;
    if (use_lora && !kv_only && ctx->full_set) {  // decoder rows with private weights
        if (!fp || !layer_mfma_supported(ctx)) return fail(ctx, ICARUS_ERR_UNSUPPORTED, "private decoder weights need the matrix-core path");
        return run_layer_full(ctx, ws, L, rm, hp, *fp, R, slot_by_row, pool, bt, max_blocks, x_in, x_out, slot_out, st);
    }
    if (layer_mfma_supported(ctx)) {
        bool lg = use_lora && has_lora(ctx, ICARUS_PROJ_GATE), lu = use_lora && has_lora(ctx, ICARUS_PROJ_UP);
        if (lg == lu)
            return run_layer_mfma(ctx, ws, L, rm, hp, R, use_lora, kv_only, slot_by_row, pool, bt, max_blocks, x_in, x_out, slot_out, st,
                                  in_splits, out_splits);
    }
    if (in_splits > 0) return fail(ctx, ICARUS_ERR_UNSUPPORTED, "input rows in pieces need the matrix-core path");
    const icarus_layer_config &c = ctx->cfg;
    const Dims &dm = ctx->dm;
    int d = c.d_model, qd = c.n_q_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim, F = c.d_ffn;
    int ldq = qd + 2 * kvd;
    void *xn = ws + L.xn, *q = ws + L.q, *attn = ws + L.attn, *z = ws + L.z, *h = ws + L.h;
    float *qkv = (float *)(ws + L.qkv), *fa = (float *)(ws + L.f32a), *fb = (float *)(ws + L.f32b), *t = (float *)(ws + L.t);
    auto lora = [&](int p, const void *X, int ldx, float *Y, int ldy) -> icarus_status {
        if (!use_lora || !has_lora(ctx, p)) return ICARUS_OK;
        PHASE(ctx, st, ICARUS_PH_LORA, launch_lora_shrink_generic(dm, X, ldx, ctx->lora.A[p], proj_in(c, p), rm.row_model, t, R, st));
        PHASE(ctx, st, ICARUS_PH_LORA, launch_lora_expand_generic(dm, t, ctx->lora.B[p], proj_out(c, p), rm.row_model, Y, ldy, R, st));
        return ICARUS_OK;
    };
    PHASE(ctx, st, ICARUS_PH_NORM, launch_rmsnorm(dm, x_in, ctx->base.norm_attn, xn, R, d, st));
    if (!kv_only) {
        PHASE(ctx, st, ICARUS_PH_GEMM_QKV, launch_gemm_generic(dm, xn, d, ctx->base.w[ICARUS_PROJ_Q], R, qd, d, qkv, ldq, st));
        LORA_TRY(lora(ICARUS_PROJ_Q, xn, d, qkv, ldq));
    }
    PHASE(ctx, st, ICARUS_PH_GEMM_QKV, launch_gemm_generic(dm, xn, d, ctx->base.w[ICARUS_PROJ_K], R, kvd, d, qkv + qd, ldq, st));
    PHASE(ctx, st, ICARUS_PH_GEMM_QKV, launch_gemm_generic(dm, xn, d, ctx->base.w[ICARUS_PROJ_V], R, kvd, d, qkv + qd + kvd, ldq, st));
    PHASE(ctx, st, ICARUS_PH_ROPE_APPEND, launch_rope_append(dm, qkv, ldq, 1, 0, rm, bt, max_blocks, pool, q, slot_out, slot_by_row,
                                                             ctx->base.q_norm, ctx->base.k_norm, R, st));
    if (kv_only) return ICARUS_OK;
    LORA_TRY(run_decode_attention(ctx, ws, L, rm, hp, q, pool, bt, max_blocks, attn, R, st));
    PHASE(ctx, st, ICARUS_PH_GEMM_O, launch_gemm_generic(dm, attn, qd, ctx->base.w[ICARUS_PROJ_O], R, d, qd, fa, d, st));
    LORA_TRY(lora(ICARUS_PROJ_O, attn, qd, fa, d));
    PHASE(ctx, st, ICARUS_PH_ELEMWISE, launch_resid_store(dm, x_in, fa, z, R, d, st));
    PHASE(ctx, st, ICARUS_PH_NORM, launch_rmsnorm(dm, z, ctx->base.norm_ffn, xn, R, d, st));
    PHASE(ctx, st, ICARUS_PH_GEMM_GATEUP, launch_gemm_generic(dm, xn, d, ctx->base.w[ICARUS_PROJ_GATE], R, F, d, fa, F, st));
    LORA_TRY(lora(ICARUS_PROJ_GATE, xn, d, fa, F));
    PHASE(ctx, st, ICARUS_PH_GEMM_GATEUP, launch_gemm_generic(dm, xn, d, ctx->base.w[ICARUS_PROJ_UP], R, F, d, fb, F, st));
    LORA_TRY(lora(ICARUS_PROJ_UP, xn, d, fb, F));
    PHASE(ctx, st, ICARUS_PH_ELEMWISE, launch_silu_mul(dm, fa, fb, h, R, F, st));
    PHASE(ctx, st, ICARUS_PH_GEMM_DOWN, launch_gemm_generic(dm, h, F, ctx->base.w[ICARUS_PROJ_DOWN], R, d, F, fa, d, st));
    LORA_TRY(lora(ICARUS_PROJ_DOWN, h, F, fa, d));
    PHASE(ctx, st, ICARUS_PH_ELEMWISE, launch_resid_store(dm, z, fa, x_out, R, d, st));
    return ICARUS_OK;
}

// What a call needs once its host metadata is validated, laid out and on its way to the device:
// workspace layout, row arrays, attention plan; `extra` (optional caller ints staged with the same
// copy) lands at extra_dev.
struct Prepared {
    WsLayout L;
    RowMeta rm;
    HostPlan hp;
    FullPlan fp;
    const int32_t *extra_dev = nullptr;
};

icarus_status prepare_decode(icarus_ctx *ctx, const void *kv_pool, const int32_t *block_tables, int32_t max_blocks, int32_t S,
                             const int32_t *ctx_lens, int32_t R, const int32_t *row_seq, const int32_t *row_model, void *workspace,
                             size_t workspace_bytes, hipStream_t st, const int32_t *extra, size_t n_extra, Prepared *pr) {
    int max_ctx = 0;
    for (int s = 0; s < S; ++s) max_ctx = std::max(max_ctx, ctx_lens[s] + 1);
    pr->L = ws_layout(ctx, (size_t)R, (size_t)S, (size_t)max_ctx);
    const WsLayout &L = pr->L;
    icarus_status rc = check_common_ptrs(ctx, kv_pool, block_tables, workspace, workspace_bytes, L.total);
    if (rc) return rc;
    StageSlot *slot;
    rc = stage_acquire(ctx, L.meta_ints * 4, &slot);
    if (rc) return rc;
    int32_t *m = (int32_t *)slot->host;
    std::vector<int32_t> kvl((size_t)S), row0((size_t)S, 0), rows((size_t)S, 0);
    for (int r = 0; r < R; ++r) {
        int s = row_seq[r];
        m[r] = s;
        m[R + r] = row_model[r];
        m[2 * R + r] = ctx_lens[s];
        m[3 * R + r] = ctx_lens[s] + 1;
        if (rows[s]++ == 0) row0[s] = r;
    }
    for (int s = 0; s < S; ++s) kvl[s] = ctx_lens[s] + 1;
    char *ws = (char *)workspace;
    const int32_t *dmeta = (const int32_t *)(ws + L.meta);
    build_attn_plan(ctx, m, (size_t)4 * R, dmeta, S, kvl.data(), row0.data(), rows.data(), nullptr, false, L.max_items, &pr->hp);
    size_t used = (size_t)4 * R + pr->hp.ints;
    if (n_extra) {
        memcpy(m + used, extra, n_extra * 4);
        pr->extra_dev = dmeta + used;
        used += n_extra;
    }
    if (ctx->full_set) {  // counting sort of the rows by group
        const int n_groups = ctx->cfg.n_models + 1;
        std::vector<int32_t> &off = pr->fp.off;
        off.assign((size_t)n_groups + 1, 0);
        for (int r = 0; r < R; ++r) ++off[(size_t)row_model[r] + 2];
        for (int g = 1; g <= n_groups; ++g) off[g] += off[g - 1];
        std::vector<int32_t> next(off.begin(), off.end() - 1);
        int32_t *perm = m + used, *inv = perm + R;
        for (int r = 0; r < R; ++r) {
            int pos = next[(size_t)row_model[r] + 1]++;
            perm[pos] = r;
            inv[r] = pos;
        }
        pr->fp.perm = dmeta + used;
        pr->fp.inv = dmeta + used + R;
        used += (size_t)2 * R;
    }
    rc = stage_commit(ctx, slot, ws + L.meta, used * 4, st);
    if (rc) return rc;
    pr->rm = RowMeta{dmeta, dmeta + R, dmeta + 2 * R, dmeta + 3 * R};
    return ICARUS_OK;
}

// Validates a prefill call's host metadata; *rows = total chunk tokens.
icarus_status check_prefill(icarus_ctx *ctx, int32_t max_blocks, int32_t S, const int32_t *ctx_lens, const int32_t *chunk_lens, int *rows) {
    const icarus_layer_config &c = ctx->cfg;
    *rows = 0;
    if (S < 0 || max_blocks < 0) return fail(ctx, ICARUS_ERR_INVALID_ARG, "negative size");
    if (S == 0) return ICARUS_OK;
    if (!ctx_lens || !chunk_lens) return fail(ctx, ICARUS_ERR_INVALID_ARG, "null metadata array");
    int64_t total = 0;
    for (int s = 0; s < S; ++s) {
        if (ctx_lens[s] < 0 || chunk_lens[s] < 0) return fail(ctx, ICARUS_ERR_INVALID_ARG, "sequence %d: negative length", s);
        int64_t end = (int64_t)ctx_lens[s] + chunk_lens[s];
        if (end > c.max_position) return fail(ctx, ICARUS_ERR_CAPACITY, "sequence %d: %lld tokens exceed max_position %d", s, (long long)end, c.max_position);
        if ((end + c.block_size - 1) / c.block_size > max_blocks)
            return fail(ctx, ICARUS_ERR_CAPACITY, "sequence %d: %lld tokens need %lld blocks, table has %d", s, (long long)end,
                        (long long)((end + c.block_size - 1) / c.block_size), max_blocks);
        total += chunk_lens[s];
    }
    if (total > 65535) return fail(ctx, ICARUS_ERR_UNSUPPORTED, "at most 65535 rows per call (got %lld)", (long long)total);
    *rows = (int)total;
    return ICARUS_OK;
}

icarus_status prepare_prefill(icarus_ctx *ctx, const void *kv_pool, const int32_t *block_tables, int32_t max_blocks, int32_t S,
                              const int32_t *ctx_lens, const int32_t *chunk_lens, int R, bool want_attention, void *workspace,
                              size_t workspace_bytes, hipStream_t st, const int32_t *extra, size_t n_extra, Prepared *pr) {
    const icarus_layer_config &c = ctx->cfg;
    int max_ctx = 0;
    for (int s = 0; s < S; ++s) max_ctx = std::max(max_ctx, ctx_lens[s] + chunk_lens[s]);
    pr->L = ws_layout(ctx, (size_t)R, (size_t)S, (size_t)max_ctx);
    const WsLayout &L = pr->L;
    icarus_status rc = check_common_ptrs(ctx, kv_pool, block_tables, workspace, workspace_bytes, L.total);
    if (rc) return rc;
    StageSlot *slot;
    rc = stage_acquire(ctx, L.meta_ints * 4, &slot);
    if (rc) return rc;
    int32_t *m = (int32_t *)slot->host;
    int r = 0;
    for (int s = 0; s < S; ++s)
        for (int i = 0; i < chunk_lens[s]; ++i, ++r) {
            m[r] = s;
            m[R + r] = -1;
            m[2 * R + r] = ctx_lens[s] + i;
            m[3 * R + r] = ctx_lens[s] + i + 1;
        }
    // Attention plan: the chunk's tokens are cut into groups of consecutive tokens whose stacked query
    // heads fill one workgroup of the prefill attention; each group is one plan sequence with a causal
    // stagger.
    char *ws = (char *)workspace;
    const int32_t *dmeta = (const int32_t *)(ws + L.meta);
    if (want_attention) {
        int g = c.n_q_heads / c.n_kv_heads, tq = std::max(1, attn_prefill_group_queries() / g);
        std::vector<int32_t> vkv, vrow0, vrows, vbt;
        int row = 0;
        for (int s = 0; s < S; ++s) {
            for (int t0 = 0; t0 < chunk_lens[s]; t0 += tq) {
                int n = std::min(tq, chunk_lens[s] - t0);
                vkv.push_back(ctx_lens[s] + t0 + n);
                vrow0.push_back(row + t0);
                vrows.push_back(n);
                vbt.push_back(s);
            }
            row += chunk_lens[s];
        }
        build_attn_plan(ctx, m, (size_t)4 * R, dmeta, (int)vkv.size(), vkv.data(), vrow0.data(), vrows.data(), vbt.data(), true,
                        L.max_items, &pr->hp);
    }
    size_t used = (size_t)4 * R + pr->hp.ints;
    if (n_extra) {
        memcpy(m + used, extra, n_extra * 4);
        pr->extra_dev = dmeta + used;
        used += n_extra;
    }
    rc = stage_commit(ctx, slot, ws + L.meta, used * 4, st);
    if (rc) return rc;
    pr->rm = RowMeta{dmeta, dmeta + R, dmeta + 2 * R, dmeta + 3 * R};
    return ICARUS_OK;
}

// ---- layer stack: workspace after the layer workspace, and the launch sequence ------------------------
struct StackLayout {
    size_t xa, xb, xn, logits, tok, total;
};

StackLayout stack_layout_from(const icarus_stack *st, const WsLayout &L, size_t rows, size_t logit_rows) {
    const icarus_layer_config &c = st->layers[0]->cfg;
    size_t es = c.dtype == ICARUS_BF16 ? 2 : 4;
    StackLayout s{};
    size_t off = align_up(L.total, 256);
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    s.xa = take(rows * c.d_model * es);
    s.xb = take(rows * c.d_model * es);
    s.xn = take(logit_rows * c.d_model * es * 2);  // gathered rows, then their normalised form
    s.logits = take(logit_rows * (size_t)st->vocab * 4);
    s.tok = take(logit_rows * 4);
    s.total = off;
    return s;
}

StackLayout stack_layout(const icarus_stack *st, size_t rows, size_t seqs, size_t max_ctx, size_t logit_rows) {
    return stack_layout_from(st, ws_layout(st->layers[0], rows, seqs, max_ctx), rows, logit_rows);
}

icarus_status stack_fail(icarus_stack *st, icarus_status rc, const char *msg) {
    snprintf(st->err, sizeof st->err, "%s", msg);
    return rc;
}

#define STACK_TRY(call) do { hipError_t e__ = (call); if (e__ != hipSuccess) return stack_fail(st, ICARUS_ERR_HIP, hipGetErrorString(e__)); } while (0)

// tok / tok_idx: the token of row r is tok[tok_idx ? tok_idx[r] : r].  head_rows: rows that go through
// the LM head (null: all R rows, n_head = R).  next_out [n_head]; pick [n_pick] / seq_next: optional
// seq_next[s] = next_out[pick[s]].
icarus_status run_stack(icarus_stack *st, char *ws, const StackLayout &SL, const Prepared &pr, void *const *kv_pools,
                        const int32_t *bt, int max_blocks, int R, bool decode, const int32_t *tok, const int32_t *tok_idx,
                        const int32_t *head_rows, int n_head, int32_t *next_out, const int32_t *pick, int n_pick, int32_t *seq_next,
                        float *logits, hipStream_t s) {
    icarus_ctx *c0 = st->layers[0];
    const Dims &dm = c0->dm;
    const size_t es = dm.bf16 ? 2 : 4;
    const int row_bytes = (int)(dm.d * es);
    void *xa = ws + SL.xa, *xb = ws + SL.xb;
    for (size_t l = 0; l < st->layers.size(); ++l) {
        icarus_status rc = check_common_ptrs(st->layers[l], kv_pools[l], bt, ws, SL.total, 0);
        if (rc) return stack_fail(st, rc, st->layers[l]->err);
    }
    STACK_TRY(launch_embed_rows(st->embed, tok, tok_idx, xa, R, row_bytes, s));
    // A layer whose down projection was split over K leaves its slices (and the residual) in the workspace when the
    // next layer can form its input rows from them: the separate reduction launch between two layers is saved.
    int pending = 0;
    for (size_t l = 0; l < st->layers.size(); ++l) {
        int left = 0;
        // the last layer may do the same when every row goes to the LM head as it is: the final norm sums the slices
        const bool head_takes_slices = !head_rows && n_head == R && layer_mfma_supported(c0) && gemm_mfma_supported(dm, dm.d);
        const bool may_defer = l + 1 < st->layers.size() ? layer_takes_slices(st->layers[l + 1], decode) : head_takes_slices;
        icarus_status rc = run_layer(st->layers[l], ws, pr.L, pr.rm, &pr.hp, R, decode, false, decode ? 0 : 1, kv_pools[l], bt, max_blocks,
                                     xa, xb, nullptr, s, &pr.fp, pending, may_defer ? &left : nullptr);
        if (rc) return stack_fail(st, rc, st->layers[l]->err);
        pending = left;
        std::swap(xa, xb);
    }
    // final norm + LM head on the chosen rows, greedy token
    char *xg = ws + SL.xn, *xn = xg + (size_t)n_head * row_bytes;
    const void *xh = xa;
    if (head_rows) {
        STACK_TRY(launch_gather_rows(xa, head_rows, xg, n_head, row_bytes, s));
        xh = xg;
    }
    float *lg = logits ? logits : (float *)(ws + SL.logits);
    if (layer_mfma_supported(c0) && gemm_mfma_supported(dm, dm.d)) {
        if (pending > 0)  // the last layer left its output in pieces (only when head_takes_slices)
            STACK_TRY(launch_sum_norm_shrink(dm, (const float *)(ws + pr.L.gemm_part), pending, (size_t)R * dm.d, ws + pr.L.z, xa, st->final_norm,
                                             xn, n_head, dm.d, nullptr, nullptr, nullptr, nullptr, s));
        else
            STACK_TRY(launch_norm_shrink(dm, xh, st->final_norm, xn, n_head, dm.d, nullptr, nullptr, nullptr, nullptr, nullptr, 0, s));
        GemmArgs g{};
        g.X = (const bf16_raw *)xn; g.ldx = dm.d; g.R = n_head; g.K = dm.d;
        g.W[0] = (const bf16_raw *)st->lm_head; g.n_seg[0] = st->vocab; g.nseg = 1;
        g.mode = GEMM_PLAIN; g.epi = EPI_F32; g.splits = 1;
        g.Y = lg; g.ldy = st->vocab;
        STACK_TRY(launch_gemm_mfma(g, s));
    } else {
        STACK_TRY(launch_rmsnorm(dm, xh, st->final_norm, xn, n_head, dm.d, s));
        STACK_TRY(launch_gemm_generic(dm, xn, dm.d, st->lm_head, n_head, st->vocab, dm.d, lg, st->vocab, s));
    }
    // the normed rows are dead once the logits exist: their buffer takes the argmax partials
    if (argmax_scratch_bytes(n_head) > (size_t)n_head * row_bytes) return stack_fail(st, ICARUS_ERR_UNSUPPORTED, "d_model too small for the argmax scratch");
    STACK_TRY(launch_argmax(lg, n_head, st->vocab, next_out, xn, s));
    if (seq_next && pick) STACK_TRY(launch_pick_rows(next_out, pick, seq_next, n_pick, s));
    return ICARUS_OK;
}

}  // namespace

// =====================================================================================
extern "C" {

const char *icarus_last_error(const icarus_ctx *ctx) { return ctx ? ctx->err : g_create_err; }

icarus_status icarus_create(const icarus_layer_config *cfg, const icarus_base_weights *base,
                            const icarus_lora_weights *lora, icarus_ctx **out) {
    if (out) *out = nullptr;
    if (!cfg || !base || !out) return fail(nullptr, ICARUS_ERR_INVALID_ARG, "cfg, base and out must not be null");
    const icarus_layer_config &c = *cfg;
    if (c.dtype != ICARUS_F32 && c.dtype != ICARUS_BF16) return fail(nullptr, ICARUS_ERR_INVALID_ARG, "dtype %d is neither ICARUS_F32 nor ICARUS_BF16", c.dtype);
    if (c.kv_dtype != ICARUS_KV_SAME && c.kv_dtype != ICARUS_KV_FP8_E4M3) return fail(nullptr, ICARUS_ERR_INVALID_ARG, "kv_dtype %d unknown", c.kv_dtype);
    if (c.kv_dtype == ICARUS_KV_FP8_E4M3 && !(c.k_scale > 0.0 && c.v_scale > 0.0 && std::isfinite(c.k_scale) && std::isfinite(c.v_scale)))
        return fail(nullptr, ICARUS_ERR_INVALID_ARG, "k_scale and v_scale must be finite and > 0 for an FP8 cache");
    if (c.d_model <= 0 || c.n_q_heads <= 0 || c.n_kv_heads <= 0 || c.head_dim <= 0 || c.d_ffn <= 0 || c.block_size <= 0 ||
        c.num_blocks <= 0 || c.max_position <= 0 || c.n_models < 0 || c.lora_rank < 0)
        return fail(nullptr, ICARUS_ERR_SHAPE, "all sizes must be positive (n_models, lora_rank non-negative)");
    if (c.n_q_heads % c.n_kv_heads) return fail(nullptr, ICARUS_ERR_SHAPE, "n_q_heads %d is not a multiple of n_kv_heads %d", c.n_q_heads, c.n_kv_heads);
    if (c.head_dim % 2 || c.head_dim > 256) return fail(nullptr, ICARUS_ERR_SHAPE, "head_dim %d must be even and at most 256", c.head_dim);
    if (!(c.rope_theta > 1.0) || !(c.rms_eps >= 0.0)) return fail(nullptr, ICARUS_ERR_INVALID_ARG, "rope_theta must exceed 1 and rms_eps be non-negative");
    if ((int64_t)c.num_blocks * c.block_size > (int64_t)1 << 40) return fail(nullptr, ICARUS_ERR_SHAPE, "pool too large");
    for (int p = 0; p < ICARUS_NPROJ; ++p) {
        if (!base->w[p]) return fail(nullptr, ICARUS_ERR_INVALID_ARG, "base weight %d is null", p);
        if (!aligned16(base->w[p])) return fail(nullptr, ICARUS_ERR_ALIGNMENT, "base weight %d is not 16-byte aligned", p);
    }
    if (!base->norm_attn || !base->norm_ffn) return fail(nullptr, ICARUS_ERR_INVALID_ARG, "norm weights are null");
    if (c.qk_norm && (!base->q_norm || !base->k_norm)) return fail(nullptr, ICARUS_ERR_INVALID_ARG, "qk_norm set but q_norm / k_norm is null");
    if (!aligned16(base->norm_attn) || !aligned16(base->norm_ffn) || !aligned16(base->q_norm) || !aligned16(base->k_norm))
        return fail(nullptr, ICARUS_ERR_ALIGNMENT, "norm weights must be 16-byte aligned");
    icarus_ctx *ctx = new (std::nothrow) icarus_ctx();
    if (!ctx) return fail(nullptr, ICARUS_ERR_INVALID_ARG, "out of host memory");
    ctx->cfg = c;
    ctx->base = *base;
    memset(&ctx->lora, 0, sizeof(ctx->lora));
    ctx->err[0] = 0;
    if (lora) ctx->lora = *lora;
    for (int p = 0; p < ICARUS_NPROJ; ++p) {
        if (!has_lora(ctx, p)) continue;
        if (!ctx->lora.A[p] || !ctx->lora.B[p]) {
            delete ctx;
            return fail(nullptr, ICARUS_ERR_INVALID_ARG, "projection %d is a LoRA target but its A or B is null", p);
        }
        if (!aligned16(ctx->lora.A[p]) || !aligned16(ctx->lora.B[p])) {
            delete ctx;
            return fail(nullptr, ICARUS_ERR_ALIGNMENT, "LoRA weights of projection %d are not 16-byte aligned", p);
        }
    }
    Dims &dm = ctx->dm;
    dm.d = c.d_model; dm.Hq = c.n_q_heads; dm.Hkv = c.n_kv_heads; dm.D = c.head_dim; dm.F = c.d_ffn; dm.Bk = c.block_size;
    dm.M = c.n_models; dm.r = c.lora_rank; dm.bf16 = c.dtype == ICARUS_BF16; dm.qk_norm = c.qk_norm != 0;
    dm.theta = c.rope_theta; dm.eps = (float)c.rms_eps; dm.lora_scale = (float)c.lora_scale;
    dm.kv8 = c.kv_dtype == ICARUS_KV_FP8_E4M3; dm.k_scale = dm.kv8 ? (float)c.k_scale : 1.f; dm.v_scale = dm.kv8 ? (float)c.v_scale : 1.f;
    *out = ctx;
    return ICARUS_OK;
}

void icarus_destroy(icarus_ctx *ctx) {
    if (!ctx) return;
    for (auto &sp : ctx->timer.pending) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
    for (auto e : ctx->timer.pool) (void)hipEventDestroy(e);
    for (auto &s : ctx->slots) {
        if (s.in_flight && s.ev) (void)hipEventSynchronize(s.ev);
        if (s.ev) (void)hipEventDestroy(s.ev);
        if (s.host) (void)hipHostFree(s.host);
    }
    delete ctx;
}

icarus_status icarus_set_full_decoders(icarus_ctx *ctx, const icarus_full_weights *fw) {
    if (!ctx) return ICARUS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(ctx->mu);
    if (!fw) {
        ctx->full_set = false;
        return ICARUS_OK;
    }
    const icarus_layer_config &c = ctx->cfg;
    if (c.n_models < 1) return fail(ctx, ICARUS_ERR_SHAPE, "private decoder weights need n_models >= 1");
    if (c.dtype != ICARUS_BF16 || !gemm_mfma_supported(ctx->dm, c.d_model) || !gemm_mfma_supported(ctx->dm, c.n_q_heads * c.head_dim) ||
        !gemm_mfma_supported(ctx->dm, c.d_ffn))
        return fail(ctx, ICARUS_ERR_UNSUPPORTED, "private decoder weights need the matrix-core path (bf16, K dimensions multiple of 64)");
    for (int p : {ICARUS_PROJ_Q, ICARUS_PROJ_O, ICARUS_PROJ_GATE, ICARUS_PROJ_UP, ICARUS_PROJ_DOWN}) {
        if (!fw->w[p]) return fail(ctx, ICARUS_ERR_INVALID_ARG, "private weights of projection %d are null", p);
        if (!aligned16(fw->w[p])) return fail(ctx, ICARUS_ERR_ALIGNMENT, "private weights of projection %d are not 16-byte aligned", p);
    }
    ctx->full = *fw;
    ctx->full_set = true;
    return ICARUS_OK;
}

icarus_status icarus_set_kernel_mode(icarus_ctx *ctx, int32_t mode) {
    if (!ctx) return ICARUS_ERR_INVALID_ARG;
    if (mode != 0 && mode != 1) return fail(ctx, ICARUS_ERR_INVALID_ARG, "kernel mode %d unknown", mode);
    ctx->mode = mode;
    return ICARUS_OK;
}

icarus_status icarus_timing_enable(icarus_ctx *ctx, int32_t on) {
    if (!ctx) return ICARUS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(ctx->mu);
    ctx->timer.on = on != 0;
    return ICARUS_OK;
}

icarus_status icarus_timing_read(icarus_ctx *ctx, double *ms, int32_t *launches) {
    if (!ctx || !ms || !launches) return ICARUS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(ctx->mu);
    PhaseTimer &tm = ctx->timer;
    for (auto &sp : tm.pending) {
        HIP_TRY(ctx, hipEventSynchronize(sp.b));
        float t = 0.f;
        HIP_TRY(ctx, hipEventElapsedTime(&t, sp.a, sp.b));
        tm.ms[sp.phase] += t;
        tm.launches[sp.phase] += 1;
        tm.pool.push_back(sp.a);
        tm.pool.push_back(sp.b);
    }
    tm.pending.clear();
    for (int i = 0; i < ICARUS_NPHASE; ++i) {
        ms[i] = tm.ms[i];
        launches[i] = tm.launches[i];
        tm.ms[i] = 0;
        tm.launches[i] = 0;
    }
    return ICARUS_OK;
}

icarus_status icarus_bench_copy(const void *src, void *dst, size_t bytes, void *stream) {
    if (!src || !dst || bytes % 16 || !aligned16(src) || !aligned16(dst)) return ICARUS_ERR_INVALID_ARG;
    return launch_bench_copy(src, dst, bytes, (hipStream_t)stream) == hipSuccess ? ICARUS_OK : ICARUS_ERR_HIP;
}

icarus_status icarus_bench_read(const void *src, size_t bytes, uint32_t *out, void *stream) {
    if (!src || !out || bytes % 8192 || !aligned16(src)) return ICARUS_ERR_INVALID_ARG;
    return launch_bench_read(src, bytes, out, (hipStream_t)stream) == hipSuccess ? ICARUS_OK : ICARUS_ERR_HIP;
}

icarus_status icarus_bench_mfma(float *out, int32_t waves, int32_t iters, void *stream) {
    if (!out || waves <= 0 || waves % 4 || iters <= 0) return ICARUS_ERR_INVALID_ARG;
    return launch_bench_mfma(out, waves, iters, (hipStream_t)stream) == hipSuccess ? ICARUS_OK : ICARUS_ERR_HIP;
}

size_t icarus_workspace_bytes(const icarus_ctx *ctx, int32_t max_rows, int32_t max_seqs, int32_t max_ctx) {
    if (!ctx || max_rows < 0 || max_seqs < 0 || max_ctx < 0) return 0;
    return ws_layout(ctx, (size_t)std::max(1, max_rows), (size_t)std::max(1, max_seqs), (size_t)max_ctx).total;
}

icarus_status icarus_validate_decode(icarus_ctx *ctx, int32_t max_blocks, int32_t S, const int32_t *ctx_lens, int32_t R,
                                     const int32_t *row_seq, const int32_t *row_model) {
    if (!ctx) return ICARUS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(ctx->mu);
    return check_decode_rows(ctx, max_blocks, S, ctx_lens, R, row_seq, row_model);
}

icarus_status icarus_decode_step(icarus_ctx *ctx, void *kv_pool, const int32_t *block_tables, int32_t max_blocks, int32_t S,
                                 const int32_t *ctx_lens, int32_t R, const int32_t *row_seq, const int32_t *row_model,
                                 const void *x_in, void *x_out, int64_t *slot_out, void *workspace, size_t workspace_bytes,
                                 void *stream) {
    if (!ctx) return ICARUS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(ctx->mu);
    icarus_status rc = check_decode_rows(ctx, max_blocks, S, ctx_lens, R, row_seq, row_model);
    if (rc) return rc;
    if (R == 0) return ICARUS_OK;
    if (!x_in || !x_out) return fail(ctx, ICARUS_ERR_INVALID_ARG, "x_in / x_out is null");
    if (!aligned16(x_in) || !aligned16(x_out) || (slot_out && !aligned16(slot_out))) return fail(ctx, ICARUS_ERR_ALIGNMENT, "x_in, x_out and slot_out must be 16-byte aligned");
    Prepared pr;
    rc = prepare_decode(ctx, kv_pool, block_tables, max_blocks, S, ctx_lens, R, row_seq, row_model, workspace, workspace_bytes,
                        (hipStream_t)stream, nullptr, 0, &pr);
    if (rc) return rc;
    return run_layer(ctx, (char *)workspace, pr.L, pr.rm, &pr.hp, R, true, false, 0, kv_pool, block_tables, max_blocks, x_in, x_out,
                     slot_out, (hipStream_t)stream, &pr.fp);
}

icarus_status icarus_prefill_kv(icarus_ctx *ctx, void *kv_pool, const int32_t *block_tables, int32_t max_blocks, int32_t S,
                                const int32_t *ctx_lens, const int32_t *chunk_lens, const void *x_in, void *x_out,
                                int64_t *slot_out, void *workspace, size_t workspace_bytes, void *stream) {
    if (!ctx) return ICARUS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(ctx->mu);
    int R = 0;
    icarus_status rc = check_prefill(ctx, max_blocks, S, ctx_lens, chunk_lens, &R);
    if (rc) return rc;
    if (R == 0) return ICARUS_OK;
    if (!x_in) return fail(ctx, ICARUS_ERR_INVALID_ARG, "x_in is null");
    if (!aligned16(x_in) || (x_out && !aligned16(x_out)) || (slot_out && !aligned16(slot_out))) return fail(ctx, ICARUS_ERR_ALIGNMENT, "x_in, x_out and slot_out must be 16-byte aligned");
    Prepared pr;
    rc = prepare_prefill(ctx, kv_pool, block_tables, max_blocks, S, ctx_lens, chunk_lens, R, x_out != nullptr, workspace,
                         workspace_bytes, (hipStream_t)stream, nullptr, 0, &pr);
    if (rc) return rc;
    return run_layer(ctx, (char *)workspace, pr.L, pr.rm, &pr.hp, R, false, x_out == nullptr, 1, kv_pool, block_tables, max_blocks, x_in,
                     x_out, slot_out, (hipStream_t)stream);
}

// Shared-KV attention alone.  use_static: the device scratch is the library's static array (nothing is allocated,
// the metadata travels as kernel arguments); else the caller's workspace and the pinned staging ring.
static icarus_status attn_shared_kv_impl(icarus_ctx *ctx, const void *q, const void *kv_pool, const int32_t *block_tables,
                                         int32_t max_blocks, int32_t S, const int32_t *kv_lens, int32_t R, const int32_t *row_seq,
                                         void *out, void *workspace, size_t workspace_bytes, bool use_static, void *stream) {
    if (!ctx) return ICARUS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(ctx->mu);
    const icarus_layer_config &c = ctx->cfg;
    if (S < 0 || R < 0 || max_blocks < 0) return fail(ctx, ICARUS_ERR_INVALID_ARG, "negative size");
    if (R == 0) return ICARUS_OK;
    if (!kv_lens || !row_seq) return fail(ctx, ICARUS_ERR_INVALID_ARG, "null metadata array");
    if (R > 65535) return fail(ctx, ICARUS_ERR_UNSUPPORTED, "at most 65535 rows per call (got %d)", R);
    int max_ctx = 0;
    for (int s = 0; s < S; ++s) {
        if (kv_lens[s] < 0) return fail(ctx, ICARUS_ERR_INVALID_ARG, "kv_lens[%d] is negative", s);
        if (kv_lens[s] > c.max_position) return fail(ctx, ICARUS_ERR_CAPACITY, "sequence %d: %d tokens exceed max_position %d", s, kv_lens[s], c.max_position);
        if (((int64_t)kv_lens[s] + c.block_size - 1) / c.block_size > max_blocks)
            return fail(ctx, ICARUS_ERR_CAPACITY, "sequence %d: %d tokens need more than %d blocks", s, kv_lens[s], max_blocks);
        max_ctx = std::max(max_ctx, kv_lens[s]);
    }
    for (int r = 0; r < R; ++r) {
        if (row_seq[r] < 0 || row_seq[r] >= S) return fail(ctx, ICARUS_ERR_INVALID_ARG, "row %d: sequence id %d outside 0..%d", r, row_seq[r], S - 1);
        if (r && row_seq[r] < row_seq[r - 1]) return fail(ctx, ICARUS_ERR_ROW_ORDER, "row %d: rows must be grouped by sequence in non-decreasing order", r);
    }
    if (!q || !out) return fail(ctx, ICARUS_ERR_INVALID_ARG, "q / out is null");
    if (!aligned16(q) || !aligned16(out)) return fail(ctx, ICARUS_ERR_ALIGNMENT, "q and out must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    WsLayout L = ws_layout(ctx, (size_t)R, (size_t)S, (size_t)max_ctx);
    icarus_status rc;
    char *ws = (char *)workspace;
    StageSlot *slot = nullptr;
    std::vector<int32_t> hostmeta;
    int32_t *m;
    if (use_static) {
        if (!kv_pool || !block_tables) return fail(ctx, ICARUS_ERR_INVALID_ARG, "kv_pool / block_tables is null");
        if (!aligned16(kv_pool) || !aligned16(block_tables)) return fail(ctx, ICARUS_ERR_ALIGNMENT, "kv_pool and block_tables must be 16-byte aligned");
        rc = static_scratch(ctx, &ws);
        if (rc) return rc;
        hostmeta.resize(L.meta_ints);
        m = hostmeta.data();
    } else {
        rc = check_common_ptrs(ctx, kv_pool, block_tables, workspace, workspace_bytes, L.total);
        if (rc) return rc;
        rc = stage_acquire(ctx, L.meta_ints * 4, &slot);
        if (rc) return rc;
        m = (int32_t *)slot->host;
    }
    std::vector<int32_t> row0((size_t)S, 0), rows((size_t)S, 0);
    for (int r = 0; r < R; ++r) {
        int s = row_seq[r];
        m[r] = s;
        m[R + r] = 0;
        m[2 * R + r] = kv_lens[s] - 1;
        m[3 * R + r] = kv_lens[s];
        if (rows[s]++ == 0) row0[s] = r;
    }
    if (use_static) L.meta = 0;  // the static scratch starts with the metadata
    const int32_t *dmeta = (const int32_t *)(ws + L.meta);
    HostPlan hp;
    build_attn_plan(ctx, m, (size_t)4 * R, dmeta, S, kv_lens, row0.data(), rows.data(), nullptr, false, L.max_items, &hp);
    const size_t used = (size_t)4 * R + hp.ints;
    if (use_static) {
        // what THIS call needs, from its own plan: metadata, then the partial results of its pieces
        const size_t pj = hp.valid ? (size_t)hp.pl.n_items * c.n_kv_heads * hp.pl.g_max : 0;
        L.part_o = align_up(used * 4, 256);
        L.part_ml = align_up(L.part_o + pj * c.head_dim * 4, 256);
        const size_t need = L.part_ml + pj * 2 * 4;
        if (need > kStaticScratchBytes)
            return fail(ctx, ICARUS_ERR_CAPACITY, "this call needs %zu bytes of scratch, the static array holds %zu", need, kStaticScratchBytes);
        rc = stage_by_kernarg(ctx, m, used, (int32_t *)ws, st);
    } else {
        rc = stage_commit(ctx, slot, ws + L.meta, used * 4, st);
    }
    if (rc) return rc;
    RowMeta rm{dmeta, dmeta + R, dmeta + 2 * R, dmeta + 3 * R};
    return run_decode_attention(ctx, ws, L, rm, &hp, q, kv_pool, block_tables, max_blocks, out, R, st);
}

icarus_status icarus_attn_shared_kv(icarus_ctx *ctx, const void *q, const void *kv_pool, const int32_t *block_tables,
                                    int32_t max_blocks, int32_t S, const int32_t *kv_lens, int32_t R, const int32_t *row_seq,
                                    void *out, void *workspace, size_t workspace_bytes, void *stream) {
    return attn_shared_kv_impl(ctx, q, kv_pool, block_tables, max_blocks, S, kv_lens, R, row_seq, out, workspace, workspace_bytes, false,
                               stream);
}

icarus_status icarus_attn_shared_kv_static(icarus_ctx *ctx, const void *q, const void *kv_pool, const int32_t *block_tables,
                                           int32_t max_blocks, int32_t S, const int32_t *kv_lens, int32_t R,
                                           const int32_t *row_seq, void *out, void *stream) {
    return attn_shared_kv_impl(ctx, q, kv_pool, block_tables, max_blocks, S, kv_lens, R, row_seq, out, nullptr, 0, true, stream);
}

icarus_status icarus_set_attn_piece_limit(icarus_ctx *ctx, int32_t tokens) {
    if (!ctx) return ICARUS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(ctx->mu);
    if (tokens < 0) return fail(ctx, ICARUS_ERR_INVALID_ARG, "piece limit %d is negative", tokens);
    ctx->attn_chunk_override = tokens;
    return ICARUS_OK;
}

icarus_status icarus_validate_block_tables(icarus_ctx *ctx, const int32_t *tables, int32_t max_blocks, int32_t S,
                                           const int32_t *ctx_lens, const int32_t *extra) {
    if (!ctx) return ICARUS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(ctx->mu);
    const icarus_layer_config &c = ctx->cfg;
    if (S < 0 || max_blocks < 0) return fail(ctx, ICARUS_ERR_INVALID_ARG, "negative size");
    if (S == 0) return ICARUS_OK;
    if (!tables || !ctx_lens) return fail(ctx, ICARUS_ERR_INVALID_ARG, "null table / ctx_lens");
    std::vector<int32_t> writer((size_t)c.num_blocks, -1);  // sequence that appends into the block
    for (int s = 0; s < S; ++s) {
        const int64_t add = extra ? extra[s] : 1;
        if (ctx_lens[s] < 0 || add < 0) return fail(ctx, ICARUS_ERR_INVALID_ARG, "sequence %d: negative length", s);
        const int64_t end = (int64_t)ctx_lens[s] + add;
        const int64_t nb = (end + c.block_size - 1) / c.block_size;
        if (nb > max_blocks) return fail(ctx, ICARUS_ERR_CAPACITY, "sequence %d: %lld tokens need %lld blocks, table has %d", s, (long long)end, (long long)nb, max_blocks);
        const int32_t *row = tables + (size_t)s * max_blocks;
        for (int64_t b = 0; b < nb; ++b)
            if (row[b] < 0 || row[b] >= c.num_blocks)
                return fail(ctx, ICARUS_ERR_CAPACITY, "sequence %d: block table entry %lld is %d, the pool has blocks 0..%d", s, (long long)b, row[b], c.num_blocks - 1);
        if (add == 0) continue;
        for (int64_t b = ctx_lens[s] / c.block_size; b < nb; ++b) {
            int32_t &w = writer[(size_t)row[b]];
            if (w >= 0 && w != s)
                return fail(ctx, ICARUS_ERR_INVALID_ARG, "block %d would be appended to by sequences %d and %d", row[b], w, s);
            w = s;
        }
    }
    return ICARUS_OK;
}

// ---- layer stack -----------------------------------------------------------------------------------------

icarus_status icarus_stack_create(const icarus_stack_config *cfg, icarus_stack **out) {
    if (!cfg || !out) return fail(nullptr, ICARUS_ERR_INVALID_ARG, "null argument");
    *out = nullptr;
    if (cfg->n_layers < 1 || !cfg->layers) return fail(nullptr, ICARUS_ERR_INVALID_ARG, "a stack needs at least one layer");
    if (cfg->vocab < 8 || cfg->vocab % 8) return fail(nullptr, ICARUS_ERR_SHAPE, "vocab %d must be a positive multiple of 8", cfg->vocab);
    if (!cfg->embed || !cfg->final_norm || !cfg->lm_head) return fail(nullptr, ICARUS_ERR_INVALID_ARG, "null embed / final_norm / lm_head");
    if (!aligned16(cfg->embed) || !aligned16(cfg->final_norm) || !aligned16(cfg->lm_head))
        return fail(nullptr, ICARUS_ERR_ALIGNMENT, "embed, final_norm and lm_head must be 16-byte aligned");
    for (int l = 0; l < cfg->n_layers; ++l) {
        if (!cfg->layers[l]) return fail(nullptr, ICARUS_ERR_INVALID_ARG, "layer %d is null", l);
        if (memcmp(&cfg->layers[l]->cfg, &cfg->layers[0]->cfg, sizeof(icarus_layer_config)) != 0)
            return fail(nullptr, ICARUS_ERR_SHAPE, "layer %d differs in configuration from layer 0", l);
    }
    const icarus_layer_config &c = cfg->layers[0]->cfg;
    if ((c.d_model * (c.dtype == ICARUS_BF16 ? 2 : 4)) % 16) return fail(nullptr, ICARUS_ERR_SHAPE, "d_model rows must be a multiple of 16 bytes");
    // the greedy token's partial results take the place of the normed rows once the logits exist
    if (argmax_scratch_bytes(1) > (size_t)c.d_model * (c.dtype == ICARUS_BF16 ? 2 : 4))
        return fail(nullptr, ICARUS_ERR_UNSUPPORTED, "a row of d_model must hold at least %zu bytes", argmax_scratch_bytes(1));
    icarus_stack *st = new (std::nothrow) icarus_stack();
    if (!st) return fail(nullptr, ICARUS_ERR_HIP, "out of host memory");
    st->layers.assign(cfg->layers, cfg->layers + cfg->n_layers);
    st->vocab = cfg->vocab;
    st->embed = cfg->embed;
    st->final_norm = cfg->final_norm;
    st->lm_head = cfg->lm_head;
    st->err[0] = 0;
    *out = st;
    return ICARUS_OK;
}

void icarus_stack_destroy(icarus_stack *st) { delete st; }

const char *icarus_stack_last_error(const icarus_stack *st) { return st ? st->err : g_create_err; }

size_t icarus_stack_workspace_bytes(const icarus_stack *st, int32_t max_rows, int32_t max_seqs, int32_t max_ctx,
                                    int32_t max_logit_rows) {
    if (!st || max_rows < 0 || max_seqs < 0 || max_ctx < 0 || max_logit_rows < 0) return 0;
    return stack_layout(st, (size_t)std::max(1, max_rows), (size_t)std::max(1, max_seqs), (size_t)max_ctx,
                        (size_t)std::max(1, max_logit_rows)).total;
}

icarus_status icarus_stack_prefill(icarus_stack *st, void *const *kv_pools, const int32_t *block_tables, int32_t max_blocks,
                                   int32_t S, const int32_t *ctx_lens, const int32_t *chunk_lens, const int32_t *tokens,
                                   int32_t *next_token, float *logits, void *workspace, size_t workspace_bytes, void *stream) {
    if (!st) return ICARUS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(st->mu);
    icarus_ctx *c0 = st->layers[0];
    int R = 0;
    icarus_status rc = check_prefill(c0, max_blocks, S, ctx_lens, chunk_lens, &R);
    if (rc) return stack_fail(st, rc, c0->err);
    if (R == 0) return ICARUS_OK;
    if (!kv_pools || !tokens || !next_token) return stack_fail(st, ICARUS_ERR_INVALID_ARG, "null kv_pools / tokens / next_token");
    std::vector<int32_t> extra((size_t)R + S);  // prompt tokens, then each sequence's last chunk row (-1: empty chunk)
    int n_logit = 0;
    {
        int row = 0;
        for (int s = 0; s < S; ++s) {
            for (int i = 0; i < chunk_lens[s]; ++i, ++row) {
                if (tokens[row] < 0 || tokens[row] >= st->vocab) return stack_fail(st, ICARUS_ERR_INVALID_ARG, "token out of range");
                extra[row] = tokens[row];
            }
            if (chunk_lens[s] == 0) return stack_fail(st, ICARUS_ERR_INVALID_ARG, "every sequence of a stack prefill needs at least one token");
            extra[(size_t)R + n_logit++] = row - 1;
        }
    }
    Prepared pr;
    // the layer workspace sits at the start of the stack workspace
    rc = prepare_prefill(c0, kv_pools[0], block_tables, max_blocks, S, ctx_lens, chunk_lens, R, true, workspace, workspace_bytes,
                         (hipStream_t)stream, extra.data(), extra.size(), &pr);
    if (rc) return stack_fail(st, rc, c0->err);
    StackLayout SL = stack_layout_from(st, pr.L, (size_t)R, (size_t)S);
    if (workspace_bytes < SL.total) return stack_fail(st, ICARUS_ERR_CAPACITY, "workspace too small");
    return run_stack(st, (char *)workspace, SL, pr, kv_pools, block_tables, max_blocks, R, false, pr.extra_dev, nullptr,
                     pr.extra_dev + R, S, next_token, nullptr, 0, nullptr, logits, (hipStream_t)stream);
}

icarus_status icarus_stack_decode(icarus_stack *st, void *const *kv_pools, const int32_t *block_tables, int32_t max_blocks,
                                  int32_t S, const int32_t *ctx_lens, int32_t R, const int32_t *row_seq,
                                  const int32_t *row_model, const int32_t *seq_token, int32_t *row_next, int32_t *seq_next,
                                  float *logits, void *workspace, size_t workspace_bytes, void *stream) {
    if (!st) return ICARUS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(st->mu);
    icarus_ctx *c0 = st->layers[0];
    icarus_status rc = check_decode_rows(c0, max_blocks, S, ctx_lens, R, row_seq, row_model);
    if (rc) return stack_fail(st, rc, c0->err);
    if (R == 0) return ICARUS_OK;
    if (!kv_pools || !seq_token || !row_next) return stack_fail(st, ICARUS_ERR_INVALID_ARG, "null kv_pools / seq_token / row_next");
    std::vector<int32_t> extra((size_t)S, -1);  // last row of each sequence
    for (int r = 0; r < R; ++r) extra[row_seq[r]] = r;
    for (int s = 0; s < S; ++s)
        if (extra[s] < 0) extra[s] = 0;  // a sequence without rows: its seq_next entry is meaningless
    Prepared pr;
    rc = prepare_decode(c0, kv_pools[0], block_tables, max_blocks, S, ctx_lens, R, row_seq, row_model, workspace, workspace_bytes,
                        (hipStream_t)stream, extra.data(), extra.size(), &pr);
    if (rc) return stack_fail(st, rc, c0->err);
    StackLayout SL = stack_layout_from(st, pr.L, (size_t)R, (size_t)R);
    if (workspace_bytes < SL.total) return stack_fail(st, ICARUS_ERR_CAPACITY, "workspace too small");
    return run_stack(st, (char *)workspace, SL, pr, kv_pools, block_tables, max_blocks, R, true, seq_token, pr.rm.row_seq, nullptr, R,
                     row_next, pr.extra_dev, S, seq_next, logits, (hipStream_t)stream);
}

}  // extern "C"

/*
 * ICaRus shared-KV layer step -- CPU ORACLE.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of one transformer layer's
 * shared-KV step as the paper defines it: a frozen logical encoder (base
 * weights) is the only writer of the KV cache (Eq. 4), and task-specific
 * logical decoders (base weights + a LoRA adapter each) only issue queries
 * against that cache (Eq. 5).  Nothing in the product library links, includes
 * or calls this file; it shares no code, table or constant with the GPU path.
 * Only the tests, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * Arithmetic: inputs and weights are float32 arrays (holding bf16-representable
 * values in the bf16 configurations); every intermediate is float64; no
 * blocking, fusion or reordering beyond what each definition states.
 * Contractual roundings: K and V are rounded to the cache precision when they
 * are written to the cache, and x_out is rounded to the storage precision
 * (bf16 when cfg.bf16 != 0, float32 otherwise).
 *
 * Pinned by tests/test_oracle_*.py (closed forms, brute force on tiny shapes,
 * a float64 library cross-check of the adapter-free special case, and the
 * paper's structural invariants).  No function here is "parity unpinned".
 *
 * Readings of points on which the paper is silent or garbled:
 *  - Alg. 2 prints the adapter applied to the base linear's OUTPUT; read as
 *    standard LoRA on the layer INPUT: y = W x + s * B (A x)  (Sec. 3.2 names
 *    LoRA as the adapter).
 *  - Alg. 3 stacks exactly two rows; generalised to 1 + m rows per sequence.
 *  - Alg. 3's concat over heads: every stream's head h uses kv-head floor(h/g),
 *    as in the base model.
 *  - Block internals (norms, residuals, SwiGLU, RoPE) follow the base model
 *    families the paper evaluates (Sec. 4.1): pre-norm RMSNorm, rotate-half
 *    RoPE with inv_freq_i = theta^(-2i/D), SwiGLU down(silu(gate) * up).
 *  - K is cached after RoPE; the current token attends to itself (append
 *    first, then attend over positions 0..p inclusive; Sec. 3.3, Alg. 3).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_Q = 0, ORC_K, ORC_V, ORC_O, ORC_GATE, ORC_UP, ORC_DOWN, ORC_NPROJ };

typedef struct {
    int32_t d_model, n_q_heads, n_kv_heads, head_dim, d_ffn;
    int32_t block_size, num_blocks, n_models, lora_rank;
    int32_t lora_target_mask; /* bit p set: projection p carries an adapter */
    int32_t qk_norm;          /* per-head RMSNorm on q and k before RoPE */
    int32_t bf16;             /* 1: cache and x_out hold bf16 values; 0: float32 */
    double rope_theta, rms_eps, lora_scale;
    int32_t kv_fp8;           /* 1: the cache holds FP8 E4M3 codes with one scale for all K and one for all V */
    double k_scale, v_scale;  /* value = code * scale (kv_fp8 only) */
} orc_config;

typedef struct {
    const float *w[ORC_NPROJ]; /* W_p [out_p, in_p] row-major */
    const float *norm_attn, *norm_ffn; /* [d_model] */
    const float *q_norm, *k_norm;      /* [head_dim], only if qk_norm */
} orc_base;

typedef struct {
    const float *A[ORC_NPROJ]; /* A_p [n_models, r, in_p]  */
    const float *B[ORC_NPROJ]; /* B_p [n_models, out_p, r] */
    const float *F[ORC_NPROJ]; /* or: F_p [n_models, out_p, in_p], a private full weight per decoder
                                  (full fine-tuning, or any adapter merged into the weight: Sec. 3.2
                                  leaves the decoder's adaptation method open); overrides A, B */
} orc_lora;

static int proj_in(const orc_config *c, int p) {
    switch (p) {
    case ORC_Q: case ORC_K: case ORC_V: case ORC_GATE: case ORC_UP: return c->d_model;
    case ORC_O: return c->n_q_heads * c->head_dim;
    default: return c->d_ffn;
    }
}
static int proj_out(const orc_config *c, int p) {
    switch (p) {
    case ORC_Q: return c->n_q_heads * c->head_dim;
    case ORC_K: case ORC_V: return c->n_kv_heads * c->head_dim;
    case ORC_GATE: case ORC_UP: return c->d_ffn;
    default: return c->d_model;
    }
}

/* ---- rounding to storage precision ------------------------------------- */

/* Round a double to the nearest bfloat16 value (8 significant bits), ties to
 * even, directly from double (no intermediate float rounding). */
double orc_round_bf16(double x) {
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    (void)frexp(x, &e);           /* |x| = m * 2^e, m in [0.5,1) */
    int q = e - 8;                /* quantum exponent for 8 significant bits */
    if (q < -133) q = -133;       /* bf16 subnormal quantum 2^-133 */
    double r = ldexp(nearbyint(ldexp(x, -q)), q); /* nearbyint: ties-to-even */
    return r;
}
/* Round a double to the nearest FP8 E4M3 value of the OCP 8-bit floating point
 * specification (4 exponent bits, bias 7, 3 mantissa bits, no infinities, largest
 * finite value 448, subnormals down to 2^-9), ties to even; magnitudes beyond 448
 * saturate to +-448.  The quantised KV cache is this paper's "orthogonal" prior
 * work (Sec. 1); the format is that of the hardware's FP8 conversions. */
double orc_round_e4m3(double x) {
    if (x == 0.0 || isnan(x)) return x;
    double a = fabs(x);
    if (a >= 448.0) return copysign(448.0, x);
    int e;
    (void)frexp(a, &e);           /* a = m * 2^e, m in [0.5,1) */
    int q = e - 4;                /* quantum exponent for 4 significant bits */
    if (q < -9) q = -9;           /* subnormal quantum 2^-9 (smallest normal 2^-6) */
    double r = ldexp(nearbyint(ldexp(a, -q)), q);
    if (r > 448.0) r = 448.0;
    return copysign(r, x);
}

/* What the cache holds for a K (kv = 0) or V (kv = 1) element x. */
static double round_cache(const orc_config *c, double x, int kv) {
    if (!c->kv_fp8) return c->bf16 ? orc_round_bf16(x) : (double)(float)x;
    double s = kv ? c->v_scale : c->k_scale;
    return orc_round_e4m3(x / s) * s;
}
static double round_store(const orc_config *c, double x) {
    return c->bf16 ? orc_round_bf16(x) : (double)(float)x;
}

/* ---- elementary operations --------------------------------------------- */

/* RMSNorm: y_i = x_i / sqrt(mean(x^2) + eps) * w_i. */
void orc_rmsnorm(const double *x, const float *w, double eps, int n, double *y) {
    double ss = 0.0;
    for (int i = 0; i < n; ++i) ss += x[i] * x[i];
    double inv = 1.0 / sqrt(ss / n + eps);
    for (int i = 0; i < n; ++i) y[i] = x[i] * inv * (double)w[i];
}

/* Linear (Alg. 1, Alg. 2): y = W x, W [out, in] row-major. */
void orc_linear(const float *W, int out, int in, const double *x, double *y) {
#pragma omp parallel for schedule(static) if ((long)out * in > (1L << 18))
    for (int o = 0; o < out; ++o) {
        const float *wr = W + (size_t)o * in;
        double acc = 0.0;
        for (int i = 0; i < in; ++i) acc += (double)wr[i] * x[i];
        y[o] = acc;
    }
}

/* AdaptiveLinear (Alg. 2), read as LoRA: delta = s * B (A x),
 * A [r, in], B [out, r]. */
void orc_adaptive_linear(const float *A, const float *B, int out, int in, int r,
                         double s, const double *x, double *delta) {
    double *t = (double *)malloc(sizeof(double) * (size_t)r);
    orc_linear(A, r, in, x, t);
    for (int o = 0; o < out; ++o) {
        double acc = 0.0;
        for (int k = 0; k < r; ++k) acc += (double)B[(size_t)o * r + k] * t[k];
        delta[o] = s * acc;
    }
    free(t);
}

/* ICaRusLinear (Alg. 2) over T stacked rows: the base Linear on every row, then
 * the adapter delta added on the decoder rows only (model[t] >= 0).  Row 0 of a
 * stack is the logical encoder (model -1). */
void orc_icarus_linear(const orc_config *c, const orc_base *b, const orc_lora *l,
                       int p, int T, const int32_t *model, const double *X, double *Y) {
    int in = proj_in(c, p), out = proj_out(c, p), r = c->lora_rank;
    if (l && l->F[p]) {  /* private decoder weights: a decoder row uses its own matrix, an encoder row the base */
        for (int t = 0; t < T; ++t)
            orc_linear(model[t] < 0 ? b->w[p] : l->F[p] + (size_t)model[t] * out * in, out, in, X + (size_t)t * in,
                       Y + (size_t)t * out);
        return;
    }
    for (int t = 0; t < T; ++t)
        orc_linear(b->w[p], out, in, X + (size_t)t * in, Y + (size_t)t * out);
    if (!l || !((c->lora_target_mask >> p) & 1) || !l->A[p] || !l->B[p]) return;
    double *delta = (double *)malloc(sizeof(double) * (size_t)out);
    for (int t = 0; t < T; ++t) {
        int j = model[t];
        if (j < 0) continue;
        orc_adaptive_linear(l->A[p] + (size_t)j * r * in, l->B[p] + (size_t)j * out * r,
                            out, in, r, c->lora_scale, X + (size_t)t * in, delta);
        for (int o = 0; o < out; ++o) Y[(size_t)t * out + o] += delta[o];
    }
    free(delta);
}

/* Rotary position embedding, rotate-half pairing (i, i + D/2):
 * angle_i = pos * theta^(-2i/D); (a, b) -> (a cos - b sin, b cos + a sin). */
void orc_rope(double *v, int H, int D, int pos, double theta) {
    int half = D / 2;
    for (int h = 0; h < H; ++h) {
        double *x = v + (size_t)h * D;
        for (int i = 0; i < half; ++i) {
            double ang = (double)pos * pow(theta, -2.0 * i / D);
            double cs = cos(ang), sn = sin(ang);
            double a = x[i], bb = x[i + half];
            x[i] = a * cs - bb * sn;
            x[i + half] = bb * cs + a * sn;
        }
    }
}

/* Per-head RMSNorm over head_dim with one shared weight vector [D]. */
static void head_rmsnorm(double *v, int H, int D, const float *w, double eps) {
    for (int h = 0; h < H; ++h) orc_rmsnorm(v + (size_t)h * D, w, eps, D, v + (size_t)h * D);
}

static double silu(double x) { return x / (1.0 + exp(-x)); }

/* ---- the paged shared cache -------------------------------------------- */

/* Physical slot of logical position pos: block_table[pos / Bk] * Bk + pos % Bk. */
int64_t orc_slot(const int32_t *bt_row, int32_t pos, int32_t Bk) {
    return (int64_t)bt_row[pos / Bk] * Bk + pos % Bk;
}

/* Oracle pool layout: float [num_blocks][2][Hkv][Bk][D] (0 = K, 1 = V). */
static float *pool_at(const orc_config *c, float *pool, int64_t slot, int kv, int head) {
    int64_t blk = slot / c->block_size, off = slot % c->block_size;
    return pool + ((((size_t)blk * 2 + kv) * c->n_kv_heads + head) * c->block_size + off) * c->head_dim;
}

/* concat_sequence (Alg. 3): append one token's k, v [Hkv, D] at position pos. */
static int64_t cache_append(const orc_config *c, float *pool, const int32_t *bt_row, int pos,
                            const double *k, const double *v) {
    int64_t slot = orc_slot(bt_row, pos, c->block_size);
    for (int h = 0; h < c->n_kv_heads; ++h) {
        float *kd = pool_at(c, pool, slot, 0, h), *vd = pool_at(c, pool, slot, 1, h);
        for (int i = 0; i < c->head_dim; ++i) {
            kd[i] = (float)round_cache(c, k[(size_t)h * c->head_dim + i], 0);
            vd[i] = (float)round_cache(c, v[(size_t)h * c->head_dim + i], 1);
        }
    }
    return slot;
}

/* Gather positions 0..n-1 of one sequence into contiguous K, V [n, Hkv, D]. */
void orc_gather_kv(const orc_config *c, const float *pool, const int32_t *bt_row, int n,
                   float *Kc, float *Vc) {
    size_t hd = (size_t)c->n_kv_heads * c->head_dim;
    for (int t = 0; t < n; ++t) {
        int64_t slot = orc_slot(bt_row, t, c->block_size);
        for (int h = 0; h < c->n_kv_heads; ++h) {
            memcpy(Kc + t * hd + (size_t)h * c->head_dim, pool_at(c, (float *)pool, slot, 0, h),
                   sizeof(float) * c->head_dim);
            memcpy(Vc + t * hd + (size_t)h * c->head_dim, pool_at(c, (float *)pool, slot, 1, h),
                   sizeof(float) * c->head_dim);
        }
    }
}

/* ---- attention: the definition ----------------------------------------- */

/* GQA over contiguous K, V [n, Hkv, D] for U stacked query heads q [U, D];
 * stacked head u uses kv-head kv_of[u].
 * o_u = sum_n softmax_n(q_u . K[n][c] / sqrt(D)) V[n][c]   (max-subtracted). */
void orc_attention(int U, int D, int Hkv, const int32_t *kv_of, const double *q,
                   const float *Kc, const float *Vc, int n, double *o) {
    double scale = 1.0 / sqrt((double)D);
    size_t hd = (size_t)Hkv * D;
#pragma omp parallel for schedule(dynamic) if ((long)U * n > 4096)
    for (int u = 0; u < U; ++u) {
        int cc = kv_of[u];
        double *sc = (double *)malloc(sizeof(double) * (size_t)n);
        double mx = -INFINITY;
        for (int t = 0; t < n; ++t) {
            const float *kr = Kc + t * hd + (size_t)cc * D;
            double acc = 0.0;
            for (int i = 0; i < D; ++i) acc += q[(size_t)u * D + i] * (double)kr[i];
            sc[t] = acc * scale;
            if (sc[t] > mx) mx = sc[t];
        }
        double den = 0.0;
        for (int t = 0; t < n; ++t) { sc[t] = exp(sc[t] - mx); den += sc[t]; }
        for (int i = 0; i < D; ++i) {
            double acc = 0.0;
            for (int t = 0; t < n; ++t) acc += sc[t] * (double)Vc[t * hd + (size_t)cc * D + i];
            o[(size_t)u * D + i] = acc / den;
        }
        free(sc);
    }
}

/* Attention alone for a batch of stacked rows (Alg. 3, the GQA line): q [R, Hq, D]
 * already normed and rotated, kv_lens[s] INCLUDES the current token.  Rows of a
 * sequence are stacked on the head axis and attend once to that sequence's cache. */
void orc_attn_shared_kv(const orc_config *c, const float *q, const float *pool,
                        const int32_t *block_tables, int max_blocks, int S,
                        const int32_t *kv_lens, int R, const int32_t *row_seq, double *out) {
    int Hq = c->n_q_heads, D = c->head_dim, g = Hq / c->n_kv_heads;
    size_t hd = (size_t)c->n_kv_heads * D;
    for (int s = 0; s < S; ++s) {
        int n = kv_lens[s];
        int T = 0, r0 = -1;
        for (int r = 0; r < R; ++r) if (row_seq[r] == s) { if (r0 < 0) r0 = r; ++T; }
        if (T == 0) continue;
        int U = T * Hq;
        float *Kc = (float *)malloc(sizeof(float) * hd * (size_t)(n > 0 ? n : 1));
        float *Vc = (float *)malloc(sizeof(float) * hd * (size_t)(n > 0 ? n : 1));
        orc_gather_kv(c, pool, block_tables + (size_t)s * max_blocks, n, Kc, Vc);
        double *qs = (double *)malloc(sizeof(double) * (size_t)U * D);
        int32_t *kv_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)U);
        for (int t = 0; t < T; ++t)
            for (int h = 0; h < Hq; ++h) {
                kv_of[t * Hq + h] = h / g;
                for (int i = 0; i < D; ++i)
                    qs[((size_t)t * Hq + h) * D + i] = (double)q[((size_t)(r0 + t) * Hq + h) * D + i];
            }
        orc_attention(U, D, c->n_kv_heads, kv_of, qs, Kc, Vc, n, out + (size_t)r0 * Hq * D);
        free(Kc); free(Vc); free(qs); free(kv_of);
    }
}

/* ---- one sequence's stack through the layer ---------------------------- */

/* K/V step of the logical encoder (Alg. 3: Linear(X; W_k), Linear(X; W_v) with
 * base weights only; Alg. 1 for prefill rows): from the normed encoder row to
 * the rounded cache entry at position pos.  Returns the slot. */
static int64_t encoder_kv_step(const orc_config *c, const orc_base *b, float *pool,
                               const int32_t *bt_row, int pos, const double *xn) {
    int kvd = c->n_kv_heads * c->head_dim;
    double *k = (double *)malloc(sizeof(double) * kvd), *v = (double *)malloc(sizeof(double) * kvd);
    orc_linear(b->w[ORC_K], kvd, c->d_model, xn, k);
    orc_linear(b->w[ORC_V], kvd, c->d_model, xn, v);
    if (c->qk_norm) head_rmsnorm(k, c->n_kv_heads, c->head_dim, b->k_norm, c->rms_eps);
    orc_rope(k, c->n_kv_heads, c->head_dim, pos, c->rope_theta);
    int64_t slot = cache_append(c, pool, bt_row, pos, k, v);
    free(k); free(v);
    return slot;
}

/* Everything after the cache append for T stacked rows of one sequence that all
 * sit at position pos (Alg. 3 from the ICaRusLinear for Q to the FFN).
 * X, Xn [T, d]: raw and attention-normed inputs.  Y [T, d]: unrounded outputs. */
static void stack_after_append(const orc_config *c, const orc_base *b, const orc_lora *l,
                               const float *pool, const int32_t *bt_row, int pos, int T,
                               const int32_t *model, const double *X, const double *Xn, double *Y) {
    int d = c->d_model, Hq = c->n_q_heads, D = c->head_dim, F = c->d_ffn, g = Hq / c->n_kv_heads;
    int qd = Hq * D, n = pos + 1;
    size_t hd = (size_t)c->n_kv_heads * D;
    double *Q = (double *)malloc(sizeof(double) * (size_t)T * qd);
    orc_icarus_linear(c, b, l, ORC_Q, T, model, Xn, Q);
    for (int t = 0; t < T; ++t) {
        if (c->qk_norm) head_rmsnorm(Q + (size_t)t * qd, Hq, D, b->q_norm, c->rms_eps);
        orc_rope(Q + (size_t)t * qd, Hq, D, pos, c->rope_theta);
    }
    /* concat over heads: [T, Hq, D] is already [T*Hq, D]; stacked head u = t*Hq + h */
    int32_t *kv_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)T * Hq);
    for (int u = 0; u < T * Hq; ++u) kv_of[u] = (u % Hq) / g;
    float *Kc = (float *)malloc(sizeof(float) * hd * (size_t)n), *Vc = (float *)malloc(sizeof(float) * hd * (size_t)n);
    orc_gather_kv(c, pool, bt_row, n, Kc, Vc);
    double *A = (double *)malloc(sizeof(double) * (size_t)T * qd);
    orc_attention(T * Hq, D, c->n_kv_heads, kv_of, Q, Kc, Vc, n, A);
    /* split back to rows, output projection, residual */
    double *Z = (double *)malloc(sizeof(double) * (size_t)T * d);
    orc_icarus_linear(c, b, l, ORC_O, T, model, A, Z);
    for (size_t i = 0; i < (size_t)T * d; ++i) Z[i] += X[i];
    /* FFN: up -> act -> down, each an ICaRusLinear; SwiGLU; residual */
    double *Zn = (double *)malloc(sizeof(double) * (size_t)T * d);
    for (int t = 0; t < T; ++t) orc_rmsnorm(Z + (size_t)t * d, b->norm_ffn, c->rms_eps, d, Zn + (size_t)t * d);
    double *G = (double *)malloc(sizeof(double) * (size_t)T * F), *U = (double *)malloc(sizeof(double) * (size_t)T * F);
    orc_icarus_linear(c, b, l, ORC_GATE, T, model, Zn, G);
    orc_icarus_linear(c, b, l, ORC_UP, T, model, Zn, U);
    for (size_t i = 0; i < (size_t)T * F; ++i) G[i] = silu(G[i]) * U[i];
    orc_icarus_linear(c, b, l, ORC_DOWN, T, model, G, Y);
    for (size_t i = 0; i < (size_t)T * d; ++i) Y[i] += Z[i];
    free(Q); free(kv_of); free(Kc); free(Vc); free(A); free(Z); free(Zn); free(G); free(U);
}

/* ---- decode (Alg. 3, one layer) ---------------------------------------- */

/* Rows are grouped by sequence, the encoder row (model -1) first in each group.
 * ctx_lens[s] = tokens cached before this step = position of the token decoded.
 * sequential == 0: the stacked pass of Alg. 3 (all rows of a sequence together).
 * sequential != 0: logical encoder first (Eq. 4), then each logical decoder on
 *                  its own (Eq. 5) -- the unoptimised order Sec. 3.3 starts from.
 * x_out is double; rounded to the storage precision. Returns 0, or -1 on a
 * malformed row list. */
int orc_decode_step(const orc_config *c, const orc_base *b, const orc_lora *l, float *pool,
                    const int32_t *block_tables, int max_blocks, int S, const int32_t *ctx_lens,
                    int R, const int32_t *row_seq, const int32_t *row_model, const float *x_in,
                    double *x_out, int64_t *slot_out, int sequential) {
    int d = c->d_model;
    int r = 0;
    for (int s = 0; s < S; ++s) {
        if (r >= R || row_seq[r] != s || row_model[r] != -1) return -1;
        int r0 = r, T = 1;
        while (r0 + T < R && row_seq[r0 + T] == s) { if (row_model[r0 + T] < 0) return -1; ++T; }
        r = r0 + T;
        int pos = ctx_lens[s];
        const int32_t *bt_row = block_tables + (size_t)s * max_blocks;
        double *X = (double *)malloc(sizeof(double) * (size_t)T * d);
        double *Xn = (double *)malloc(sizeof(double) * (size_t)T * d);
        double *Y = (double *)malloc(sizeof(double) * (size_t)T * d);
        for (size_t i = 0; i < (size_t)T * d; ++i) X[i] = (double)x_in[(size_t)r0 * d + i];
        for (int t = 0; t < T; ++t) orc_rmsnorm(X + (size_t)t * d, b->norm_attn, c->rms_eps, d, Xn + (size_t)t * d);
        /* the encoder row, base weights only, is the sole writer of the cache */
        int64_t slot = encoder_kv_step(c, b, pool, bt_row, pos, Xn);
        if (slot_out) slot_out[s] = slot;
        if (!sequential) {
            stack_after_append(c, b, l, pool, bt_row, pos, T, row_model + r0, X, Xn, Y);
        } else {
            for (int t = 0; t < T; ++t)
                stack_after_append(c, b, l, pool, bt_row, pos, 1, row_model + r0 + t,
                                   X + (size_t)t * d, Xn + (size_t)t * d, Y + (size_t)t * d);
        }
        for (size_t i = 0; i < (size_t)T * d; ++i) x_out[(size_t)r0 * d + i] = round_store(c, Y[i]);
        free(X); free(Xn); free(Y);
    }
    return r == R ? 0 : -1;
}

/* ---- prefill (Alg. 1, one layer, chunk over an existing prefix) --------- */

/* Logical encoder only.  Sequence s appends chunk_lens[s] rows at positions
 * ctx_lens[s] .. ctx_lens[s] + chunk_lens[s] - 1; the row at chunk offset i
 * attends to cache positions 0 .. ctx_lens[s] + i.  K/V of the whole chunk are
 * written first.  select [sum T] (may be NULL = all): rows whose x_out is
 * computed; other rows of x_out are left untouched.  slot_out [sum T] or NULL. */
int orc_prefill(const orc_config *c, const orc_base *b, float *pool, const int32_t *block_tables,
                int max_blocks, int S, const int32_t *ctx_lens, const int32_t *chunk_lens,
                const float *x_in, double *x_out, const uint8_t *select, int64_t *slot_out) {
    int d = c->d_model;
    size_t row0 = 0;
    int32_t enc = -1;
    for (int s = 0; s < S; ++s) {
        int L = ctx_lens[s], T = chunk_lens[s];
        const int32_t *bt_row = block_tables + (size_t)s * max_blocks;
        double *X = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * d);
        double *Xn = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * d);
        for (size_t i = 0; i < (size_t)T * d; ++i) X[i] = (double)x_in[row0 * d + i];
        for (int t = 0; t < T; ++t) {
            orc_rmsnorm(X + (size_t)t * d, b->norm_attn, c->rms_eps, d, Xn + (size_t)t * d);
            int64_t slot = encoder_kv_step(c, b, pool, bt_row, L + t, Xn + (size_t)t * d);
            if (slot_out) slot_out[row0 + t] = slot;
        }
        if (x_out) {
            double *Y = (double *)malloc(sizeof(double) * (size_t)d);
            for (int t = 0; t < T; ++t) {
                if (select && !select[row0 + t]) continue;
                stack_after_append(c, b, NULL, pool, bt_row, L + t, 1, &enc,
                                   X + (size_t)t * d, Xn + (size_t)t * d, Y);
                for (int i = 0; i < d; ++i) x_out[(row0 + t) * d + i] = round_store(c, Y[i]);
            }
            free(Y);
        }
        free(X); free(Xn);
        row0 += (size_t)T;
    }
    return 0;
}

/* ---- layer stack: final norm, LM head, greedy token ------------------------
 * The outer loop of Alg. 3 (and the last lines of Alg. 1): after the last layer the
 * hidden row goes through the final RMSNorm (base weight) and the LM head; greedy
 * sampling takes the first index of the largest logit.
 * x [R, d] (double, already rounded to storage by the last layer), logits [R, vocab]. */
void orc_lm_head(const double *x, int R, int d, const float *w_norm, double eps, const float *W_lm, int vocab,
                 double *logits, int32_t *tokens) {
    double *xn = (double *)malloc(sizeof(double) * (size_t)d);
    for (int r = 0; r < R; ++r) {
        orc_rmsnorm(x + (size_t)r * d, w_norm, eps, d, xn);
        double *lg = logits + (size_t)r * vocab;
        orc_linear(W_lm, vocab, d, xn, lg);
        int best = 0;
        for (int v = 1; v < vocab; ++v)
            if (lg[v] > lg[best]) best = v;
        tokens[r] = best;
    }
    free(xn);
}

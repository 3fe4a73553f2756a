// Row-wise kernels of the decode step (bf16 storage): RMSNorm and the LoRA shrink of Alg. 2.
//
// A decoder row needs the shrink t = s * A_j x of its own model j only (r outputs, r = adapter
// rank), so with a few hundred stacked rows the shrink is a batch of small gathered mat-vecs, not a
// GEMM: one workgroup per row reads the r rows of A_j (shared through L2 by all rows of model j)
// and writes the row of T that the ICaRusLinear GEMM consumes as extra K columns -- the r values in
// the column block of model j, zeros elsewhere (encoder rows: all zeros).  Where the shrink's input
// is the output of an RMSNorm, both run in one kernel: the normalised row is rounded to bf16,
// stored, and fed to the mat-vecs as it is stored.
#include "device_util.h"
#include "kernels.h"

#include <algorithm>

namespace icarus {

namespace {

constexpr int kRowThreads = 512;  // threads per row: 8 waves share the K range of one row
constexpr int kRowMaxWorkgroups = 512;  // a row's accumulators are split over more workgroups while the launch stays below this

__device__ __forceinline__ void unpack8(uint4 v, float (&f)[8]) {
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
}

__device__ __forceinline__ uint32_t pack2(float a, float b) {
    return (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
}

// Where a row comes from.
//   SRC_PLAIN:  it is stored (x).
//   SRC_SLICES: it is still in pieces, residual + split-K partials (fp32) of the projection before it.
//   SRC_ATTN:   it is the attention output of a sequence whose cached tokens were cut into several
//               pieces: per (piece, kv-head, stacked query) an unnormalised partial output with its
//               running maximum and denominator, merged here (rows of uncut sequences are stored).
// Rows that are formed here are rounded to bf16 and stored at x, and everything downstream sees them
// as stored.
enum { SRC_PLAIN = 0, SRC_SLICES = 1, SRC_ATTN = 2 };

struct RowArgs {
    bf16_t *x; int ldx; int K;                       // the rows [R][ldx], K used columns
    const bf16_t *wn; float eps; bf16_t *y;          // NORM: y = rmsnorm(x) * wn, [R][K]
    const bf16_t *A0, *A1; int r, M;                 // adapter A of the one or two targets reading this input, [M][r][K]
    const int32_t *row_model; float scale; bf16_t *T; int ldt;  // T [R][ldt], ldt = targets * M * r
    int *zero; int n_zero;                           // small per-call counters cleared by row 0
    const float *psum; int splits; size_t slice; const bf16_t *resid;  // SRC_SLICES
    const float *part_o, *part_ml;                   // SRC_ATTN: partials [(piece, kv-head, query)][D] and [..][2]
    const int32_t *row_pseq, *seq_nparts, *seq_part0, *seq_row0; int Hq, Hkv, g_max;
};

constexpr int kHeadChunks = 16;  // 16-byte chunks per attention head (head_dim 128)

// One workgroup per row.  NACC = targets * r accumulators (0: no shrink).  The row's mat-vecs are a
// chain of dependent memory round trips if written naively (row model -> row -> norm -> adapter
// rows), so the adapter rows, which depend on the row's model only, are requested first and stay
// one group of loads ahead of the arithmetic throughout.
// SHRINK: the row has an adapter (a compile-time flag, so that every load of the main loop is unconditional:
// the compiler then knows how many younger loads are in flight when it waits for a group and leaves them in
// flight; with a load under a run-time condition it waits for everything, the group requested ahead included).
template <int SRC, bool NORM, int NACC, bool SHRINK>
__device__ __forceinline__ void row_body(const RowArgs &a, int j, float *__restrict__ red,
                                         float (*__restrict__ part)[NACC > 0 ? NACC : 1], float *__restrict__ res) {
    constexpr int NA = NACC > 0 ? NACC : 1;
    constexpr int GRP = (NA == 16 || NA == 32) ? 4 : (NA >= 8 ? 8 : NA);  // adapter rows per group of loads (two groups in flight)
    constexpr int NG = NA / GRP;              // groups per chunk: 1, 2, 4 or 8
    constexpr int U = NG < 2 ? 2 : NG;        // steps per unrolled round (two load buffers)
    constexpr bool FIRST_PASS = NORM || SRC != SRC_PLAIN;
    constexpr bool shrink = SHRINK;
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    // blockIdx.y: which NACC of the row's targets * r accumulators this workgroup computes.  Every part forms the
    // row with the same arithmetic in the same order and stores it (the same bytes from every part: a thread
    // reads back chunks it stored itself, never another workgroup's).
    const int part_id = blockIdx.y, acc0 = part_id * NA;
    const bool owner = part_id == 0;
    const int K = a.K, n_chunks = K >> 3;
    const int mr = a.M * a.r;
    if (!shrink && !owner) {  // a row without adapter: the other parts only clear their share of its row of T
        if (NACC > 0)
            for (int c = tid; c < a.ldt; c += kRowThreads)
                if (((c / mr) * a.r + c % a.r) / NA == part_id) a.T[(size_t)row * a.ldt + c] = 0;
        return;
    }
    if (row == 0 && owner)
        for (int i = tid; i < a.n_zero; i += kRowThreads) a.zero[i] = 0;
    bf16_t *xr = a.x + (size_t)row * a.ldx;
    const bf16_t *pA0 = a.A0 + (size_t)(shrink ? j : 0) * a.r * K;
    const bf16_t *pA1 = a.A1 ? a.A1 + (size_t)(shrink ? j : 0) * a.r * K : pA0;
    const int my_chunks = tid < n_chunks ? (n_chunks - tid + kRowThreads - 1) / kRowThreads : 0;
    const int n_steps = my_chunks * NG;  // step t: chunk t / NG of this thread, adapter rows (t % NG) * GRP ...

    uint4 av[2][GRP], xb[2], wb[2];
    // a step past this thread's last one repeats the row's last chunk and its data is dropped
    auto issue = [&](int t, int gi, int b) {
        const int c = min(tid + (t / NG) * kRowThreads, n_chunks - 1);
        if (gi == 0) {
            if (t > 0 || !FIRST_PASS) xb[b] = *(const uint4 *)(xr + c * 8);  // chunk 0 stays in registers after the first pass
            if (NORM) wb[b] = *(const uint4 *)(a.wn + c * 8);
        }
        if (shrink) {
#pragma unroll
            for (int q = 0; q < GRP; ++q) {
                const int ai = acc0 + gi * GRP + q;
                av[b][q] = *(const uint4 *)((ai < a.r ? pA0 + (size_t)ai * K : pA1 + (size_t)(ai - a.r) * K) + c * 8);
            }
        }
    };
    issue(0, 0, 0);

    // first pass: form the row (and store it), sum of squares
    float f0[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, inv = 1.f;
    if (FIRST_PASS) {
        float ss = 0.f;
        int np = 1, p0 = 0, jq0 = 0, g = 1;
        if (SRC == SRC_ATTN) {
            const int s = a.row_pseq[row];
            np = a.seq_nparts[s]; p0 = a.seq_part0[s]; g = a.Hq / a.Hkv;
            jq0 = (row - a.seq_row0[s]) * g;
        }
        for (int ci = 0; ci < my_chunks; ++ci) {
            const int c = tid + ci * kRowThreads;
            float f[8];
            bool formed = false;
            if (SRC == SRC_SLICES) {
                unpack8(*(const uint4 *)(a.resid + (size_t)row * K + c * 8), f);
                const float *pp = a.psum + (size_t)row * K + c * 8;
                int z = 0;
                for (; z + 4 <= a.splits; z += 4) {  // four slices in flight
                    float4 v[8];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        v[2 * q] = *(const float4 *)(pp + (z + q) * a.slice);
                        v[2 * q + 1] = *(const float4 *)(pp + (z + q) * a.slice + 4);
                    }
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        f[0] += v[2 * q].x; f[1] += v[2 * q].y; f[2] += v[2 * q].z; f[3] += v[2 * q].w;
                        f[4] += v[2 * q + 1].x; f[5] += v[2 * q + 1].y; f[6] += v[2 * q + 1].z; f[7] += v[2 * q + 1].w;
                    }
                }
                for (; z < a.splits; ++z) {
                    const float4 v0 = *(const float4 *)(pp + z * a.slice), v1 = *(const float4 *)(pp + z * a.slice + 4);
                    f[0] += v0.x; f[1] += v0.y; f[2] += v0.z; f[3] += v0.w;
                    f[4] += v1.x; f[5] += v1.y; f[6] += v1.z; f[7] += v1.w;
                }
                formed = true;
            } else if (SRC == SRC_ATTN && np > 1) {
                const int h = c / kHeadChunks, d0 = (c % kHeadChunks) * 8;
                const size_t pj0 = ((size_t)p0 * a.Hkv + h / g) * a.g_max + jq0 + h % g;
                const size_t pstep = (size_t)a.Hkv * a.g_max;  // between consecutive pieces
                // four pieces' loads in flight at a time (a piece past the last repeats it with weight zero)
                float mx = -INFINITY;
                for (int p = 0; p < np; p += 4) {
                    float m4[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) m4[u] = a.part_ml[(pj0 + min(p + u, np - 1) * pstep) * 2];
#pragma unroll
                    for (int u = 0; u < 4; ++u) mx = fmaxf(mx, m4[u]);
                }
                float den = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) f[e] = 0.f;
                for (int p = 0; p < np; p += 4) {
                    float2 ml[4];
                    float4 v0[4], v1[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const size_t pj = pj0 + min(p + u, np - 1) * pstep;
                        ml[u] = *(const float2 *)(a.part_ml + pj * 2);
                        v0[u] = *(const float4 *)(a.part_o + pj * (kHeadChunks * 8) + d0);
                        v1[u] = *(const float4 *)(a.part_o + pj * (kHeadChunks * 8) + d0 + 4);
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {  // in piece order, as a loop over single pieces would add them
                        const float wgt = p + u < np ? __builtin_amdgcn_exp2f(ml[u].x - mx) : 0.f;
                        den += wgt * ml[u].y;
                        f[0] += wgt * v0[u].x; f[1] += wgt * v0[u].y; f[2] += wgt * v0[u].z; f[3] += wgt * v0[u].w;
                        f[4] += wgt * v1[u].x; f[5] += wgt * v1[u].y; f[6] += wgt * v1[u].z; f[7] += wgt * v1[u].w;
                    }
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) f[e] = f[e] / den;
                formed = true;
            }
            if (formed) {
                uint4 o;
                o.x = pack2(f[0], f[1]); o.y = pack2(f[2], f[3]); o.z = pack2(f[4], f[5]); o.w = pack2(f[6], f[7]);
                *(uint4 *)(xr + c * 8) = o;
                unpack8(o, f);
            } else {
                unpack8(*(const uint4 *)(xr + c * 8), f);
            }
            if (NORM) {
#pragma unroll
                for (int e = 0; e < 8; ++e) ss += f[e] * f[e];
            }
            if (ci == 0) {
#pragma unroll
                for (int e = 0; e < 8; ++e) f0[e] = f[e];
            }
        }
        if (NORM) {
            ss = block_sum(ss, red);
            inv = rsqrtf(ss / (float)K + a.eps);
        }
    }
    if (!NORM && NACC == 0) return;

    // second pass: normalise and store, multiply with the adapter rows
    float acc[NA];
#pragma unroll
    for (int q = 0; q < NA; ++q) acc[q] = 0.f;
    float f[8];
    for (int t0 = 0; t0 < n_steps; t0 += U) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u, gi = u % NG, b = u & 1;
            if (t < n_steps) {
                issue(t + 1, (u + 1) % NG, (u + 1) & 1);
                if (gi == 0) {
                    const int c = tid + (t / NG) * kRowThreads;
                    if (FIRST_PASS && t == 0) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) f[e] = f0[e];
                    } else {
                        unpack8(xb[b], f);
                    }
                    if (NORM) {
                        float wf[8];
                        unpack8(wb[b], wf);
                        uint4 o;
                        o.x = pack2(f[0] * inv * wf[0], f[1] * inv * wf[1]);
                        o.y = pack2(f[2] * inv * wf[2], f[3] * inv * wf[3]);
                        o.z = pack2(f[4] * inv * wf[4], f[5] * inv * wf[5]);
                        o.w = pack2(f[6] * inv * wf[6], f[7] * inv * wf[7]);
                        *(uint4 *)(a.y + (size_t)row * K + c * 8) = o;
                        unpack8(o, f);  // the shrink sees the row as stored
                    }
                }
                if (shrink) {
#pragma unroll
                    for (int q = 0; q < GRP; ++q) {
                        float af[8];
                        unpack8(av[b][q], af);
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[gi * GRP + q] += f[e] * af[e];
                    }
                }
            }
        }
    }
    if (NACC == 0) return;
    if (shrink) {
#pragma unroll
        for (int q = 0; q < NA; ++q) {
            float s = wave_sum(acc[q]);
            if (lane == 0) part[wv][q] = s;
        }
        __syncthreads();
        if (tid < NA) {
            float v = 0.f;
#pragma unroll
            for (int q = 0; q < kRowThreads / 64; ++q) v += part[q][tid];
            res[tid] = v * a.scale;
        }
        __syncthreads();
    }
    // the row of T: entry (target t, model jj, i) belongs to the part that holds accumulator t * r + i
    for (int c = tid; c < a.ldt; c += kRowThreads) {
        const int t = c / mr, jj = (c % mr) / a.r, i = c % a.r, ai = t * a.r + i - acc0;
        if (ai >= 0 && ai < NA) a.T[(size_t)row * a.ldt + c] = f32_to_bf16(shrink && jj == j ? res[ai] : 0.f);
    }
}

template <int SRC, bool NORM, int NACC>
__global__ void __launch_bounds__(kRowThreads, NACC == 64 ? 2 : 4) k_row(RowArgs a) {  // four waves per SIMD = two rows per CU, where the registers allow
    constexpr int NA = NACC > 0 ? NACC : 1;
    __shared__ float red[16];
    __shared__ float part[kRowThreads / 64][NA];
    __shared__ float res[NA];
    const int j = NACC > 0 ? a.row_model[blockIdx.x] : -1;  // uniform over the workgroup
    if (NACC > 0 && j >= 0) row_body<SRC, NORM, NACC, true>(a, j, red, part, res);
    else row_body<SRC, NORM, NACC, false>(a, j, red, part, res);
}

// nacc: the row's accumulators (targets * r).  With few rows they are split over several workgroups per row
// (each computes 8 or more of them against its share of the adapter rows and forms the row for itself), so
// that a handful of rows still spreads over the chip and a thread's chain of dependent load groups gets shorter.
template <int SRC, bool NORM>
hipError_t launch_row(int nacc, int R, hipStream_t st, const RowArgs &a) {
    int parts = 1;
    while (nacc / (2 * parts) >= 8 && R * 2 * parts <= kRowMaxWorkgroups) parts *= 2;
    nacc /= parts;
#define ICARUS_ROW(N) hipLaunchKernelGGL((k_row<SRC, NORM, N>), dim3(R, parts), dim3(kRowThreads), 0, st, a)
    switch (nacc) {
    case 0: ICARUS_ROW(0); break;
    case 8: ICARUS_ROW(8); break;
    case 16: ICARUS_ROW(16); break;
    case 32: ICARUS_ROW(32); break;
    case 64: ICARUS_ROW(64); break;
    default: return hipErrorInvalidValue;
    }
#undef ICARUS_ROW
    return hipGetLastError();
}

RowArgs shrink_args(const Dims &dm, const void *A0, const void *A1, const int32_t *row_model, void *T) {
    RowArgs a{};
    int targets = A0 ? (A1 ? 2 : 1) : 0;
    a.A0 = (const bf16_t *)A0; a.A1 = (const bf16_t *)A1; a.r = dm.r; a.M = dm.M; a.row_model = row_model;
    a.scale = dm.lora_scale; a.T = (bf16_t *)T; a.ldt = targets * dm.M * dm.r;
    return a;
}

}  // namespace

bool row_shrink_supported(int r, int targets) {
    int n = r * targets;
    return n == 8 || n == 16 || n == 32 || n == 64;
}

hipError_t launch_norm_shrink(const Dims &dm, const void *x, const void *wn, void *y, int R, int K, const void *A0, const void *A1,
                              const int32_t *row_model, void *T, int *zero, int n_zero, hipStream_t st) {
    if (R <= 0) return hipSuccess;
    RowArgs a = shrink_args(dm, A0, A1, row_model, T);
    a.x = (bf16_t *)x; a.ldx = K; a.K = K; a.wn = (const bf16_t *)wn; a.eps = dm.eps; a.y = (bf16_t *)y;
    a.zero = zero; a.n_zero = n_zero;
    return launch_row<SRC_PLAIN, true>(a.ldt / std::max(1, dm.M), R, st, a);
}

hipError_t launch_sum_norm_shrink(const Dims &dm, const float *part, int splits, size_t slice, const void *resid, void *xsum,
                                  const void *wn, void *y, int R, int K, const void *A0, const void *A1, const int32_t *row_model,
                                  void *T, hipStream_t st) {
    if (R <= 0) return hipSuccess;
    RowArgs a = shrink_args(dm, A0, A1, row_model, T);
    a.x = (bf16_t *)xsum; a.ldx = K; a.K = K; a.wn = (const bf16_t *)wn; a.eps = dm.eps; a.y = (bf16_t *)y;
    a.psum = part; a.splits = splits; a.slice = slice; a.resid = (const bf16_t *)resid;
    return launch_row<SRC_SLICES, true>(a.ldt / std::max(1, dm.M), R, st, a);
}

hipError_t launch_row_shrink(const Dims &dm, const void *x, int ldx, int R, int K, const void *A0, const int32_t *row_model, void *T,
                             hipStream_t st) {
    if (R <= 0) return hipSuccess;
    RowArgs a = shrink_args(dm, A0, nullptr, row_model, T);
    a.x = (bf16_t *)x; a.ldx = ldx; a.K = K;
    return launch_row<SRC_PLAIN, false>(dm.r, R, st, a);
}

hipError_t launch_merge_shrink(const Dims &dm, const float *part_o, const float *part_ml, const AttnPlan &pl, const int32_t *row_pseq,
                               void *attn, int R, const void *A0, const int32_t *row_model, void *T, hipStream_t st) {
    if (R <= 0) return hipSuccess;
    if (dm.D != kHeadChunks * 8) return hipErrorInvalidValue;
    RowArgs a = shrink_args(dm, A0, nullptr, row_model, T);
    a.x = (bf16_t *)attn; a.ldx = dm.Hq * dm.D; a.K = dm.Hq * dm.D;
    a.part_o = part_o; a.part_ml = part_ml; a.row_pseq = row_pseq; a.seq_nparts = pl.seq_nparts; a.seq_part0 = pl.seq_part0;
    a.seq_row0 = pl.seq_row0; a.Hq = dm.Hq; a.Hkv = dm.Hkv; a.g_max = pl.g_max;
    return launch_row<SRC_ATTN, false>(A0 ? dm.r : 0, R, st, a);
}

}  // namespace icarus

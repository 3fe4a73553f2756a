// Small kernels around the layer stack (Alg. 3 outer loop): token embedding lookup, greedy
// sampling (first index of the largest logit), row gathers.  Index work; fp32 compares only.
#include "device_util.h"
#include "kernels.h"

namespace icarus {

namespace {

// x[row, :] = embed[token_of(row), :], token_of(row) = tok[idx ? idx[row] : row]; 16 bytes per thread step
__global__ void __launch_bounds__(256) k_embed_rows(const uint4 *__restrict__ embed, const int32_t *__restrict__ tok,
                                                    const int32_t *__restrict__ idx, uint4 *__restrict__ x, int row_vec) {
    const int row = blockIdx.x;
    const int t = tok[idx ? idx[row] : row];
    const uint4 *src = embed + (size_t)t * row_vec;
    uint4 *dst = x + (size_t)row * row_vec;
    for (int i = threadIdx.x; i < row_vec; i += 256) dst[i] = src[i];
}

// out[i, :] = x[rows[i], :]
__global__ void __launch_bounds__(256) k_gather_rows(const uint4 *__restrict__ x, const int32_t *__restrict__ rows,
                                                     uint4 *__restrict__ out, int row_vec) {
    const uint4 *src = x + (size_t)rows[blockIdx.x] * row_vec;
    uint4 *dst = out + (size_t)blockIdx.x * row_vec;
    for (int i = threadIdx.x; i < row_vec; i += 256) dst[i] = src[i];
}

// token[row] = first index of the largest of logits[row, 0..V), in two stages so that a few rows of a large
// vocabulary still fill the chip: kArgmaxParts workgroups per row leave (value, index) partials, one wave per row
// picks among them.  Lower index wins among equal values; within a thread the scan ascends and '>' keeps the first.
constexpr int kArgmaxParts = 32;

__device__ __forceinline__ void argmax_merge(float &best, int &bi, float ov, int oi) {
    if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
}

__global__ void __launch_bounds__(256) k_argmax_part(const float *__restrict__ logits, int V, float *__restrict__ pv,
                                                     int32_t *__restrict__ pi) {
    __shared__ float sv[4];
    __shared__ int si[4];
    const int row = blockIdx.x / kArgmaxParts, part = blockIdx.x % kArgmaxParts;
    const int chunk = (V + kArgmaxParts - 1) / kArgmaxParts;
    const int lo = part * chunk, hi = min(V, lo + chunk);
    const float *lg = logits + (size_t)row * V;
    float best = -INFINITY;
    int bi = 0x7fffffff;  // an empty part keeps this index and loses every comparison
#pragma unroll 4
    for (int i = lo + threadIdx.x; i < hi; i += 256) {
        float v = lg[i];
        if (v > best || bi == 0x7fffffff) { best = v; bi = i; }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) argmax_merge(best, bi, __shfl_xor(best, o, 64), __shfl_xor(bi, o, 64));
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (lane == 0) { sv[w] = best; si[w] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int k = 1; k < 4; ++k) argmax_merge(best, bi, sv[k], si[k]);
        pv[blockIdx.x] = best;
        pi[blockIdx.x] = bi;
    }
}

__global__ void __launch_bounds__(64) k_argmax_pick(const float *__restrict__ pv, const int32_t *__restrict__ pi,
                                                    int32_t *__restrict__ token) {
    static_assert(kArgmaxParts <= 64, "one wave picks among a row's partials");
    const int lane = threadIdx.x;
    float best = lane < kArgmaxParts ? pv[blockIdx.x * kArgmaxParts + lane] : -INFINITY;
    int bi = lane < kArgmaxParts ? pi[blockIdx.x * kArgmaxParts + lane] : 0x7fffffff;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) argmax_merge(best, bi, __shfl_xor(best, o, 64), __shfl_xor(bi, o, 64));
    if (lane == 0) token[blockIdx.x] = bi;
}

// seq_next[s] = row_next[last_row[s]]
__global__ void k_pick_rows(const int32_t *__restrict__ row_next, const int32_t *__restrict__ last_row,
                            int32_t *__restrict__ seq_next, int S) {
    int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s < S) seq_next[s] = row_next[last_row[s]];
}

}  // namespace

hipError_t launch_embed_rows(const void *embed, const int32_t *tok, const int32_t *idx, void *x, int R, int row_bytes, hipStream_t st) {
    if (R <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_embed_rows, dim3(R), dim3(256), 0, st, (const uint4 *)embed, tok, idx, (uint4 *)x, row_bytes / 16);
    return hipGetLastError();
}

hipError_t launch_gather_rows(const void *x, const int32_t *rows, void *out, int n, int row_bytes, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_gather_rows, dim3(n), dim3(256), 0, st, (const uint4 *)x, rows, (uint4 *)out, row_bytes / 16);
    return hipGetLastError();
}

size_t argmax_scratch_bytes(int R) { return (size_t)R * kArgmaxParts * 8; }

hipError_t launch_argmax(const float *logits, int R, int V, int32_t *token, void *scratch, hipStream_t st) {
    if (R <= 0) return hipSuccess;
    float *pv = (float *)scratch;
    int32_t *pi = (int32_t *)(pv + (size_t)R * kArgmaxParts);
    hipLaunchKernelGGL(k_argmax_part, dim3(R * kArgmaxParts), dim3(256), 0, st, logits, V, pv, pi);
    hipLaunchKernelGGL(k_argmax_pick, dim3(R), dim3(64), 0, st, pv, pi, token);
    return hipGetLastError();
}

hipError_t launch_pick_rows(const int32_t *row_next, const int32_t *last_row, int32_t *seq_next, int S, hipStream_t st) {
    if (S <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_pick_rows, dim3((S + 255) / 256), dim3(256), 0, st, row_next, last_row, seq_next, S);
    return hipGetLastError();
}

}  // namespace icarus

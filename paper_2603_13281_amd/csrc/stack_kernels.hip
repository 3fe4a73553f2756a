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

// token[row] = first index of the largest of logits[row, 0..V)
__global__ void __launch_bounds__(1024) k_argmax(const float *__restrict__ logits, int V, int32_t *__restrict__ token) {
    __shared__ float sv[16];
    __shared__ int si[16];
    const float *lg = logits + (size_t)blockIdx.x * V;
    float best = -INFINITY;
    int bi = 0x7fffffff;
    for (int i = threadIdx.x; i < V; i += 1024) {  // ascending i per thread: '>' keeps the first maximum
        float v = lg[i];
        if (v > best || bi == 0x7fffffff) { best = v; bi = i; }
    }
    // lower index wins among equal values
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        float ov = __shfl_xor(best, o, 64);
        int oi = __shfl_xor(bi, o, 64);
        if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
    }
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (lane == 0) { sv[w] = best; si[w] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int k = 1; k < 16; ++k)
            if (sv[k] > best || (sv[k] == best && si[k] < bi)) { best = sv[k]; bi = si[k]; }
        token[blockIdx.x] = bi;
    }
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

hipError_t launch_argmax(const float *logits, int R, int V, int32_t *token, hipStream_t st) {
    if (R <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_argmax, dim3(R), dim3(1024), 0, st, logits, V, token);
    return hipGetLastError();
}

hipError_t launch_pick_rows(const int32_t *row_next, const int32_t *last_row, int32_t *seq_next, int S, hipStream_t st) {
    if (S <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_pick_rows, dim3((S + 255) / 256), dim3(256), 0, st, row_next, last_row, seq_next, S);
    return hipGetLastError();
}

}  // namespace icarus

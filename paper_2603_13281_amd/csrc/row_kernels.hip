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

namespace icarus {

namespace {

constexpr int kRowThreads = 512;  // threads per row: 8 waves share the K range of one row

__device__ __forceinline__ void unpack8(uint4 v, float (&f)[8]) {
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
}

__device__ __forceinline__ uint32_t pack2(float a, float b) {
    return (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
}

// NORM: y[row] = rmsnorm(x[row]) * wn (bf16), and the shrink reads y; else the shrink reads x.
// NACC = targets * r accumulators per row (0: no shrink).  A0/A1: adapter A of the one or two
// targets that share this input, each [M][r][K].  T: [R][ldt], ldt = targets * M * r.
template <bool NORM, int NACC>
__global__ void __launch_bounds__(kRowThreads) k_norm_shrink(const bf16_t *__restrict__ x, int ldx, int K, const bf16_t *__restrict__ wn,
                                                     float eps, bf16_t *__restrict__ y, const bf16_t *__restrict__ A0,
                                                     const bf16_t *__restrict__ A1, int r, int M, const int32_t *__restrict__ row_model,
                                                     float scale, bf16_t *__restrict__ T, int ldt, int *__restrict__ zero, int n_zero,
                                                     const float *__restrict__ psum, int splits, size_t slice,
                                                     const bf16_t *__restrict__ resid, bf16_t *__restrict__ xsum) {
    __shared__ float red[16];
    __shared__ float part[kRowThreads / 64][NACC > 0 ? NACC : 1];
    __shared__ float res[NACC > 0 ? NACC : 1];
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int n_chunks = K >> 3;
    const bf16_t *xr = x + (size_t)row * ldx;
    if (row == 0)  // the layer's first kernel also clears small per-call counters
        for (int i = tid; i < n_zero; i += kRowThreads) zero[i] = 0;
    float inv = 1.f;
    if (NORM) {
        float ss = 0.f;
        for (int c = tid; c < n_chunks; c += kRowThreads) {
            float f[8];
            if (psum) {
                // the row is still in pieces: residual + split-K partials of the projection before the
                // norm.  Sum them, round to storage, keep (xsum is x): each thread re-reads below
                // only the chunks it wrote itself.
                unpack8(*(const uint4 *)(resid + (size_t)row * K + c * 8), f);
                for (int z = 0; z < splits; ++z) {
                    const float *pp = psum + z * slice + (size_t)row * K + c * 8;
                    const float4 p0 = *(const float4 *)pp, p1 = *(const float4 *)(pp + 4);
                    f[0] += p0.x; f[1] += p0.y; f[2] += p0.z; f[3] += p0.w;
                    f[4] += p1.x; f[5] += p1.y; f[6] += p1.z; f[7] += p1.w;
                }
                uint4 o;
                o.x = pack2(f[0], f[1]); o.y = pack2(f[2], f[3]); o.z = pack2(f[4], f[5]); o.w = pack2(f[6], f[7]);
                *(uint4 *)(xsum + (size_t)row * K + c * 8) = o;
                unpack8(o, f);
            } else {
                unpack8(*(const uint4 *)(xr + c * 8), f);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += f[e] * f[e];
        }
        ss = block_sum(ss, red);
        inv = rsqrtf(ss / (float)K + eps);
    }
    const int j = NACC > 0 ? row_model[row] : -1;
    float acc[NACC > 0 ? NACC : 1];
#pragma unroll
    for (int a = 0; a < (NACC > 0 ? NACC : 1); ++a) acc[a] = 0.f;
    for (int c = tid; c < n_chunks; c += kRowThreads) {
        float f[8];
        unpack8(*(const uint4 *)(xr + c * 8), f);
        if (NORM) {
            float wf[8];
            unpack8(*(const uint4 *)(wn + c * 8), wf);
            uint4 o;
            o.x = pack2(f[0] * inv * wf[0], f[1] * inv * wf[1]);
            o.y = pack2(f[2] * inv * wf[2], f[3] * inv * wf[3]);
            o.z = pack2(f[4] * inv * wf[4], f[5] * inv * wf[5]);
            o.w = pack2(f[6] * inv * wf[6], f[7] * inv * wf[7]);
            *(uint4 *)(y + (size_t)row * K + c * 8) = o;
            unpack8(o, f);  // the shrink sees the row as stored
        }
        if (NACC > 0 && j >= 0) {
            const bf16_t *p0 = A0 + ((size_t)j * r) * K + c * 8;
            const bf16_t *p1 = A1 ? A1 + ((size_t)j * r) * K + c * 8 : p0;
            constexpr int GRP = NACC < 16 ? (NACC > 0 ? NACC : 1) : 16;  // loads in flight per thread
#pragma unroll
            for (int a0 = 0; a0 < NACC; a0 += GRP) {
                uint4 av[GRP];
#pragma unroll
                for (int a = 0; a < GRP; ++a)
                    av[a] = *(const uint4 *)(a0 + a < r ? p0 + (size_t)(a0 + a) * K : p1 + (size_t)(a0 + a - r) * K);
#pragma unroll
                for (int a = 0; a < GRP; ++a) {
                    float af[8];
                    unpack8(av[a], af);
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[a0 + a] += f[e] * af[e];
                }
            }
        }
    }
    if (NACC == 0) return;
    if (j >= 0) {  // uniform over the workgroup
#pragma unroll
        for (int a = 0; a < NACC; ++a) {
            float s = wave_sum(acc[a]);
            if (lane == 0) part[wv][a] = s;
        }
        __syncthreads();
        if (tid < NACC) {
            float v = 0.f;
#pragma unroll
            for (int q = 0; q < kRowThreads / 64; ++q) v += part[q][tid];
            res[tid] = v * scale;
        }
        __syncthreads();
    }
    const int mr = M * r;
    for (int c = tid; c < ldt; c += kRowThreads) {
        int t = c / mr, jj = (c % mr) / r, i = c % r;
        T[(size_t)row * ldt + c] = f32_to_bf16(jj == j ? res[t * r + i] : 0.f);
    }
}

template <bool NORM>
hipError_t launch_ns(int nacc, int R, hipStream_t st, const bf16_t *x, int ldx, int K, const bf16_t *wn, float eps, bf16_t *y,
                     const bf16_t *A0, const bf16_t *A1, int r, int M, const int32_t *row_model, float scale, bf16_t *T, int ldt,
                     int *zero, int n_zero, const float *part = nullptr, int splits = 0, size_t slice = 0,
                     const bf16_t *resid = nullptr, bf16_t *xsum = nullptr) {
#define ICARUS_NS(N)                                                                                                          \
    hipLaunchKernelGGL((k_norm_shrink<NORM, N>), dim3(R), dim3(kRowThreads), 0, st, x, ldx, K, wn, eps, y, A0, A1, r, M, row_model, \
                       scale, T, ldt, zero, n_zero, part, splits, slice, resid, xsum)
    switch (nacc) {
    case 0: ICARUS_NS(0); break;
    case 8: ICARUS_NS(8); break;
    case 16: ICARUS_NS(16); break;
    case 32: ICARUS_NS(32); break;
    case 64: ICARUS_NS(64); break;
    default: return hipErrorInvalidValue;
    }
#undef ICARUS_NS
    return hipGetLastError();
}

}  // namespace

bool row_shrink_supported(int r, int targets) {
    int n = r * targets;
    return n == 8 || n == 16 || n == 32 || n == 64;
}

hipError_t launch_norm_shrink(const Dims &dm, const void *x, const void *wn, void *y, int R, int K, const void *A0, const void *A1,
                              const int32_t *row_model, void *T, int *zero, int n_zero, hipStream_t st) {
    if (R <= 0) return hipSuccess;
    int targets = A0 ? (A1 ? 2 : 1) : 0;
    return launch_ns<true>(targets * dm.r, R, st, (const bf16_t *)x, K, K, (const bf16_t *)wn, dm.eps, (bf16_t *)y, (const bf16_t *)A0,
                           (const bf16_t *)A1, dm.r, dm.M, row_model, dm.lora_scale, (bf16_t *)T, targets * dm.M * dm.r, zero, n_zero);
}

hipError_t launch_sum_norm_shrink(const Dims &dm, const float *part, int splits, size_t slice, const void *resid, void *xsum,
                                  const void *wn, void *y, int R, int K, const void *A0, const void *A1, const int32_t *row_model,
                                  void *T, hipStream_t st) {
    if (R <= 0) return hipSuccess;
    int targets = A0 ? (A1 ? 2 : 1) : 0;
    return launch_ns<true>(targets * dm.r, R, st, (const bf16_t *)xsum, K, K, (const bf16_t *)wn, dm.eps, (bf16_t *)y,
                           (const bf16_t *)A0, (const bf16_t *)A1, dm.r, dm.M, row_model, dm.lora_scale, (bf16_t *)T,
                           targets * dm.M * dm.r, nullptr, 0, part, splits, slice, (const bf16_t *)resid, (bf16_t *)xsum);
}

hipError_t launch_row_shrink(const Dims &dm, const void *x, int ldx, int R, int K, const void *A0, const int32_t *row_model, void *T,
                             hipStream_t st) {
    if (R <= 0) return hipSuccess;
    return launch_ns<false>(dm.r, R, st, (const bf16_t *)x, ldx, K, nullptr, 0.f, nullptr, (const bf16_t *)A0, nullptr, dm.r, dm.M,
                            row_model, dm.lora_scale, (bf16_t *)T, dm.M * dm.r, nullptr, 0);
}

}  // namespace icarus

// Device-side helpers shared by the gfx950 kernels: storage-type conversion and
// wave/block reductions.  Wavefronts are 64 lanes wide.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace icarus {

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
    return __uint_as_float(((uint32_t)v) << 16);
}

// float -> bfloat16, round to nearest even (NaN kept quiet).
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float ld(const float *p) { return *p; }
    static __device__ __forceinline__ void st(float *p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float ld(const bf16_t *p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void st(bf16_t *p, float v) { *p = f32_to_bf16(v); }
};

// FP8 E4M3 (OCP: largest finite value 448, no infinities) cache element.  gfx950's conversion instructions
// implement this format: decode is exact, encode rounds to nearest even and turns magnitudes of 480 and
// more into NaN, so values are clamped to +-448 first.
struct fp8_t { uint8_t v; };
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float fp8_to_f32(uint32_t code) { return __builtin_amdgcn_cvt_pk_f32_fp8(code, false)[0]; }
__device__ __forceinline__ uint32_t f32_to_fp8(float x) {
    if (!(x == x)) return 0x7fu;
    x = fminf(fmaxf(x, -448.f), 448.f);
    return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(x, 0.f, 0, false) & 0xffu;
}

// Cache element access: value = stored element (x scale for FP8 codes).
template <typename KT> struct KVElem {
    static __device__ __forceinline__ float ld(const KT *p, float) { return Elem<KT>::ld(p); }
    static __device__ __forceinline__ void st(KT *p, float v, float) { Elem<KT>::st(p, v); }
};
template <> struct KVElem<fp8_t> {
    static __device__ __forceinline__ float ld(const fp8_t *p, float scale) { return fp8_to_f32(p->v) * scale; }
    static __device__ __forceinline__ void st(fp8_t *p, float v, float scale) { p->v = (uint8_t)f32_to_fp8(v / scale); }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Block-wide reductions for blocks of up to 1024 threads; `red` is a shared float[16].
// Every thread gets the result.
__device__ __forceinline__ float block_sum(float v, float *red) {
    int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    v = wave_sum(v);
    __syncthreads();
    if (lane == 0) red[w] = v;
    __syncthreads();
    float r = 0.f;
    for (int i = 0; i < nw; ++i) r += red[i];
    return r;
}
__device__ __forceinline__ float block_max(float v, float *red) {
    int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    v = wave_max(v);
    __syncthreads();
    if (lane == 0) red[w] = v;
    __syncthreads();
    float r = red[0];
    for (int i = 1; i < nw; ++i) r = fmaxf(r, red[i]);
    return r;
}

}  // namespace icarus

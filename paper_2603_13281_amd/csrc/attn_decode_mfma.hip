// Shared-KV paged GQA decode attention on gfx950 matrix cores (bf16 storage, head_dim 128,
// block_size 16).
//
// All stacked queries of one sequence that share a kv-head -- (1 + m_s) streams x g heads --
// form the N dimension of the MFMA tiles, so each KV block is fetched from HBM once for all
// of the sequence's models.  A workgroup (4 waves) owns one kv-head of one equal share of the
// call's cached tokens and walks the share's pieces (token ranges of one sequence each) in turn.
// Per 32-token group a wave computes
//     S^T[32 tok x G]  = K[32 tok x 128] . Q^T          (A = K straight from global memory)
//     O^T[128 x G]    += V^T[128 x 32 tok] . P^T         (A = V^T straight from global memory)
// with an online softmax on the S^T accumulators.  The cache layout (K token-major, V
// transposed inside the block) makes every global load a 128-bit load that lands directly in
// MFMA operand registers: no LDS staging and no register shuffles for P.
//
// Work split inside the workgroup:
//   up to 3 query tiles (G <= 48): the four waves take the chunk's groups w, w+4, ... with all tiles;
//   4 or 5 query tiles (G <= 80):  the O^T accumulators of all tiles do not fit one wave, so waves
//     0,1 take tiles [0, NA) and waves 2,3 tiles [NA, NA+NB), each pair splitting the groups two
//     ways.  A group is then loaded by two waves; the second load is served by the caches.
//
// MFMA 16x16x32 bf16 operand layout (lane l, q = l / 16):
//   A[row l%16][k 8q..8q+7], B[k 8q..8q+7][col l%16], C[row 4q+i][col l%16] (i = 0..3).
// Token <-> tile-row mapping inside a 32-token group (two KV blocks), chosen so that the 8
// P values a lane owns after the two S^T tiles are 8 consecutive tokens of one block:
//   S^T tile t, row 4q'+i'  <->  block q'/2, token-in-block 8(q'%2) + 4t + i'
//   PV contraction index k = 8q + 4t + i  <->  block q/2, token-in-block 8(q%2) + 4t + i.
#include "device_util.h"
#include "kernels.h"

namespace icarus {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

namespace {

constexpr int kD = 128;       // head_dim
constexpr int kBk = 16;       // tokens per block
constexpr int kGrp = 32;      // tokens per wave iteration (two blocks)
constexpr int kKS = kD / 32;  // k-steps of the QK^T contraction
constexpr int kDT = kD / 16;  // d tiles of the PV product
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kSlack = 8.f;  // log2 units a score may exceed the softmax reference before it is moved
constexpr int kAttnMaxChunk = 16384;  // tokens per workgroup chunk, at most
constexpr size_t kRingBytes = (size_t)2 * 4 * 16 * 64 * 16;  // shared KV ring: 2 rounds x 4 groups x 16 KB

struct KVFrag {
    bf16x8 k[2][kKS];  // k[t][ks]: A operand of S^T tile t, k-step ks
    bf16x8 v[kDT];     // v[dt]:    A operand of O^T tile dt
};

__device__ __forceinline__ bf16x8 zero8() {
    bf16x8 z;
#pragma unroll
    for (int i = 0; i < 8; ++i) z[i] = (__bf16)0.f;
    return z;
}

// Issue the 16 loads of one 32-token group.  blk0/blk1: physical block ids (wave-uniform).
__device__ __forceinline__ void load_group(KVFrag &f, const bf16_t *__restrict__ pool, int blk0, int blk1, int c, int Hkv,
                                           int lane) {
    const int m = lane & 15, q = lane >> 4;
    const size_t head_stride = (size_t)2 * kBk * kD;
    // K rows: lane m reads block m/8, token-in-block 8((m/4)%2) + 4t + m%4, d = 32ks + 8q
    const bf16_t *kb = pool + ((size_t)((m >> 3) ? blk1 : blk0) * Hkv + c) * head_stride;
    const int tok0 = 8 * ((m >> 2) & 1) + (m & 3);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks)
            f.k[t][ks] = *(const bf16x8 *)(kb + (size_t)(tok0 + 4 * t) * kD + 32 * ks + 8 * q);
    // V^T rows: lane reads block q/2, d = 16dt + m, tokens 8(q%2) .. +7
    const bf16_t *vb = pool + ((size_t)((q >> 1) ? blk1 : blk0) * Hkv + c) * head_stride + (size_t)kBk * kD;
#pragma unroll
    for (int dt = 0; dt < kDT; ++dt) f.v[dt] = *(const bf16x8 *)(vb + (size_t)(16 * dt + m) * kBk + 8 * (q & 1));
}

// The O^T accumulators live in the accumulation registers, where the matrix cores update them in place.  The
// rare rescale (a moved softmax reference) multiplies copies in ordinary registers; left to itself the
// compiler then keeps the accumulators of the common path in ordinary registers too and moves all of them
// across for every group.  An empty statement that demands its operand in an accumulation register, placed
// where the two paths meet, keeps the copies inside the rare branch.
#define ICARUS_IN_ACC(x) asm volatile("" : "+a"(x))

// Where the decode walks keep the wave's Q fragments: in registers when the wave has two or three query tiles (a
// wave issues in order and is alone on its SIMD, so a fragment read in front of the MFMAs that need it stalls it for
// the read's whole latency, up to twelve times per group); with one tile they stay in LDS, which keeps that
// instantiation at two workgroups per CU.
template <int NT>
constexpr bool kQInRegs = NT > 1;

// Per-wave running state for NT query tiles.
template <int NT>
struct State {
    f32x4 o[kDT][NT];  // O^T accumulators: [d 16dt + 4q + i][query 16qt + l%16]
    float m[NT];       // running max (log2 domain), uniform over the 4 lanes sharing a query
    float l[NT];       // running sum, per-lane partial (reduced over q at the end)
};

// One 32-token group: S^T, online softmax, PV, one 16-query tile at a time so that only one
// tile's scores are live.  Uses the first N tiles of st.  Q fragments of those tiles (B operands): qr, in
// registers, or qlds, in LDS as [qt][ks][lane] (see kQInRegs).
// tail == false: all 32 tokens are valid for every query.
// tail == true:  `left` tokens of the chunk remain from this group's first token on (for the row
//   with the longest context); query tile qt of this lane may attend only to the first
//   left - stag[qt] of them (stag: how many positions the lane's query row ends before the last
//   row -- 0 at decode, the causal stagger of a prefill chunk).
template <int NT, int N, bool tail>
__device__ __forceinline__ void compute_group(State<NT> &st, KVFrag &f, const bf16x8 (&qr)[NT][kKS], const bf16x8 *__restrict__ qlds, int left,
                                              const int (&stag)[NT], float scale_log2, int lane) {
    const int q = lane >> 4;
    // token index inside the group of S^T element (tile t, register i) on this lane: tbase + 4t + i
    const int tbase = 16 * (q >> 1) + 8 * (q & 1);
    if (tail) {
        // stale cache bytes past the end may hold anything: zero those V columns (scores are masked below)
#pragma unroll
        for (int dt = 0; dt < kDT; ++dt)
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (tbase + e >= left) f.v[dt][e] = (__bf16)0.f;
    }
#pragma unroll
    for (int qt = 0; qt < N; ++qt) {
#pragma unroll
        for (int dt = 0; dt < kDT; ++dt) ICARUS_IN_ACC(st.o[dt][qt]);
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks) {
            const bf16x8 qv = kQInRegs<NT> ? qr[qt][ks] : qlds[(qt * kKS + ks) * 64 + lane];
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.k[0][ks], qv, s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.k[1][ks], qv, s1, 0, 0, 0);
        }
        // raw scores; the softmax scale (> 0) is applied to their maximum and inside the exponent's fused
        // multiply-add, not to each score
        float sv[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            sv[i] = s0[i];
            sv[4 + i] = s1[i];
        }
        if (tail) {
            const int lim = left - stag[qt];
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (tbase + e >= lim) sv[e] = -INFINITY;
        }
        float mx = sv[0];
#pragma unroll
        for (int e = 1; e < 8; ++e) mx = fmaxf(mx, sv[e]);
        mx *= scale_log2;
        // st.m is a reference exponent, not necessarily the exact running max: it moves (and the
        // accumulators are rescaled) only when some score exceeds it by more than kSlack, so
        // p = 2^(s - m) stays below 2^kSlack and the common case needs no cross-lane exchange.
        if (__any(mx > st.m[qt] + kSlack)) {
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_old = st.m[qt];
            const float m_new = fmaxf(m_old, mx);
            st.m[qt] = m_new;
            // in a tail group a query may have no valid token yet (m_new still -inf): nothing to rescale
            float alpha = (tail && m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m_old - m_new);
            st.l[qt] *= alpha;
#pragma unroll
            for (int dt = 0; dt < kDT; ++dt) {
                st.o[dt][qt][0] *= alpha; st.o[dt][qt][1] *= alpha; st.o[dt][qt][2] *= alpha; st.o[dt][qt][3] *= alpha;
                ICARUS_IN_ACC(st.o[dt][qt]);
            }
        }
        const float m_ref = st.m[qt];
        float rs = 0.f;
        bf16x8 pb;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[e], scale_log2, -m_ref));
            if (tail && m_ref == -INFINITY) p = 0.f;
            rs += p;
            pb[e] = (__bf16)p;
        }
        st.l[qt] += rs;
#pragma unroll
        for (int dt = 0; dt < kDT; ++dt) st.o[dt][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.v[dt], pb, st.o[dt][qt], 0, 0, 0);
    }
}

// A wave's walk over its share of the chunk: groups first, first + stride, ... with N query tiles.
// The first n_clean groups are valid for every query: they run in a loop with two register buffers,
// loads issued one group ahead.  The few groups after them (a partial last group, the causal
// stagger of a prefill chunk) are done with masks by the waves they fall to.
template <int NT, int N>
__device__ __forceinline__ void wave_walk(State<NT> &st, const bf16_t *__restrict__ pool, const int *__restrict__ blds,
                                          int n_blk, int n_tok, int n_clean, const int (&stag)[NT], int first, int stride,
                                          int c, int Hkv, const bf16x8 (&qr)[NT][kKS], const bf16x8 *__restrict__ qlds, float scale_log2, int lane) {
    const int n_grp = (n_tok + kGrp - 1) / kGrp;
    auto blk_of = [&](int grp, int which) {
        return __builtin_amdgcn_readfirstlane(blds[min(grp * 2 + which, n_blk - 1)]);
    };
    KVFrag f0, f1;
    if (first < n_clean) load_group(f0, pool, blk_of(first, 0), blk_of(first, 1), c, Hkv, lane);
    // The loads of the loop are unconditional (past the end blk_of repeats the chunk's last block and the
    // data is dropped): with a load under a condition the compiler no longer knows how many younger loads
    // are in flight when a buffer is consumed and waits for all of them, the prefetch included.
#pragma nounroll
    for (int grp = first; grp < n_clean; grp += 2 * stride) {
        load_group(f1, pool, blk_of(grp + stride, 0), blk_of(grp + stride, 1), c, Hkv, lane);
        compute_group<NT, N, false>(st, f0, qr, qlds, kGrp, stag, scale_log2, lane);
        load_group(f0, pool, blk_of(grp + 2 * stride, 0), blk_of(grp + 2 * stride, 1), c, Hkv, lane);
        if (grp + stride < n_clean) compute_group<NT, N, false>(st, f1, qr, qlds, kGrp, stag, scale_log2, lane);
    }
#pragma nounroll
    for (int grp = n_clean; grp < n_grp; ++grp) {
        if (grp % stride != first) continue;
        load_group(f0, pool, blk_of(grp, 0), blk_of(grp, 1), c, Hkv, lane);
        compute_group<NT, N, true>(st, f0, qr, qlds, n_tok - grp * kGrp, stag, scale_log2, lane);
    }
}

// ---- FP8 (E4M3) cache: 1-byte codes, value = code * scale (one scale for K, one for V) ----------------
// The codes are exact in bf16, so they go through the same bf16 MFMAs after a register conversion; the
// scales are folded into the softmax scale (K) and the final normalisation (V).  Loads stay 16 bytes
// per lane for K: a lane's 16 codes are 16 consecutive d of one token, i.e. the lane's operand
// elements of TWO k-steps, so the contraction index is laid out differently from the bf16 path
//   k-step 2s + h, lane quarter q  <->  d = 64 s + 16 q + 8 h .. + 7
// and the Q fragments are staged in the same order (a dot product does not care).  V^T rows hold 16
// tokens in 16 bytes; a lane needs the 8 of its quarter: 8-byte loads, 16 rows x 16 bytes of a block
// fully used by each wave-wide load.
struct KVRaw8 {
    uint4 k[2][2];  // k[t][s]: tile t, d slab s (64 codes per row, 16 per lane)
    uint2 v[kDT];   // v[dt]: 8 tokens of row d = 16 dt + l%16
};

__device__ __forceinline__ void load_group8(KVRaw8 &f, const uint8_t *__restrict__ pool, int blk0, int blk1, int c, int Hkv,
                                            int lane) {
    const int m = lane & 15, q = lane >> 4;
    const size_t head_stride = (size_t)2 * kBk * kD;  // bytes
    const uint8_t *kb = pool + ((size_t)((m >> 3) ? blk1 : blk0) * Hkv + c) * head_stride;
    const int tok0 = 8 * ((m >> 2) & 1) + (m & 3);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) f.k[t][sl] = *(const uint4 *)(kb + (size_t)(tok0 + 4 * t) * kD + 64 * sl + 16 * q);
    const uint8_t *vb = pool + ((size_t)((q >> 1) ? blk1 : blk0) * Hkv + c) * head_stride + (size_t)kBk * kD;
#pragma unroll
    for (int dt = 0; dt < kDT; ++dt) f.v[dt] = *(const uint2 *)(vb + (size_t)(16 * dt + m) * kBk + 8 * (q & 1));
}

// 8 FP8 codes (two dwords) -> 8 bf16, exactly.
__device__ __forceinline__ bf16x8 cvt8(uint32_t lo, uint32_t hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    uint4 r;
    r.x = __builtin_bit_cast(uint32_t, (bf16x2)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, false));
    r.y = __builtin_bit_cast(uint32_t, (bf16x2)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, true));
    r.z = __builtin_bit_cast(uint32_t, (bf16x2)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, false));
    r.w = __builtin_bit_cast(uint32_t, (bf16x2)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, true));
    return __builtin_bit_cast(bf16x8, r);
}

// compute_group for raw FP8 fragments: the scores of all N tiles first (K codes are converted one
// k-step at a time and die at once), then the softmax of every tile, then PV with V^T codes converted
// one d tile at a time.  scale_log2 includes the K scale; the V scale is applied when the piece ends.
template <int NT, int N, bool tail>
__device__ __forceinline__ void compute_group8(State<NT> &st, const KVRaw8 &f, const bf16x8 (&qr)[NT][kKS], const bf16x8 *__restrict__ qlds, int left,
                                               const int (&stag)[NT], float scale_log2, int lane) {
    const int q = lane >> 4;
    const int tbase = 16 * (q >> 1) + 8 * (q & 1);
    f32x4 s0[N], s1[N];
#pragma unroll
    for (int qt = 0; qt < N; ++qt) {
        s0[qt] = f32x4{0.f, 0.f, 0.f, 0.f}; s1[qt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int dt = 0; dt < kDT; ++dt) ICARUS_IN_ACC(st.o[dt][qt]);
    }
#pragma unroll
    for (int ks = 0; ks < kKS; ++ks) {
        const uint4 r0 = f.k[0][ks >> 1], r1 = f.k[1][ks >> 1];
        const bf16x8 a0 = (ks & 1) ? cvt8(r0.z, r0.w) : cvt8(r0.x, r0.y);
        const bf16x8 a1 = (ks & 1) ? cvt8(r1.z, r1.w) : cvt8(r1.x, r1.y);
#pragma unroll
        for (int qt = 0; qt < N; ++qt) {
            const bf16x8 qv = kQInRegs<NT> ? qr[qt][ks] : qlds[(qt * kKS + ks) * 64 + lane];
            s0[qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, qv, s0[qt], 0, 0, 0);
            s1[qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, qv, s1[qt], 0, 0, 0);
        }
    }
    bf16x8 pb[N];
#pragma unroll
    for (int qt = 0; qt < N; ++qt) {
        float sv[8];  // raw scores, see compute_group
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            sv[i] = s0[qt][i];
            sv[4 + i] = s1[qt][i];
        }
        if (tail) {
            const int lim = left - stag[qt];
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (tbase + e >= lim) sv[e] = -INFINITY;  // also replaces whatever stale codes produced
        }
        float mx = sv[0];
#pragma unroll
        for (int e = 1; e < 8; ++e) mx = fmaxf(mx, sv[e]);
        mx *= scale_log2;
        if (__any(mx > st.m[qt] + kSlack)) {  // see compute_group: lazy softmax reference
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_old = st.m[qt];
            const float m_new = fmaxf(m_old, mx);
            st.m[qt] = m_new;
            float alpha = (tail && m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m_old - m_new);
            st.l[qt] *= alpha;
#pragma unroll
            for (int dt = 0; dt < kDT; ++dt) {
                st.o[dt][qt][0] *= alpha; st.o[dt][qt][1] *= alpha; st.o[dt][qt][2] *= alpha; st.o[dt][qt][3] *= alpha;
                ICARUS_IN_ACC(st.o[dt][qt]);
            }
        }
        const float m_ref = st.m[qt];
        float rs = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[e], scale_log2, -m_ref));
            if (tail && m_ref == -INFINITY) p = 0.f;
            rs += p;
            pb[qt][e] = (__bf16)p;
        }
        st.l[qt] += rs;
    }
#pragma unroll
    for (int dt = 0; dt < kDT; ++dt) {
        bf16x8 av = cvt8(f.v[dt].x, f.v[dt].y);
        if (tail) {  // stale codes past the end may decode to anything, NaN included
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (tbase + e >= left) av[e] = (__bf16)0.f;
        }
#pragma unroll
        for (int qt = 0; qt < N; ++qt) st.o[dt][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, pb[qt], st.o[dt][qt], 0, 0, 0);
    }
}

// wave_walk over an FP8 cache: the two register buffers hold raw codes (48 registers each).
template <int NT, int N>
__device__ __forceinline__ void wave_walk8(State<NT> &st, const uint8_t *__restrict__ pool, const int *__restrict__ blds,
                                           int n_blk, int n_tok, int n_clean, const int (&stag)[NT], int first, int stride,
                                           int c, int Hkv, const bf16x8 (&qr)[NT][kKS], const bf16x8 *__restrict__ qlds, float scale_log2, int lane) {
    const int n_grp = (n_tok + kGrp - 1) / kGrp;
    auto blk_of = [&](int grp, int which) {
        return __builtin_amdgcn_readfirstlane(blds[min(grp * 2 + which, n_blk - 1)]);
    };
    KVRaw8 f0, f1;
    if (first < n_clean) load_group8(f0, pool, blk_of(first, 0), blk_of(first, 1), c, Hkv, lane);
#pragma nounroll
    for (int grp = first; grp < n_clean; grp += 2 * stride) {  // unconditional loads, see wave_walk
        load_group8(f1, pool, blk_of(grp + stride, 0), blk_of(grp + stride, 1), c, Hkv, lane);
        compute_group8<NT, N, false>(st, f0, qr, qlds, kGrp, stag, scale_log2, lane);
        load_group8(f0, pool, blk_of(grp + 2 * stride, 0), blk_of(grp + 2 * stride, 1), c, Hkv, lane);
        if (grp + stride < n_clean) compute_group8<NT, N, false>(st, f1, qr, qlds, kGrp, stag, scale_log2, lane);
    }
#pragma nounroll
    for (int grp = n_clean; grp < n_grp; ++grp) {
        if (grp % stride != first) continue;
        load_group8(f0, pool, blk_of(grp, 0), blk_of(grp, 1), c, Hkv, lane);
        compute_group8<NT, N, true>(st, f0, qr, qlds, n_tok - grp * kGrp, stag, scale_log2, lane);
    }
}

// The walk used when the query tiles are split over wave pairs (more than 3 tiles), for an FP8 cache (a bf16
// cache takes shared_walk_dma below).  Every group must reach two waves (one per tile set) but should come
// from HBM once and stay a distinct load in flight, so loading and computing are decoupled: in each round of
// four groups wave w loads the raw codes of group 4r + w into registers, expands them to bf16 MFMA fragments
// (k-step order of KVRaw8) as it publishes them to an LDS ring in lane order, and after one barrier computes
// the two groups of its parity (half) for its own tiles from the ring.  The loads of the next round are in
// flight while a round is computed.  ring: [2][4][16][64] x 16 B.
template <int NT, int N>
__device__ __forceinline__ void shared_walk8(State<NT> &st, const uint8_t *__restrict__ pool8, const int *__restrict__ blds,
                                             int n_blk, int n_tok, int n_clean, const int (&stag)[NT], int w, int half, int c,
                                             int Hkv, bf16x8 *__restrict__ ring, const bf16x8 (&qr)[NT][kKS], const bf16x8 *__restrict__ qlds,
                                             float scale_log2, int lane) {
    const int n_grp = (n_tok + kGrp - 1) / kGrp;                       // groups, the masked ones included
    const int n_round = (n_grp + 3) / 4;                               // the same for every wave
    auto blk_of = [&](int grp, int which) {
        return __builtin_amdgcn_readfirstlane(blds[min(grp * 2 + which, n_blk - 1)]);
    };
    KVRaw8 f8;
    auto load = [&](int grp) { load_group8(f8, pool8, blk_of(grp, 0), blk_of(grp, 1), c, Hkv, lane); };
    if (w < n_grp) load(w);
#pragma nounroll
    for (int r = 0; r < n_round; ++r) {
        bf16x8 *stage = ring + (size_t)(r & 1) * 4 * 16 * 64;
        const int mine = 4 * r + w;
        if (mine < n_grp) {
            bf16x8 *dst = stage + (size_t)w * 16 * 64 + lane;
#pragma unroll
            for (int i = 0; i < 2 * kKS; ++i) {
                const uint4 rk = f8.k[i / kKS][(i % kKS) >> 1];
                dst[i * 64] = (i & 1) ? cvt8(rk.z, rk.w) : cvt8(rk.x, rk.y);
            }
#pragma unroll
            for (int dt = 0; dt < kDT; ++dt) dst[(2 * kKS + dt) * 64] = cvt8(f8.v[dt].x, f8.v[dt].y);
        }
        if (mine + 4 < n_grp) load(mine + 4);
        __syncthreads();
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int gi = half + 2 * u, grp = 4 * r + gi;
            if (grp < n_grp) {
                const bf16x8 *src = stage + (size_t)gi * 16 * 64 + lane;
                KVFrag gfr;
#pragma unroll
                for (int i = 0; i < 2 * kKS; ++i) gfr.k[i / kKS][i % kKS] = src[i * 64];
#pragma unroll
                for (int dt = 0; dt < kDT; ++dt) gfr.v[dt] = src[(2 * kKS + dt) * 64];
                if (grp >= n_clean)
                    compute_group<NT, N, true>(st, gfr, qr, qlds, n_tok - grp * kGrp, stag, scale_log2, lane);
                else
                    compute_group<NT, N, false>(st, gfr, qr, qlds, kGrp, stag, scale_log2, lane);
            }
        }
    }
    __syncthreads();  // the ring may be reused now
}

// 16-byte LDS-direct load: lane i copies 16 bytes from its own global address to LDS byte lds_base + 16 i
// (lds_base wave-uniform, passed in m0); the load counts in vmcnt until the data is in LDS.
__device__ __forceinline__ void dma16(const void *g, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(g) : "memory");
}

// The shared walk of a bf16 cache with the ring filled by LDS-direct loads.  A wave's 16-byte loads of a
// group ARE its MFMA fragments in lane order, so they can land in the ring as they are: no register buffer,
// and what is in flight is bounded by LDS, not by VGPRs.  The ring (the same 128 KB) is cut into four
// stages of two groups; in round r wave w loads half (w & 1: K or V^T fragments) of group 2r + w/2, three
// rounds ahead -- 96 KB in flight per CU against 64 KB with one group per wave in registers, which is what
// the five-tile walk was short of (a round waited for the load issued one round earlier).  Each wave issues
// exactly 8 loads per round (a group past the end is clamped to the last one and never read), so the
// number of younger loads at a wait is known: vmcnt(16) leaves the two younger rounds in flight.  One
// barrier per round: after it every wave's loads of round r are in LDS and every wave has finished round
// r-1, whose stage takes the loads of round r+3.
template <int NT, int N>
__device__ __forceinline__ void shared_walk_dma(State<NT> &st, const bf16_t *__restrict__ pool, const int *__restrict__ blds,
                                                int n_blk, int n_tok, int n_clean, const int (&stag)[NT], int w, int half, int c,
                                                int Hkv, bf16x8 *__restrict__ ring, const bf16x8 (&qr)[NT][kKS], const bf16x8 *__restrict__ qlds,
                                                float scale_log2, int lane) {
    constexpr int kStages = 4, kStageFrags = 2 * 16;  // fragments (1 KiB each) per stage
    static_assert(kRingBytes == (size_t)kStages * kStageFrags * 1024, "ring size");
    const int n_grp = (n_tok + kGrp - 1) / kGrp;
    const int n_round = (n_grp + 1) / 2;
    const int part = w & 1, gl = w >> 1;
    const int m = lane & 15, q = lane >> 4;
    const size_t head_stride = (size_t)2 * kBk * kD;
    const uint32_t ring0 = (uint32_t)(size_t)(__attribute__((address_space(3))) char *)ring;
    auto issue = [&](int r) {
        const int grp = min(2 * r + gl, n_grp - 1);
        const int blk0 = __builtin_amdgcn_readfirstlane(blds[min(grp * 2, n_blk - 1)]);
        const int blk1 = __builtin_amdgcn_readfirstlane(blds[min(grp * 2 + 1, n_blk - 1)]);
        const uint32_t dst = __builtin_amdgcn_readfirstlane(ring0 + ((r & (kStages - 1)) * kStageFrags + gl * 16 + part * 8) * 1024);
        if (part == 0) {  // K fragments k[t][ks]: block m/8, token 8((m/4)%2) + 4t + m%4, d = 32ks + 8q
            const bf16_t *kb = pool + ((size_t)((m >> 3) ? blk1 : blk0) * Hkv + c) * head_stride +
                               (size_t)(8 * ((m >> 2) & 1) + (m & 3)) * kD + 8 * q;
#pragma unroll
            for (int i = 0; i < 2 * kKS; ++i) dma16(kb + (size_t)(4 * (i / kKS)) * kD + 32 * (i % kKS), dst + i * 1024);
        } else {  // V^T fragments v[dt]: block q/2, d = 16dt + m, tokens 8(q%2) .. +7
            const bf16_t *vb = pool + ((size_t)((q >> 1) ? blk1 : blk0) * Hkv + c) * head_stride + (size_t)kBk * kD +
                               (size_t)m * kBk + 8 * (q & 1);
#pragma unroll
            for (int dt = 0; dt < kDT; ++dt) dma16(vb + (size_t)(16 * dt) * kBk, dst + dt * 1024);
        }
    };
#pragma unroll
    for (int r = 0; r < kStages - 1; ++r)
        if (r < n_round) issue(r);
#pragma nounroll
    for (int r = 0; r < n_round; ++r) {
        const int younger = min(n_round, r + kStages - 1) - (r + 1);  // rounds this wave has issued after round r
        if (younger >= 2) __builtin_amdgcn_s_waitcnt(0x0f70 | 0x4000);  // vmcnt(16)
        else if (younger == 1) __builtin_amdgcn_s_waitcnt(0x0f70 | 8);  // vmcnt(8)
        else __builtin_amdgcn_s_waitcnt(0x0f70);                        // vmcnt(0)
        __syncthreads();
        if (r + kStages - 1 < n_round) issue(r + kStages - 1);
        const int grp = 2 * r + half;
        if (grp < n_grp) {
            const bf16x8 *src = ring + ((size_t)(r & (kStages - 1)) * kStageFrags + half * 16) * 64 + lane;
            KVFrag gfr;
#pragma unroll
            for (int i = 0; i < 2 * kKS; ++i) gfr.k[i / kKS][i % kKS] = src[i * 64];
#pragma unroll
            for (int dt = 0; dt < kDT; ++dt) gfr.v[dt] = src[(2 * kKS + dt) * 64];
            if (grp >= n_clean)
                compute_group<NT, N, true>(st, gfr, qr, qlds, n_tok - grp * kGrp, stag, scale_log2, lane);
            else
                compute_group<NT, N, false>(st, gfr, qr, qlds, kGrp, stag, scale_log2, lane);
        }
    }
    __syncthreads();  // the ring may be reused now
}

// LDS image of a state: o as [dt][qt][i][lane], then m[qt][lane], l[qt][lane].
template <int NT>
__device__ __forceinline__ void merge_from_lds(State<NT> &st, const float *__restrict__ lds, int lane) {
    const float *lo = lds;
    const float *lm = lds + kDT * NT * 4 * 64;
    const float *ll = lm + NT * 64;
#pragma unroll
    for (int qt = 0; qt < NT; ++qt) {
        float m2 = lm[qt * 64 + lane], l2 = ll[qt * 64 + lane];
        float mn = fmaxf(st.m[qt], m2);
        float a1 = st.m[qt] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(st.m[qt] - mn);
        float a2 = m2 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m2 - mn);
        st.m[qt] = mn;
        st.l[qt] = st.l[qt] * a1 + l2 * a2;
#pragma unroll
        for (int dt = 0; dt < kDT; ++dt)
#pragma unroll
            for (int i = 0; i < 4; ++i) st.o[dt][qt][i] = st.o[dt][qt][i] * a1 + lo[((dt * NT + qt) * 4 + i) * 64 + lane] * a2;
    }
}
template <int NT>
__device__ __forceinline__ void store_to_lds(const State<NT> &st, float *__restrict__ lds, int lane) {
    float *lo = lds;
    float *lm = lds + kDT * NT * 4 * 64;
    float *ll = lm + NT * 64;
#pragma unroll
    for (int qt = 0; qt < NT; ++qt) {
        lm[qt * 64 + lane] = st.m[qt];
        ll[qt * 64 + lane] = st.l[qt];
#pragma unroll
        for (int dt = 0; dt < kDT; ++dt)
#pragma unroll
            for (int i = 0; i < 4; ++i) lo[((dt * NT + qt) * 4 + i) * 64 + lane] = st.o[dt][qt][i];
    }
}

// Write tiles [0, n) of st as the call's query tiles qt0 .. qt0+n-1: the final output when the
// sequence has a single chunk, else this chunk's partial result.
template <int NT>
__device__ __forceinline__ void finish(State<NT> &st, int qt0, int n, int G, int g, int row0, int c, int Hq, int Hkv,
                                       int direct, int slot, int g_max, bf16_t *__restrict__ out,
                                       float *__restrict__ part_o, float *__restrict__ part_ml, int lane) {
    const int m = lane & 15, q = lane >> 4;
#pragma unroll
    for (int qt = 0; qt < NT; ++qt) {
        float l = st.l[qt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        int j = 16 * (qt0 + qt) + m;
        if (qt >= n || j >= G) continue;
        if (direct) {
            float inv = 1.f / l;
            bf16_t *op = out + ((size_t)(row0 + j / g) * Hq + c * g + j % g) * kD;
#pragma unroll
            for (int dt = 0; dt < kDT; ++dt) {
                uint2 pk;
                pk.x = (uint32_t)f32_to_bf16(st.o[dt][qt][0] * inv) | ((uint32_t)f32_to_bf16(st.o[dt][qt][1] * inv) << 16);
                pk.y = (uint32_t)f32_to_bf16(st.o[dt][qt][2] * inv) | ((uint32_t)f32_to_bf16(st.o[dt][qt][3] * inv) << 16);
                *(uint2 *)(op + 16 * dt + 4 * q) = pk;
            }
        } else {
            size_t pj = ((size_t)slot * Hkv + c) * g_max + j;
            float *po = part_o + pj * kD;
#pragma unroll
            for (int dt = 0; dt < kDT; ++dt) *(f32x4 *)(po + 16 * dt + 4 * q) = st.o[dt][qt];
            if (q == 0) {
                part_ml[pj * 2] = st.m[qt];
                part_ml[pj * 2 + 1] = l;
            }
        }
    }
}

// NA: query tiles of waves 0,1 (of all four waves when NB == 0); NB: query tiles of waves 2,3.
// KV8: the pool holds FP8 codes (scale_log2 then includes the K scale, v_scale multiplies the output).
template <int NA, int NB, bool KV8 = false>
__global__ void __launch_bounds__(256) k_attn_decode(const bf16_t *__restrict__ qg, const void *__restrict__ pool_v,
                                                     const int32_t *__restrict__ bt, int max_blocks, AttnPlan pl,
                                                     bf16_t *__restrict__ out, float *__restrict__ part_o,
                                                     float *__restrict__ part_ml, int Hq, int Hkv, float scale_log2,
                                                     float v_scale) {
    const bf16_t *pool = (const bf16_t *)pool_v;
    constexpr int NQT = NA + NB;
    constexpr int kImg = kDT * NA * 4 * 64 + 2 * NA * 64;  // floats per wave image of the merge
    extern __shared__ float lds[];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int g = Hq / Hkv;
    const int m = lane & 15, q = lane >> 4;
  // the pieces of this workgroup's share, one after the other; the Hkv workgroups of a share (one per
  // kv-head, on different XCDs) walk the same blocks at about the same time
  const int share = blockIdx.x / Hkv, c = blockIdx.x % Hkv;
  for (int item = pl.wg_first[share]; item < pl.wg_first[share + 1]; ++item) {
    const int s = pl.item_seq[item];
    const int tok_begin = pl.item_begin[item];
    const int tok_end = tok_begin + pl.item_len[item];
    const int row0 = pl.seq_row0[s], T = pl.seq_rows[s];
    const int G = T * g;
    const int32_t *btr = bt + (size_t)pl.seq_bt[s] * max_blocks;

    // Q fragments (B operands) go to LDS once, as [qt][ks][lane]; wave w stages k-step w.
    // query j = 16qt + m  ->  row row0 + j / g, head c*g + j % g; rows past G are zero.
    // LDS: [merge images | KV ring] [Q fragments] [block ids]; the merge images reuse the ring.
    constexpr size_t kHead = NB ? kRingBytes : (size_t)2 * kImg * sizeof(float);
    static_assert(!NB || kRingBytes >= (size_t)2 * kImg * sizeof(float), "merge images must fit the ring");
    bf16x8 *qlds = (bf16x8 *)((char *)lds + kHead);
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        int j = 16 * qt + m;
        // k-step w of this lane: d = 32 w + 8 q (bf16 cache), d = 64 (w / 2) + 16 q + 8 (w % 2) (FP8 cache, see KVRaw8)
        const int d0 = KV8 ? 64 * (w >> 1) + 16 * q + 8 * (w & 1) : 8 * q + 32 * w;
        const bf16_t *qp = qg + ((size_t)(row0 + j / g) * Hq + c * g + j % g) * kD + d0;
        qlds[(qt * kKS + w) * 64 + lane] = j < G ? *(const bf16x8 *)qp : zero8();
    }
    // The chunk's block ids go to LDS too: a lookup in the loop is then an LDS read, not a global
    // load whose wait would also drain the KV loads in flight.
    int *blds = (int *)(qlds + NQT * kKS * 64);
    const int n_tok = tok_end - tok_begin;
    const int n_blk = (n_tok + kBk - 1) / kBk;
    for (int i = threadIdx.x; i < n_blk; i += 256) blds[i] = btr[tok_begin / kBk + i];
    __syncthreads();
    // the wave's own Q fragments, see kQInRegs (waves 2, 3 of a launch with NB tiles hold tiles NA .. NA + NB - 1)
    bf16x8 qr[NA][kKS];
    if constexpr (kQInRegs<NA>) {
        const bool second = NB && (w >> 1);
        const bf16x8 *qsrc = qlds + (second ? NA * kKS * 64 : 0) + lane;
        const int nq = second ? NB : NA;
#pragma unroll
        for (int qt = 0; qt < NA; ++qt)
#pragma unroll
            for (int ks = 0; ks < kKS; ++ks) qr[qt][ks] = qt < nq ? qsrc[(qt * kKS + ks) * 64] : zero8();
    }

    State<NA> st;
#pragma unroll
    for (int qt = 0; qt < NA; ++qt) {
        st.m[qt] = -INFINITY;
        st.l[qt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < kDT; ++dt) st.o[dt][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const int direct = pl.item_direct[item];
    const int slot = pl.item_part[item];
    // every stacked query of a decode step sits at the same position: all whole groups need no mask
    const int n_clean = n_tok / kGrp;
    int stag[NA];
#pragma unroll
    for (int qt = 0; qt < NA; ++qt) stag[qt] = 0;

    if constexpr (NB == 0) {
        // the launch is sized for the largest stacked group of the call; a sequence with fewer
        // streams multiplies only the query tiles it has
        const int n_act = (G + 15) >> 4;
        if constexpr (KV8) {
            const uint8_t *pool8 = (const uint8_t *)pool_v;
            if (NA >= 3 && n_act >= 3)
                wave_walk8<NA, NA>(st, pool8, blds, n_blk, n_tok, n_clean, stag, w, 4, c, Hkv, qr, qlds, scale_log2, lane);
            else if (NA >= 2 && n_act == 2)
                wave_walk8<NA, (NA >= 2 ? 2 : 1)>(st, pool8, blds, n_blk, n_tok, n_clean, stag, w, 4, c, Hkv, qr, qlds, scale_log2, lane);
            else
                wave_walk8<NA, 1>(st, pool8, blds, n_blk, n_tok, n_clean, stag, w, 4, c, Hkv, qr, qlds, scale_log2, lane);
#pragma unroll
            for (int qt = 0; qt < NA; ++qt)
#pragma unroll
                for (int dt = 0; dt < kDT; ++dt) {
                    st.o[dt][qt][0] *= v_scale; st.o[dt][qt][1] *= v_scale; st.o[dt][qt][2] *= v_scale; st.o[dt][qt][3] *= v_scale;
                }
        } else if (NA >= 3 && n_act >= 3)
            wave_walk<NA, NA>(st, pool, blds, n_blk, n_tok, n_clean, stag, w, 4, c, Hkv, qr, qlds, scale_log2, lane);
        else if (NA >= 2 && n_act == 2)
            wave_walk<NA, (NA >= 2 ? 2 : 1)>(st, pool, blds, n_blk, n_tok, n_clean, stag, w, 4, c, Hkv, qr, qlds, scale_log2, lane);
        else
            wave_walk<NA, 1>(st, pool, blds, n_blk, n_tok, n_clean, stag, w, 4, c, Hkv, qr, qlds, scale_log2, lane);
        // tree merge of the four waves through LDS: (2,3) -> (0,1), then 1 -> 0
        if (w >= 2) store_to_lds<NA>(st, lds + (w - 2) * kImg, lane);
        __syncthreads();
        if (w < 2) merge_from_lds<NA>(st, lds + w * kImg, lane);
        __syncthreads();
        if (w == 1) store_to_lds<NA>(st, lds, lane);
        __syncthreads();
        if (w == 0) {
            merge_from_lds<NA>(st, lds, lane);
            finish<NA>(st, 0, NA, G, g, row0, c, Hq, Hkv, direct, slot, pl.g_max, out, part_o, part_ml, lane);
        }
    } else {
        const int role = w >> 1, half = w & 1;  // role: which query tiles; half: which groups
        bf16x8 *ring = (bf16x8 *)lds;
        if constexpr (KV8) {  // codes are expanded on the way into the ring: through registers
            const uint8_t *pool8 = (const uint8_t *)pool_v;
            if (role == 0)
                shared_walk8<NA, NA>(st, pool8, blds, n_blk, n_tok, n_clean, stag, w, half, c, Hkv, ring, qr, qlds, scale_log2, lane);
            else
                shared_walk8<NA, NB>(st, pool8, blds, n_blk, n_tok, n_clean, stag, w, half, c, Hkv, ring, qr, qlds,
                                     scale_log2, lane);
        } else if (role == 0) {
            shared_walk_dma<NA, NA>(st, pool, blds, n_blk, n_tok, n_clean, stag, w, half, c, Hkv, ring, qr, qlds, scale_log2, lane);
        } else {
            shared_walk_dma<NA, NB>(st, pool, blds, n_blk, n_tok, n_clean, stag, w, half, c, Hkv, ring, qr, qlds,
                                    scale_log2, lane);
        }
        if constexpr (KV8) {
#pragma unroll
            for (int qt = 0; qt < NA; ++qt)
#pragma unroll
                for (int dt = 0; dt < kDT; ++dt) {
                    st.o[dt][qt][0] *= v_scale; st.o[dt][qt][1] *= v_scale; st.o[dt][qt][2] *= v_scale; st.o[dt][qt][3] *= v_scale;
                }
        }
        // each pair merges its two halves through its own LDS image
        if (half == 1) store_to_lds<NA>(st, lds + role * kImg, lane);
        __syncthreads();
        if (half == 0) {
            merge_from_lds<NA>(st, lds + role * kImg, lane);
            finish<NA>(st, role ? NA : 0, role ? NB : NA, G, g, row0, c, Hq, Hkv, direct, slot, pl.g_max, out, part_o, part_ml, lane);
        }
    }
    __syncthreads();  // LDS (Q fragments, block ids, merge images) is reused by the next piece
  }
}

// compute_group for a group that sits in LDS as fragments (src[i * 64]: K fragments i = 0..7, then
// V^T fragments) with the wave's Q fragments in registers (qr[qt][ks]).  A wave issues in order and a
// fragment read takes a few hundred cycles to come back, so the reads are batched ahead of the MFMAs
// that need them instead of sitting between them: the eight K fragments at the top, the eight V^T
// fragments as soon as the S^T MFMAs are issued (into the registers the K fragments leave), so that
// they travel while the softmax arithmetic runs and the P V MFMAs follow each other without a wait.
template <int NT, bool tail>
__device__ __forceinline__ void compute_group_lds(State<NT> &st, const bf16x8 *__restrict__ src, const bf16x8 (&qr)[NT][kKS],
                                                  int left, const int (&stag)[NT], float scale_log2, int lane) {
    const int q = lane >> 4;
    const int tbase = 16 * (q >> 1) + 8 * (q & 1);
    float sv[NT][8];
    __builtin_amdgcn_s_setprio(1);  // matrix-core sections run at raised priority, see prefill_walk
    {
        f32x4 s0[NT], s1[NT];
#pragma unroll
        for (int qt = 0; qt < NT; ++qt) { s0[qt] = f32x4{0.f, 0.f, 0.f, 0.f}; s1[qt] = f32x4{0.f, 0.f, 0.f, 0.f}; }
        bf16x8 kf[2 * kKS];
#pragma unroll
        for (int i = 0; i < 2 * kKS; ++i) kf[i] = src[i * 64];
        __builtin_amdgcn_sched_barrier(0);  // all reads first
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks) {
#pragma unroll
            for (int qt = 0; qt < NT; ++qt) {
                s0[qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks], qr[qt][ks], s0[qt], 0, 0, 0);
                s1[qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kKS + ks], qr[qt][ks], s1[qt], 0, 0, 0);
            }
        }
#pragma unroll
        for (int qt = 0; qt < NT; ++qt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {  // raw scores, see compute_group
                sv[qt][i] = s0[qt][i];
                sv[qt][4 + i] = s1[qt][i];
            }
    }
    __builtin_amdgcn_s_setprio(0);
    bf16x8 vf[kDT];
#pragma unroll
    for (int dt = 0; dt < kDT; ++dt) vf[dt] = src[(2 * kKS + dt) * 64];
    __builtin_amdgcn_sched_barrier(0);  // the reads stay ahead of the arithmetic
    bf16x8 pb[NT];
#pragma unroll
    for (int qt = 0; qt < NT; ++qt) {
        if (tail) {
            const int lim = left - stag[qt];
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (tbase + e >= lim) sv[qt][e] = -INFINITY;
        }
        float mx = sv[qt][0];
#pragma unroll
        for (int e = 1; e < 8; ++e) mx = fmaxf(mx, sv[qt][e]);
        mx *= scale_log2;
        if (__any(mx > st.m[qt] + kSlack)) {  // see compute_group: lazy softmax reference
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_old = st.m[qt];
            const float m_new = fmaxf(m_old, mx);
            st.m[qt] = m_new;
            float alpha = (tail && m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m_old - m_new);
            st.l[qt] *= alpha;
#pragma unroll
            for (int dt = 0; dt < kDT; ++dt) {
                st.o[dt][qt][0] *= alpha; st.o[dt][qt][1] *= alpha; st.o[dt][qt][2] *= alpha; st.o[dt][qt][3] *= alpha;
            }
        }
        const float m_ref = st.m[qt];
        float rs = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[qt][e], scale_log2, -m_ref));
            if (tail && m_ref == -INFINITY) p = 0.f;
            rs += p;
            pb[qt][e] = (__bf16)p;
        }
        st.l[qt] += rs;
    }
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int dt = 0; dt < kDT; ++dt) {
        if (tail) {  // stale cache bytes past the end may hold anything: zero those V columns
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (tbase + e >= left) vf[dt][e] = (__bf16)0.f;
        }
#pragma unroll
        for (int qt = 0; qt < NT; ++qt) st.o[dt][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dt], pb[qt], st.o[dt][qt], 0, 0, 0);
    }
    __builtin_amdgcn_s_setprio(0);
}

// Half of a group's loads: part 0 = the 8 K fragments, part 1 = the 8 V^T fragments, in the order
// they take in a KVFrag (k[t][ks] as 4t + ks, then v[dt]).
__device__ __forceinline__ void load_half(bf16x8 (&h)[8], int part, const bf16_t *__restrict__ pool, int blk0, int blk1, int c,
                                          int Hkv, int lane) {
    const int m = lane & 15, q = lane >> 4;
    const size_t head_stride = (size_t)2 * kBk * kD;
    if (part == 0) {
        const bf16_t *kb = pool + ((size_t)((m >> 3) ? blk1 : blk0) * Hkv + c) * head_stride;
        const int tok0 = 8 * ((m >> 2) & 1) + (m & 3);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int ks = 0; ks < kKS; ++ks) h[t * kKS + ks] = *(const bf16x8 *)(kb + (size_t)(tok0 + 4 * t) * kD + 32 * ks + 8 * q);
    } else {
        const bf16_t *vb = pool + ((size_t)((q >> 1) ? blk1 : blk0) * Hkv + c) * head_stride + (size_t)kBk * kD;
#pragma unroll
        for (int dt = 0; dt < kDT; ++dt) h[dt] = *(const bf16x8 *)(vb + (size_t)(16 * dt + m) * kBk + 8 * (q & 1));
    }
}
static_assert(2 * kKS == 8 && kDT == 8, "a half group is 8 fragments");

// The same half group from an FP8 cache: raw codes, r[i] = the 8 codes that become fragment i
// (K: i = 4 t + k-step, in the k-step order of KVRaw8; V^T: i = d tile).
__device__ __forceinline__ void load_half8(uint2 (&r)[8], int part, const uint8_t *__restrict__ pool, int blk0, int blk1, int c,
                                           int Hkv, int lane) {
    const int m = lane & 15, q = lane >> 4;
    const size_t head_stride = (size_t)2 * kBk * kD;
    if (part == 0) {
        const uint8_t *kb = pool + ((size_t)((m >> 3) ? blk1 : blk0) * Hkv + c) * head_stride;
        const int tok0 = 8 * ((m >> 2) & 1) + (m & 3);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int sl = 0; sl < 2; ++sl) {
                const uint4 v = *(const uint4 *)(kb + (size_t)(tok0 + 4 * t) * kD + 64 * sl + 16 * q);
                r[4 * t + 2 * sl] = uint2{v.x, v.y};
                r[4 * t + 2 * sl + 1] = uint2{v.z, v.w};
            }
    } else {
        const uint8_t *vb = pool + ((size_t)((q >> 1) ? blk1 : blk0) * Hkv + c) * head_stride + (size_t)kBk * kD;
#pragma unroll
        for (int dt = 0; dt < kDT; ++dt) r[dt] = *(const uint2 *)(vb + (size_t)(16 * dt + m) * kBk + 8 * (q & 1));
    }
}

// Prefill walk: the eight waves hold different query tiles and every wave needs every group, so a
// group is loaded once -- in round r wave w loads half (w & 1: K or V^T) of group 4r + w/2 into
// registers, one round ahead -- published to an LDS ring as MFMA fragments in lane order, and read
// from there by all eight.  The ring has two stages of one round each: a wave publishes round r into
// stage r % 2, whose last readers (round r - 2) all passed the barrier of round r - 1, so one barrier
// per round is enough and the waves may drift up to a round apart (the matrix-core work of one then
// overlaps the softmax arithmetic of the other on the same SIMD).  ring: [2][4][16][64] x 16 B.
template <int NT, bool KV8 = false>
__device__ __forceinline__ void prefill_walk(State<NT> &st, const void *__restrict__ pool_v, const int *__restrict__ blds,
                                             int n_blk, int n_tok, int n_clean, const int (&stag)[NT], int w, int c, int Hkv,
                                             bf16x8 *__restrict__ ring, const bf16x8 (&qr)[NT][kKS], float scale_log2,
                                             int lane) {
    const int n_grp = (n_tok + kGrp - 1) / kGrp;  // groups, the masked ones included
    const int n_round = (n_grp + 3) / 4;          // the same for every wave
    const int part = w & 1, gl = w >> 1;
    auto blk_of = [&](int grp, int which) {
        return __builtin_amdgcn_readfirstlane(blds[min(grp * 2 + which, n_blk - 1)]);
    };
    bf16x8 h[8];
    uint2 h8[8];
    auto load = [&](int grp) {
        if constexpr (KV8) load_half8(h8, part, (const uint8_t *)pool_v, blk_of(grp, 0), blk_of(grp, 1), c, Hkv, lane);
        else load_half(h, part, (const bf16_t *)pool_v, blk_of(grp, 0), blk_of(grp, 1), c, Hkv, lane);
    };
    if (gl < n_grp) load(gl);
#pragma nounroll
    for (int r = 0; r < n_round; ++r) {
        bf16x8 *stage = ring + (size_t)(r & 1) * 4 * 16 * 64;
        const int mine = 4 * r + gl;
        if (mine < n_grp) {
            bf16x8 *dst = stage + ((size_t)gl * 16 + part * 8) * 64 + lane;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if constexpr (KV8) dst[i * 64] = cvt8(h8[i].x, h8[i].y);  // codes are exact in bf16
                else dst[i * 64] = h[i];
            }
        }
        if (mine + 4 < n_grp) load(mine + 4);
        __syncthreads();
        // the round's unmasked groups, then its masked ones: two loops of one code path each (with both paths
        // in one loop body the accumulators are copied between the registers the two paths leave them in)
        const int n_here = min(4, n_grp - 4 * r), n_plain = max(0, min(n_here, n_clean - 4 * r));
#pragma nounroll
        for (int gi = 0; gi < n_plain; ++gi)
            compute_group_lds<NT, false>(st, stage + (size_t)gi * 16 * 64 + lane, qr, kGrp, stag, scale_log2, lane);
#pragma nounroll
        for (int gi = n_plain; gi < n_here; ++gi)
            compute_group_lds<NT, true>(st, stage + (size_t)gi * 16 * 64 + lane, qr, n_tok - (4 * r + gi) * kGrp, stag, scale_log2, lane);
    }
}

constexpr int kPrefillWaves = 8, kPrefillNT = 2;  // 8 waves x 2 tiles x 16 = 256 stacked queries per workgroup

// Causal attention of a prefill chunk.  A workgroup owns one kv-head of one group of T consecutive
// chunk tokens (T * g <= 256 stacked queries; token t attends to kv_len - (T-1-t) positions) and
// walks the sequence's cache once for all of them; wave w holds query tiles [w NT, (w+1) NT).
template <int NT, bool KV8 = false>
__global__ void __launch_bounds__(64 * kPrefillWaves) k_attn_prefill(const bf16_t *__restrict__ qg, const void *__restrict__ pool,
                                                                     const int32_t *__restrict__ bt, int max_blocks, AttnPlan pl,
                                                                     bf16_t *__restrict__ out, int Hq, int Hkv, float scale_log2,
                                                                     float v_scale) {
    extern __shared__ float lds[];
    const int item = blockIdx.x / Hkv, c = blockIdx.x % Hkv;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int s = pl.item_seq[item];
    const int n_tok = pl.seq_kvlen[s];  // a causal plan never splits a sequence
    const int row0 = pl.seq_row0[s], T = pl.seq_rows[s];
    const int g = Hq / Hkv, G = T * g;
    const int m = lane & 15, q = lane >> 4;
    const int32_t *btr = bt + (size_t)pl.seq_bt[s] * max_blocks;
    // LDS: [KV ring, two stages of 64 KB] [block ids]; the wave's Q fragments (B operands) stay in registers
    bf16x8 *ring = (bf16x8 *)lds;
    bf16x8 qr[NT][kKS];
#pragma unroll
    for (int qt = 0; qt < NT; ++qt) {
        int j = 16 * (w * NT + qt) + m;
        const bf16_t *qp = qg + ((size_t)(row0 + j / g) * Hq + c * g + j % g) * kD;
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks) {  // FP8 cache: the k-step order of KVRaw8
            const int d0 = KV8 ? 64 * (ks >> 1) + 16 * q + 8 * (ks & 1) : 32 * ks + 8 * q;
            qr[qt][ks] = j < G ? *(const bf16x8 *)(qp + d0) : zero8();
        }
    }
    int *blds = (int *)(ring + 2 * 4 * 16 * 64);
    const int n_blk = (n_tok + kBk - 1) / kBk;
    for (int i = threadIdx.x; i < n_blk; i += 64 * kPrefillWaves) blds[i] = btr[i];
    // every load so far has landed: the walk's waits then count its own prefetch loads only (left to its own
    // bookkeeping the compiler waits for the Q fragments inside the loop, and with them for the prefetch)
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
    __syncthreads();

    State<NT> st;
    int stag[NT];
#pragma unroll
    for (int qt = 0; qt < NT; ++qt) {
        st.m[qt] = -INFINITY;
        st.l[qt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < kDT; ++dt) st.o[dt][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
        stag[qt] = T - 1 - min((16 * (w * NT + qt) + m) / g, T - 1);
    }
    const int n_clean = max(0, n_tok - (T - 1)) / kGrp;  // groups valid for every query
    prefill_walk<NT, KV8>(st, pool, blds, n_blk, n_tok, n_clean, stag, w, c, Hkv, ring, qr, scale_log2, lane);
    if constexpr (KV8) {
#pragma unroll
        for (int qt = 0; qt < NT; ++qt)
#pragma unroll
            for (int dt = 0; dt < kDT; ++dt) {
                st.o[dt][qt][0] *= v_scale; st.o[dt][qt][1] *= v_scale; st.o[dt][qt][2] *= v_scale; st.o[dt][qt][3] *= v_scale;
            }
    }
    finish<NT>(st, w * NT, NT, G, g, row0, c, Hq, Hkv, 1, 0, 0, out, nullptr, nullptr, lane);
}

// Combine the partial results of sequences that were split into several chunks.
// One block of 128 threads per (row, query head); thread d owns output element d.
__global__ void __launch_bounds__(128) k_attn_merge(const float *__restrict__ part_o, const float *__restrict__ part_ml,
                                                    AttnPlan pl, const int32_t *__restrict__ row_seq /* row -> plan sequence */,
                                                    bf16_t *__restrict__ out, int Hq, int Hkv) {
    const int row = blockIdx.y, h = blockIdx.x, d = threadIdx.x;
    const int s = row_seq[row];
    const int g = Hq / Hkv, c = h / g;
    const int np = pl.seq_nparts[s];
    if (np <= 1) return;  // written directly by the attention kernel
    const int j = (row - pl.seq_row0[s]) * g + h % g;
    const int p0 = pl.seq_part0[s];
    float M = -INFINITY;
    for (int p = 0; p < np; ++p) M = fmaxf(M, part_ml[(((size_t)(p0 + p) * Hkv + c) * pl.g_max + j) * 2]);
    float num = 0.f, den = 0.f;
    for (int p = 0; p < np; ++p) {
        size_t pj = ((size_t)(p0 + p) * Hkv + c) * pl.g_max + j;
        float wgt = __builtin_amdgcn_exp2f(part_ml[pj * 2] - M);
        den += wgt * part_ml[pj * 2 + 1];
        num += wgt * part_o[pj * kD + d];
    }
    out[((size_t)row * Hq + h) * kD + d] = f32_to_bf16(num / den);
}

template <int NA, int NB, bool KV8 = false>
hipError_t launch_one(const void *q, const void *pool, const int32_t *bt, int max_blocks, const AttnPlan &pl, void *out,
                      float *part_o, float *part_ml, int Hq, int Hkv, float scale_log2, float v_scale, hipStream_t st) {
    constexpr int kImg = kDT * NA * 4 * 64 + 2 * NA * 64;
    // merge images + Q fragments + the chunk's block ids (chunk <= kAttnMaxChunk tokens)
    size_t shm = (NB ? kRingBytes : (size_t)2 * kImg * sizeof(float)) + (size_t)(NA + NB) * kKS * 64 * 16 +
                 (size_t)(kAttnMaxChunk / kBk) * 4;
    static bool attr_set = false;  // per instantiation
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_attn_decode<NA, NB, KV8>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((k_attn_decode<NA, NB, KV8>), dim3(pl.n_wgs * Hkv), dim3(256), shm, st, (const bf16_t *)q, pool, bt, max_blocks, pl,
                       (bf16_t *)out, part_o, part_ml, Hq, Hkv, scale_log2, v_scale);
    return hipGetLastError();
}

}  // namespace

bool attn_decode_mfma_supported(const Dims &dm, int g_max) {
    return dm.bf16 && dm.D == kD && dm.Bk == kBk && g_max >= 1 && g_max <= 80;
}

int attn_prefill_group_queries() { return kPrefillWaves * kPrefillNT * 16; }  // stacked queries one prefill workgroup holds

bool attn_prefill_mfma_supported(const Dims &dm, int g_max) {
    return dm.bf16 && dm.D == kD && dm.Bk == kBk && g_max >= 1 && g_max <= attn_prefill_group_queries();
}

hipError_t launch_attn_prefill_mfma(const Dims &dm, const void *q, const void *pool, const int32_t *bt, int max_blocks,
                                    const AttnPlan &pl, void *out, hipStream_t st) {
    if (pl.n_items <= 0) return hipSuccess;
    if (!pl.causal || pl.chunk > kAttnMaxChunk) return hipErrorInvalidValue;
    constexpr int NT = kPrefillNT;
    float scale_log2 = kLog2e / sqrtf((float)dm.D) * (dm.kv8 ? dm.k_scale : 1.f);
    size_t shm = (size_t)2 * 4 * 16 * 64 * 16 + (size_t)(kAttnMaxChunk / kBk) * 4;  // two ring stages + the block ids
    auto launch = [&](auto kernel, bool &attr_set) -> hipError_t {
        if (!attr_set) {
            hipError_t e = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm);
            if (e != hipSuccess) return e;
            attr_set = true;
        }
        hipLaunchKernelGGL(kernel, dim3(pl.n_items * dm.Hkv), dim3(64 * kPrefillWaves), shm, st, (const bf16_t *)q, pool, bt, max_blocks, pl,
                           (bf16_t *)out, dm.Hq, dm.Hkv, scale_log2, dm.kv8 ? dm.v_scale : 1.f);
        return hipGetLastError();
    };
    static bool set_bf16 = false, set_fp8 = false;
    return dm.kv8 ? launch(k_attn_prefill<NT, true>, set_fp8) : launch(k_attn_prefill<NT, false>, set_bf16);
}

hipError_t launch_attn_decode_mfma(const Dims &dm, const void *q, const void *pool, const int32_t *bt, int max_blocks,
                                   const AttnPlan &pl, void *out, float *part_o, float *part_ml, hipStream_t st) {
    if (pl.n_items <= 0) return hipSuccess;
    if (pl.causal || pl.chunk > kAttnMaxChunk || pl.n_wgs <= 0) return hipErrorInvalidValue;
    float scale_log2 = kLog2e / sqrtf((float)dm.D);
    int nqt = (pl.g_max + 15) / 16;
    if (dm.kv8) {  // FP8 codes: the K scale joins the softmax scale, the V scale the output
        scale_log2 *= dm.k_scale;
        switch (nqt) {
        case 1: return launch_one<1, 0, true>(q, pool, bt, max_blocks, pl, out, part_o, part_ml, dm.Hq, dm.Hkv, scale_log2, dm.v_scale, st);
        case 2: return launch_one<2, 0, true>(q, pool, bt, max_blocks, pl, out, part_o, part_ml, dm.Hq, dm.Hkv, scale_log2, dm.v_scale, st);
        case 3: return launch_one<3, 0, true>(q, pool, bt, max_blocks, pl, out, part_o, part_ml, dm.Hq, dm.Hkv, scale_log2, dm.v_scale, st);
        case 4: return launch_one<2, 2, true>(q, pool, bt, max_blocks, pl, out, part_o, part_ml, dm.Hq, dm.Hkv, scale_log2, dm.v_scale, st);
        case 5: return launch_one<3, 2, true>(q, pool, bt, max_blocks, pl, out, part_o, part_ml, dm.Hq, dm.Hkv, scale_log2, dm.v_scale, st);
        default: return hipErrorInvalidValue;
        }
    }
    switch (nqt) {
    case 1: return launch_one<1, 0>(q, pool, bt, max_blocks, pl, out, part_o, part_ml, dm.Hq, dm.Hkv, scale_log2, 1.f, st);
    case 2: return launch_one<2, 0>(q, pool, bt, max_blocks, pl, out, part_o, part_ml, dm.Hq, dm.Hkv, scale_log2, 1.f, st);
    case 3: return launch_one<3, 0>(q, pool, bt, max_blocks, pl, out, part_o, part_ml, dm.Hq, dm.Hkv, scale_log2, 1.f, st);
    case 4: return launch_one<2, 2>(q, pool, bt, max_blocks, pl, out, part_o, part_ml, dm.Hq, dm.Hkv, scale_log2, 1.f, st);
    case 5: return launch_one<3, 2>(q, pool, bt, max_blocks, pl, out, part_o, part_ml, dm.Hq, dm.Hkv, scale_log2, 1.f, st);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_attn_merge(const Dims &dm, const float *part_o, const float *part_ml, const AttnPlan &pl,
                             const int32_t *row_seq, void *out, int R, hipStream_t st) {
    if (R <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_attn_merge, dim3(dm.Hq, R), dim3(128), 0, st, part_o, part_ml, pl, row_seq, (bf16_t *)out, dm.Hq, dm.Hkv);
    return hipGetLastError();
}

}  // namespace icarus

// ICaRusLinear on gfx950 matrix cores: one base-weight GEMM over all stacked rows with the
// per-model LoRA delta folded in as extra K-steps (bf16 storage, fp32 accumulation).
//
//   Y[R, N] = X[R, K] . W[N, K]^T  +  T[R, M*r] . Bcat[N, M*r]^T
//
// T is the masked shrink result: T[row, j*r + i] = s * (A_j x_row)_i if row belongs to model j, else 0
// (encoder rows are all zero), so multiplying by the concatenation of every model's B applies to
// each row exactly its own adapter.  The extension costs M*r extra K on top of K (3-5 %) and needs
// no row reordering: the base weights are still read once for all streams (Alg. 2).
//
// Tiling: a workgroup of WAVES_M x WAVES_N waves owns a BM x BN output tile; each wave a
// (BM/WAVES_M) x (BN/WAVES_N) sub-tile of 32x32x16 bf16 MFMAs.  K advances BK at a time through a
// ring of NS LDS stages filled by 16-byte LDS-direct loads (global memory -> LDS without passing
// through registers), so NS-1 slabs are in flight or landed while one is computed and one barrier
// per slab suffices.  Inside LDS the 16-byte chunks of each 256-byte line are XOR-swizzled with
// the line number: the wave-wide loads write 1 KiB contiguously, and the MFMA fragment reads
// (16 bytes per lane, 32 consecutive rows) spread over all banks.  Every load reads an always-valid
// address (rows and columns past the matrix are clamped: they only feed outputs that are never
// stored; chunks that must read as zeros come from a page of zeros), so the K loop is branch-free
// apart from the switch from base-weight slabs to adapter slabs.
//
// MFMA 32x32x16 bf16 operand layout (lane l): A[row l%32][k 8(l/32)..+7], B[k 8(l/32)..+7][col l%32],
// C[row 8(r/4) + 4(l/32) + r%4][col l%32] for accumulator register r = 0..15.
#include <algorithm>
#include <cstdio>
#include <cstdlib>

#include "device_util.h"
#include "kernels.h"

namespace icarus {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

namespace {

constexpr int kKAlign = 64;  // K of every GEMM is a multiple of this

// Per-thread description of one 16-byte load of the weight (B) tile, fixed for the whole K loop.
struct BRow {
    const bf16_t *w;   // weight row + chunk offset: base-K loads are w + k
    const bf16_t *b;   // adapter B of this output column: &B[0][n][0] + chunk offset inside a model
    int kind;          // 0: no adapter columns; 1: adapter range [0, M*r); 2: range [M*r, 2*M*r) (up rows)
};

// LDS B-row b of weight tile tile_n -> weight row.  DUAL: a tile covers BN/2 output columns; inside
// each wave column of WN LDS rows the first WN/2 are gate rows and the next WN/2 the up rows of the
// same WN/2 output columns.
template <int BN, int WN>
__device__ __forceinline__ BRow b_row(const GemmArgs &g, int tile_n, int b) {
    BRow o;
    if (g.mode == GEMM_DUAL) {
        int wn = b / WN, j = (b % WN) / (WN / 2), nn = b % (WN / 2);
        int n = min(tile_n * (BN / 2) + wn * (WN / 2) + nn, g.n_seg[0] - 1);
        o.w = (j ? g.W[1] : g.W[0]) + (size_t)n * g.K;
        const bf16_t *B = j ? g.B[1] : g.B[0];
        o.kind = (g.T && B) ? 1 + j : 0;
        o.b = o.kind ? B + (size_t)n * g.r : o.w;
        return o;
    }
    // plain: up to three weight segments stacked along N; tiles never straddle segments
    int t = tile_n;
    const bf16_t *W = g.W[0];
    int n_seg = g.n_seg[0];
    bool first = true;
    if (g.nseg > 1 && t >= g.tiles_seg[0]) {
        t -= g.tiles_seg[0]; W = g.W[1]; n_seg = g.n_seg[1]; first = false;
        if (g.nseg > 2 && t >= g.tiles_seg[1]) { t -= g.tiles_seg[1]; W = g.W[2]; n_seg = g.n_seg[2]; }
    }
    int n = min(t * BN + b, n_seg - 1);
    o.w = W + (size_t)n * g.K;
    o.kind = (first && g.T && g.B[0]) ? 1 : 0;
    o.b = o.kind ? g.B[0] + (size_t)n * g.r : o.w;
    return o;
}

// 256 bytes of zeros: the source of LDS-direct loads that must read as zeros (adapter columns a
// row does not have, padding past the last adapter column).
__device__ uint4 g_zero_page[16];

// 16-byte LDS-direct load: lane i of the wave copies 16 bytes from its own global address g to LDS
// byte address lds_base + 16 i (lds_base wave-uniform).  The data bypasses the registers and the
// load stays in flight, counted by vmcnt, until it has been written to LDS.  Written as inline
// assembly so that the compiler does not tie later LDS reads to it with a full vmcnt(0) wait: the
// pipeline below waits explicitly.  m0 carries the LDS base; nothing else in these kernels uses m0.
__device__ __forceinline__ void dma16(const void *g, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(g) : "memory");
}

// s_waitcnt immediate (gfx9 encoding) for vmcnt <= N and lgkmcnt == 0: all LDS reads of the wave
// have returned and at most N of its global loads are still in flight.
constexpr int waitcnt_vm_lgkm0(int n) { return (n & 15) | (7 << 4) | (0 << 8) | ((n >> 4) << 14); }

template <int N>
__device__ __forceinline__ void wait_loads() { __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(N)); }

// Byte offset of 16-byte chunk c of tile row `row` inside an operand's LDS stage.  Rows are stored
// densely (CPR chunks each); inside every 256-byte line (one pass over the 64 banks) the chunk
// position is XOR-ed with the low bits of the line number, so that the 16-byte fragment reads of
// 16 consecutive rows, which the LDS serves together, fall into 16 different bank groups.
template <int CPR>
__device__ __forceinline__ int swz(int row, int c) {
    int q = row * CPR + c, line = q >> 4, p = q & 15;
    return (line << 8) + ((p ^ (line & (CPR - 1))) << 4);
}

template <int BM, int BN, int BK, int NS, int WAVES_M, int WAVES_N>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N) k_gemm_mfma(GemmArgs g) {
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;            // 32x32 MFMA tiles per wave
    constexpr int CPR = BK / 8;                          // 16-byte chunks per tile row
    constexpr int RPU = 64 / CPR;                        // tile rows per 1 KiB unit (one wave-wide load)
    constexpr int A_LD = BM / RPU / NW, B_LD = BN / RPU / NW;  // loads per wave and slab
    constexpr int NL = A_LD + B_LD;
    constexpr int kBOff = BM * BK * 2, kStage = (BM + BN) * BK * 2;
    static_assert(BM % (RPU * NW) == 0 && BN % (RPU * NW) == 0, "tile / wave mismatch");
    static_assert(TM >= 1 && TN >= 1 && NS >= 2 && NS <= 5 && (NS - 2) * NL < 64, "tile shape");
    extern __shared__ __attribute__((aligned(1024))) char smem[];  // [NS] stages of { A [BM][BK], B [BN][BK] }
    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) char *)smem;

    // XCD-aware tile order.  The 8 XCDs take workgroups round-robin and each runs about 32 of them
    // at a time (one per CU).  The tile grid is cut into panels of panel_m x panel_n <= run tiles
    // (run = 32 for a grid that fills the chip, less for small ones so that every XCD gets work);
    // `run` consecutive workgroups of one XCD work on one panel, so that what they stream through
    // that XCD's L2 at any moment is panel_m slabs of X and panel_n slabs of W instead of run + 1.
    // Consecutive panels (on different XCDs at the same time) walk down the rows first, sharing
    // their weight columns in the memory-side cache.
    const int Mt = g.m_tiles, Nt = g.n_tiles;
    int tile_m, tile_n;
    {
        const int bid = blockIdx.x, xcd = bid & 7, s = bid >> 3;
        const int panel = (s / g.run) * 8 + xcd, within = s % g.run;
        if (panel >= g.n_panels || within >= g.panel_m * g.panel_n) return;
        tile_m = (panel % g.panels_m) * g.panel_m + within % g.panel_m;
        tile_n = (panel / g.panels_m) * g.panel_n + within / g.panel_m;
        if (tile_m >= Mt || tile_n >= Nt) return;
    }
    const int kz = blockIdx.y;  // split-K slice
    const int k_begin = kz * g.k_per_split;
    const int k_end = min(g.K_ext, k_begin + g.k_per_split);
    const int nk = (k_end - k_begin + BK - 1) / BK;

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w / WAVES_N, wn = w % WAVES_N;
    const int row0 = tile_m * BM;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // This lane's part of every wave-wide load: LDS slot `lane` of a 1 KiB unit is 256-byte line
    // lane/16, position lane%16, which (un-swizzled) holds chunk kc/8 of unit row ru.  A wave's units
    // are NW apart (NW even), so the swizzle key of its lines is the same for every unit.  Row
    // sources are fixed for the whole K loop: base-K slabs read pointer + k, the few adapter slabs
    // past K read T (activation side) and the models' B (weight side), or the zero page.
    static_assert(NW % 2 == 0, "swizzle key must not depend on the unit");
    const int lin = lane >> 4, key = (w * 4 + lin) & (CPR - 1);
    const int qd = lin * 16 + ((lane & 15) ^ key);
    const int ru = qd / CPR, kc = (qd % CPR) * 8;
    const bf16_t *zero = (const bf16_t *)g_zero_page;
    const bf16_t *pa[A_LD], *pt[A_LD];
    BRow br[B_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        int row = min(row0 + (w + NW * i) * RPU + ru, g.R - 1);  // clamped rows feed outputs that are never stored
        pa[i] = g.X + (size_t)row * g.ldx + kc;
        pt[i] = g.T ? g.T + (size_t)row * g.ldt + kc : zero;
    }
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        br[i] = b_row<BN, WN>(g, tile_n, (w + NW * i) * RPU + ru);
        br[i].w += kc;
    }
    const int K_base = g.K, mr = g.M_models * g.r, lr = 31 - __clz(max(g.r, 1)), ldt = g.T ? g.ldt : 0;
    const int rmask = g.r - 1;
    const size_t model_stride = (size_t)g.n_seg[0] * g.r;  // elements between consecutive models' B

    // enqueue the loads of slab kt into ring stage `stage`
    auto issue = [&](int kt, int stage) {
        const int k0 = k_begin + kt * BK;
        const uint32_t la = lds0 + stage * kStage + w * 1024;
        if (k0 < K_base) {  // slab inside the base weights (K is a multiple of the slab)
#pragma unroll
            for (int i = 0; i < A_LD; ++i) dma16(pa[i] + k0, la + i * (NW * 1024));
#pragma unroll
            for (int i = 0; i < B_LD; ++i) dma16(br[i].w + k0, la + kBOff + i * (NW * 1024));
            return;
        }
        const int k2 = k0 - K_base + kc;  // this lane's adapter column (r is a power of two)
#pragma unroll
        for (int i = 0; i < A_LD; ++i) dma16(k2 < ldt ? pt[i] + (k2 - kc) : zero, la + i * (NW * 1024));
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            int kk = k2 - (br[i].kind == 2 ? mr : 0);
            bool ok = br[i].kind != 0 && kk >= 0 && kk < mr;
            dma16(ok ? br[i].b + (size_t)(kk >> lr) * model_stride + (kk & rmask) : zero, la + kBOff + i * (NW * 1024));
        }
    };

    const int fr = lane & 31, fh = lane >> 5;
    constexpr int KS = BK / 16;
    static_assert(KS % 2 == 0, "the two fragment sets alternate over the K steps of a slab");
    // Two fragment sets used alternately: while the MFMAs of one K step run from one set, the reads of
    // the next step fill the other.  A wave issues in order and an MFMA holds the issue slot until the
    // matrix pipe takes it, so the reads must be issued BEFORE the MFMAs they are to overlap with; the
    // compiler, left alone, sinks them behind the MFMAs to save the second set (measured on a bare loop:
    // 63 % of the matrix pipe's rate with 4 waves per CU, 87 % with the order pinned), hence the
    // scheduling barriers.
    bf16x8 fa[2][TM], fb[2][TN];
    auto read_frags = [&](int stage, int ks, bf16x8 (&af)[TM], bf16x8 (&bfr)[TN]) {
        const char *sA = smem + stage * kStage, *sB = sA + kBOff;
#pragma unroll
        for (int i = 0; i < TM; ++i) af[i] = *(const bf16x8 *)(sA + swz<CPR>(wm * WM + i * 32 + fr, 2 * ks + fh));
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[j] = *(const bf16x8 *)(sB + swz<CPR>(wn * WN + j * 32 + fr, 2 * ks + fh));
    };
    auto mma = [&](const bf16x8 (&af)[TM], const bf16x8 (&bfr)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    };
    // K steps 0 .. KS-2 of the slab in `stage`; set 0 holds step 0 on entry, set 1 holds step KS-1 on exit.
    // A wave issues in order, and an LDS read that the LDS cannot take yet blocks the MFMAs behind it while the
    // matrix pipe runs dry; so each fragment read of the next step sits right behind an MFMA of this one, whose
    // passes cover it (a batch of reads ahead of the MFMAs cost the sum of both).
    auto slab_head = [&](int stage) {
        const char *sA = smem + stage * kStage, *sB = sA + kBOff;
#pragma unroll
        for (int ks = 0; ks + 1 < KS; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
#pragma unroll
            for (int m = 0; m < TM * TN; ++m) {
                const int i = m / TN, j = m % TN;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
                if (TM * TN >= TM + TN) {
                    if (m < TM) fa[nxt][m] = *(const bf16x8 *)(sA + swz<CPR>(wm * WM + m * 32 + fr, 2 * (ks + 1) + fh));
                    else if (m < TM + TN) fb[nxt][m - TM] = *(const bf16x8 *)(sB + swz<CPR>(wn * WN + (m - TM) * 32 + fr, 2 * (ks + 1) + fh));
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (TM * TN < TM + TN) read_frags(stage, ks + 1, fa[nxt], fb[nxt]);  // tiles with fewer MFMAs than fragments
        }
    };
    auto wait_for_slab = [&](int younger) {  // younger: slabs enqueued after the one waited for
        if (NS > 4 && younger >= 3) wait_loads<(NS > 4 ? 3 : 0) * NL>();
        else if (NS > 3 && younger >= 2) wait_loads<(NS > 3 ? 2 : 0) * NL>();
        else if (younger >= 1) wait_loads<NL>();
        else wait_loads<0>();
    };
    // Ring of NS stages.  One barrier per slab, placed before the last 16-wide K step of slab kt is
    // multiplied: by then every wave has read all of slab kt into registers, so after the barrier
    // (which also follows each wave's wait for its own loads of slab kt+1) slab kt+1 is complete
    // in LDS and the stage of slab kt can be refilled with slab kt+NS.  The first fragments of slab
    // kt+1 are fetched right after the barrier and the pending MFMAs of slab kt cover their latency,
    // the refill's issue and the barrier's wake-up.
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < nk) issue(s, s);
    wait_for_slab(min(NS - 2, nk - 1));
    __builtin_amdgcn_s_barrier();
    if (NS - 1 < nk) issue(NS - 1, NS - 1);
    read_frags(0, 0, fa[0], fb[0]);
    int stage = 0, kt = 0;
    // Steady state: the slab to enqueue (kt+NS) lies in the base weights, so the section after the
    // barrier is straight-line code: the first fragments of slab kt+1, then the pending MFMAs of slab
    // kt alternating with the loads of slab kt+NS, so that the matrix pipe is fed while the wave
    // issues its memory instructions.
    const int n_steady = min(nk, max(0, (K_base - k_begin) / BK)) - NS;
    for (; kt < n_steady; ++kt) {
        slab_head(stage);
        const int next = stage + 1 == NS ? 0 : stage + 1;
        wait_loads<(NS - 2) * NL>();
        __builtin_amdgcn_s_barrier();
        read_frags(next, 0, fa[0], fb[0]);
        const int k0 = k_begin + (kt + NS) * BK;
        const uint32_t la = lds0 + stage * kStage + w * 1024;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < TM * TN; ++t) {
            acc[t / TN][t % TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[1][t / TN], fb[1][t % TN], acc[t / TN][t % TN], 0, 0, 0);
#pragma unroll
            for (int l = t * NL / (TM * TN); l < (t + 1) * NL / (TM * TN); ++l) {
                if (l < A_LD) dma16(pa[l] + k0, la + l * (NW * 1024));
                else dma16(br[l - A_LD].w + k0, la + kBOff + (l - A_LD) * (NW * 1024));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        stage = next;
    }
    for (; kt < nk; ++kt) {  // the last slabs: adapter columns to enqueue, or nothing left to enqueue
        slab_head(stage);
        const int next = stage + 1 == NS ? 0 : stage + 1;
        if (kt + 1 < nk) {
            wait_for_slab(min(NS - 2, nk - 2 - kt));
            __builtin_amdgcn_s_barrier();
            read_frags(next, 0, fa[0], fb[0]);
            __builtin_amdgcn_sched_barrier(0);
            if (kt + NS < nk) issue(kt + NS, stage);
        }
        mma(fa[1], fb[1]);
        __builtin_amdgcn_sched_barrier(0);
        stage = next;
    }

    // Epilogue.  Accumulator register r of MFMA tile (i, j) is row 8(r/4) + 4(lane/32) + r%4, column
    // lane%32: a lane owns single columns, which would make 2-byte stores.  Each wave therefore turns
    // 32 rows of its tile at a time through its own slice of the (now dead) ring, and reads them back
    // row-major, 8 columns per lane, for 16- and 32-byte global accesses.
    __syncthreads();  // every wave has left the K loop
    constexpr bool kMayBeDual = TN % 2 == 0;
    const bool dual = kMayBeDual && g.mode == GEMM_DUAL;
    constexpr int kEs = WN + 8;  // scratch row stride in floats: rows 4 apart fall into different bank halves
    static_assert(NW * 32 * kEs * 4 <= NS * kStage, "epilogue scratch must fit the ring");
    float *scr = (float *)smem + w * 32 * kEs;
    const int col_l = lane & 31, row_l = (lane >> 5) * 4;
    int seg = 0, t = tile_n, col_base = 0;
    if (!dual)
        while (seg + 1 < g.nseg && t >= g.tiles_seg[seg]) { t -= g.tiles_seg[seg]; col_base += g.n_seg[seg]; ++seg; }
    const int wcols = dual ? WN / 2 : WN;                                   // output columns of this wave
    const int n_wave = dual ? tile_n * (BN / 2) + wn * (WN / 2) : t * BN + wn * WN;  // first of them, inside the segment
    const int n_lim = g.n_seg[dual ? 0 : seg];
    const int lpr = wcols / 8, rpp = 64 / lpr;                              // lanes per row, rows per pass
    const int rr0 = lane / lpr, c8 = (lane % lpr) * 8;
    // The residual rows of the next 32-row group are requested before this group is turned through
    // LDS, so that their latency (HBM: another kernel wrote them) is not paid once per pass.
    constexpr int kPasses = WN / 16;  // passes over a 32-row group when the wave's columns are all outputs
    const bool with_resid = !dual && g.epi != EPI_F32;
    uint4 rres[2][kPasses];
    auto load_resid = [&](int i, uint4 (&dst)[kPasses]) {
#pragma unroll
        for (int p = 0; p < kPasses; ++p) {
            const int row = row0 + wm * WM + i * 32 + rr0 + p * rpp, n_in = n_wave + c8;
            dst[p] = (row < g.R && n_in < n_lim) ? *(const uint4 *)(g.resid + (size_t)row * g.ldr + col_base + n_in) : make_uint4(0u, 0u, 0u, 0u);
        }
    };
    if (with_resid) load_resid(0, rres[0]);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        if (with_resid && i + 1 < TM) load_resid(i + 1, rres[(i + 1) & 1]);
        if (dual) {
            if constexpr (kMayBeDual) {
#pragma unroll
                for (int j = 0; j < TN / 2; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float gt = acc[i][j][r], up = acc[i][j + TN / 2][r];
                        scr[(8 * (r >> 2) + row_l + (r & 3)) * kEs + j * 32 + col_l] = gt * __builtin_amdgcn_rcpf(1.f + __expf(-gt)) * up;  // 1 ulp reciprocal: the result is rounded to bf16
                    }
            }
        } else {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) scr[(8 * (r >> 2) + row_l + (r & 3)) * kEs + j * 32 + col_l] = acc[i][j][r];
        }
#pragma unroll
        for (int p = 0; p < kPasses; ++p) {
            const int rr = rr0 + p * rpp;
            if (rr >= 32) break;  // the fused gate/up tile has half the output columns: half the passes
            const int row = row0 + wm * WM + i * 32 + rr, n_in = n_wave + c8;
            if (row >= g.R || n_in >= n_lim) continue;  // output widths are multiples of 8
            const float4 a = *(const float4 *)(scr + rr * kEs + c8), b = *(const float4 *)(scr + rr * kEs + c8 + 4);
            float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
            const int n = col_base + n_in;
            if (!dual && g.epi == EPI_F32) {
                float *yp = (float *)g.Y + ((size_t)kz * g.R + row) * g.ldy + n;
                *(float4 *)yp = a;
                *(float4 *)(yp + 4) = b;
                continue;
            }
            if (!dual) {  // EPI_BF16_RESID
                const uint4 rv = rres[i & 1][p];
                const uint32_t rw[4] = {rv.x, rv.y, rv.z, rv.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[2 * e] += __uint_as_float(rw[e] << 16);
                    v[2 * e + 1] += __uint_as_float(rw[e] & 0xffff0000u);
                }
            }
            uint4 o;
            o.x = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
            o.y = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
            o.z = (uint32_t)f32_to_bf16(v[4]) | ((uint32_t)f32_to_bf16(v[5]) << 16);
            o.w = (uint32_t)f32_to_bf16(v[6]) | ((uint32_t)f32_to_bf16(v[7]) << 16);
            *(uint4 *)((bf16_t *)g.Y + (size_t)row * g.ldy + n) = o;
        }
    }
}

// Second pass of a split-K GEMM: sum the fp32 partials P[z][row][n] and apply the epilogue.
__global__ void __launch_bounds__(256) k_splitk_reduce(const float *__restrict__ P, int splits, int R, int N, int epi,
                                                       void *__restrict__ Y, int ldy, const bf16_t *__restrict__ resid, int ldr) {
    size_t idx = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (idx >= (size_t)R * N) return;
    int row = (int)(idx / N), n = (int)(idx % N);  // N is a multiple of 4
    float4 v = {0.f, 0.f, 0.f, 0.f};
    for (int z = 0; z < splits; ++z) {
        float4 p = *(const float4 *)(P + ((size_t)z * R + row) * N + n);
        v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    if (epi == EPI_F32) {
        *(float4 *)((float *)Y + (size_t)row * ldy + n) = v;
    } else {
        const bf16_t *rp = resid + (size_t)row * ldr + n;
        bf16_t *yp = (bf16_t *)Y + (size_t)row * ldy + n;
        yp[0] = f32_to_bf16(v.x + bf16_to_f32(rp[0]));
        yp[1] = f32_to_bf16(v.y + bf16_to_f32(rp[1]));
        yp[2] = f32_to_bf16(v.z + bf16_to_f32(rp[2]));
        yp[3] = f32_to_bf16(v.w + bf16_to_f32(rp[3]));
    }
}

// The matrix pipe alone: 8 independent accumulators per wave, operands fixed in registers.
__global__ void __launch_bounds__(256) k_bench_mfma(float *__restrict__ out, int iters) {
    const int lane = threadIdx.x & 63;
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)(0.001f * (float)((lane + e) % 7));
        b[e] = (__bf16)(0.002f * (float)((lane + 2 * e) % 5));
    }
    f32x16 acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[t], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[t][r];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

template <int BM, int BN, int BK, int NS, int WAVES_M, int WAVES_N>
hipError_t launch_cfg(GemmArgs g, hipStream_t st) {
    g.m_tiles = (g.R + BM - 1) / BM;
    g.n_tiles = 0;
    if (g.mode == GEMM_DUAL) {
        g.n_tiles = (g.n_seg[0] + BN / 2 - 1) / (BN / 2);
    } else {
        for (int s = 0; s < g.nseg; ++s) {
            g.tiles_seg[s] = (g.n_seg[s] + BN - 1) / BN;
            g.n_tiles += g.tiles_seg[s];
        }
    }
    g.run = std::max(1, std::min(32, g.m_tiles * g.n_tiles / 8));
    g.panel_m = std::min({g.m_tiles, 8, g.run});
    g.panel_n = g.run / g.panel_m;
    g.panels_m = (g.m_tiles + g.panel_m - 1) / g.panel_m;
    g.n_panels = g.panels_m * ((g.n_tiles + g.panel_n - 1) / g.panel_n);
    size_t shm = (size_t)NS * (BM + BN) * BK * sizeof(bf16_t);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_gemm_mfma<BM, BN, BK, NS, WAVES_M, WAVES_N>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((g.n_panels + 7) / 8 * 8 * g.run, g.splits);
    hipLaunchKernelGGL((k_gemm_mfma<BM, BN, BK, NS, WAVES_M, WAVES_N>), grid, dim3(64 * WAVES_M * WAVES_N), shm, st, g);
    return hipGetLastError();
}

// Tile shapes (rows x weight rows x K slab, ring stages, waves).  What bounds a tile is the bytes it
// pulls through the CU's vector memory path per MFMA cycle, 4096 (1/BM + 1/BN): 64 for 128 x 128
// (the path's peak), 32 for 256 x 256.  Many rows (prefill): 256 x 256.  Few rows (decode): every
// weight is used once, straight from HBM, and what counts is how the weight rows are fetched: 64-wide
// K slabs ask for whole 128-byte lines (32-wide slabs ask for every line twice, half each time, and
// stream at about 60% of the rate), the grid must fill 256 CUs, so tiles stay 128 wide in N and K is
// split, and the row tile is the smallest that covers the stacked rows in one or two tiles (64, 128,
// 192 rows), which keeps the activation re-reads and the ring small enough for two workgroups per CU.
enum TileKind { TILE_AUTO = 0, TILE_128, TILE_256x128, TILE_256x256_K64, TILE_192x128_N3, TILE_192x128_N2, TILE_64x128, TILE_192x256_W8, TILE_KINDS };
struct TileShape { int bm, bn, bk; };
constexpr TileShape kTileShape[TILE_KINDS] = {{0, 0, 0},      {128, 128, 64}, {256, 128, 32}, {256, 256, 64},
                                              {192, 128, 64}, {192, 128, 64}, {64, 128, 64}, {192, 256, 64}};

int n_tiles_for(const GemmArgs &g, int bm, int bn) {
    int m_tiles = (g.R + bm - 1) / bm, n_tiles = 0;
    if (g.mode == GEMM_DUAL) return m_tiles * ((g.n_seg[0] + bn / 2 - 1) / (bn / 2));
    for (int s = 0; s < g.nseg; ++s) n_tiles += (g.n_seg[s] + bn - 1) / bn;
    return m_tiles * n_tiles;
}

int pick_tile_unchecked(const GemmArgs &g) {
    if (g.tile > 0 && g.tile < TILE_KINDS) return g.tile;
    if (g.R >= 1024 && n_tiles_for(g, 256, 256) >= 192) return TILE_256x256_K64;  // enough large tiles for 256 CUs
    if (g.R <= 64) return TILE_64x128;
    if (g.R <= 128) return TILE_128;
    if (g.mode == GEMM_DUAL && g.R > 192 && g.R <= 256) return TILE_256x128;
    if (g.R <= 384) {
        if (g.mode != GEMM_DUAL) return TILE_192x128_N3;
        // The fused gate/up GEMM cannot split K.  Two 192 x 128 workgroups per CU, or, when that still fills the chip,
        // one 192 x 256 workgroup of 8 waves: the activation slab is written to LDS once for both halves (4 % faster).
        return n_tiles_for(g, 192, 256) >= 192 ? TILE_192x256_W8 : TILE_192x128_N2;
    }
    return TILE_128;
}

int pick_tile(const GemmArgs &g) {
    int kind = pick_tile_unchecked(g);
    return g.K % kTileShape[kind].bk ? TILE_128 : kind;  // K is a multiple of 64 at least
}

}  // namespace

bool gemm_mfma_supported(const Dims &dm, int K) {
    bool r_ok = dm.r == 0 || (dm.r >= 8 && (dm.r & (dm.r - 1)) == 0);  // adapter rank: a power of two >= 8
    // every output width must be a multiple of 8 (16-byte stores of the epilogue)
    bool n_ok = dm.d % 8 == 0 && dm.F % 8 == 0 && (dm.Hq * dm.D) % 8 == 0 && (dm.Hkv * dm.D) % 8 == 0;
    return dm.bf16 && K % kKAlign == 0 && r_ok && n_ok;
}

// Batches of a few hundred rows against a wide weight matrix (enough 192 x 256 tiles to fill the chip without
// splitting K: the fused gate/up projection, an LM head) take the register-staged decode kernel.  Narrow
// projections stay on the smaller LDS-direct tiles of this file: with 192 x 128 tiles they need half as many
// split-K slices, and the slices' fp32 partial sums are what their epilogues spend their time writing.
bool gemm_uses_decode(const GemmArgs &g) {
    return g.R > 128 && g.R < 1024 && g.tile == 0 && gemm_decode_supported(g) && gemm_decode_tiles(g) >= 160;
}

int gemm_mfma_max_splits(const GemmArgs &g) {
    if (gemm_uses_decode(g)) return std::max(1, gemm_decode_slabs(g) / 8);
    int k_ext = g.K + ((g.T && g.B[0]) ? g.M_models * g.r : 0);
    return std::max(1, k_ext / 256);
}

int gemm_mfma_tiles(const GemmArgs &g) {
    if (gemm_uses_decode(g)) return gemm_decode_tiles(g);
    int t = pick_tile(g);
    return n_tiles_for(g, kTileShape[t].bm, kTileShape[t].bn);
}

hipError_t launch_gemm_mfma(GemmArgs g, hipStream_t st) {
    if (g.R <= 0) return hipSuccess;
    if (gemm_uses_decode(g)) return launch_gemm_decode(g, st);
    if (g.mode == GEMM_DUAL)
        g.K_ext = g.K + (g.T ? 2 * g.M_models * g.r : 0);
    else
        g.K_ext = g.K + ((g.T && g.B[0]) ? g.M_models * g.r : 0);
    if (g.splits < 1) g.splits = 1;
    const int kind = pick_tile(g), bk = kTileShape[kind].bk;
    if (g.K % bk) return hipErrorInvalidValue;
    g.k_per_split = ((g.K_ext + g.splits - 1) / g.splits + bk - 1) / bk * bk;
    switch (kind) {
    case TILE_256x128: return launch_cfg<256, 128, 32, 4, 2, 2>(g, st);
    case TILE_256x256_K64: return launch_cfg<256, 256, 64, 2, 2, 4>(g, st);
    case TILE_192x128_N3: return launch_cfg<192, 128, 64, 3, 2, 2>(g, st);
    case TILE_192x128_N2: return launch_cfg<192, 128, 64, 2, 2, 2>(g, st);
    case TILE_64x128: return launch_cfg<64, 128, 64, 3, 2, 2>(g, st);
    case TILE_192x256_W8: return launch_cfg<192, 256, 64, 2, 2, 4>(g, st);
    default: return launch_cfg<128, 128, 64, 4, 2, 2>(g, st);
    }
}

hipError_t launch_splitk_reduce(const float *P, int splits, int R, int N, int epi, void *Y, int ldy, const void *resid,
                                int ldr, hipStream_t st) {
    size_t quads = (size_t)R * N / 4;
    if (!quads) return hipSuccess;
    hipLaunchKernelGGL(k_splitk_reduce, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, st, P, splits, R, N, epi, Y, ldy,
                       (const bf16_t *)resid, ldr);
    return hipGetLastError();
}

hipError_t launch_bench_mfma(float *out, int waves, int iters, hipStream_t st) {
    hipLaunchKernelGGL(k_bench_mfma, dim3(waves / 4), dim3(256), 0, st, out, iters);
    return hipGetLastError();
}

}  // namespace icarus

// ICaRusLinear for decode-sized batches (a few hundred stacked rows) on gfx950 matrix cores.
//
//   Y[R, N] = X[R, K] . W[N, K]^T  +  T[R, M*r] . Bcat[N, M*r]^T          (Alg. 2; T = masked LoRA shrink)
//
// At decode every weight element is used once per step, by all stacked rows together (Sec. 3.3: the shared
// parameters are loaded once for the encoder and all decoder streams), so the kernel is shaped around how the
// weights travel.  Measured on this GPU: a 16-byte-per-lane global load costs the address path of a CU about 21
// cycles when 8 adjacent lanes cover a whole 128-byte line, and about 85 cycles when the lanes of an instruction
// spread over 16 or 32 weight rows, as they would have to in order to land directly in matrix-core operand
// layout -- at a few hundred rows that is more than the MFMAs of the same K step take.  Both operands are
// therefore loaded coalesced (8 rows x 128 bytes per instruction), parked in registers while in flight -- two
// slabs ahead, which is what hides HBM latency -- written to swizzled LDS with ds_write_b128, and read back as
// fragments.  (LDS-direct loads would save the registers but occupy the LDS 2.4 times as long per byte.)
//
// Tile: 4 waves (one per SIMD, so each may hold 512 registers) as 2 x 2 over 192 rows x 256 weight rows; a wave
// owns 96 x 128 = 3 x 4 MFMA tiles of 32x32x16 (192 accumulator registers).  Per 16-wide K step the CU reads
// 4 x (96 + 128) x 32 B = 28 KB of fragments for 48 MFMAs; the square-ish wave tile is what keeps the LDS below
// the matrix pipe.  Rows beyond 192 go to further row blocks: the row blocks of one column tile sit next to each
// other on one XCD, so the second reads the weights from that XCD's L2.  Batches of at most 160 rows take a
// 160 x 256 tile instead, the four waves side by side with 160 x 64 = 5 x 2 MFMA tiles each: the same 28 KB of
// fragments for 40 MFMAs, fewer of them on rows that do not exist.
//
// Loads return in order, so everything a wave has in flight is kept at one distance (D = 2 slabs: the loads
// issued while slab i is multiplied are parked while slab i + D is), and every load is unconditional (past the
// end of the K range it re-reads valid data that meets weight rows of zeros): the number of loads between an
// issue and its use is then the same on every path and the compiler's wait counts are exact.  (Three slabs in
// flight -- three register sets and LDS stages, which the 160-row tile has room for -- were measured and are
// slower: at these sizes HBM serves the weight rows' 128-byte pieces no faster with more of them outstanding.)
// The adapter columns follow the base K range as extra slabs: the activation side reads T, the weight side the
// concatenation of all models' B (zeros for weight rows without an adapter).
#include <algorithm>
#include <type_traits>

#include "device_util.h"
#include "kernels.h"

namespace icarus {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;  // 16 bytes in flight (a native vector: stays in registers)

namespace {

// 16 bytes of zeros: weight-side chunks of adapter columns that a weight row does not have.
__device__ uint4 g_gd_zero[1];

constexpr int kBK = 64;          // K columns per slab: one 128-byte line per row
constexpr int kCPR = kBK / 8;    // 16-byte chunks per slab row

// Byte offset of 16-byte chunk c of slab row `row` inside an operand's LDS stage: rows stored densely, chunk
// positions XOR-ed with the 256-byte line number so that the fragment reads of 16 consecutive rows hit 16
// different bank groups.
__device__ __forceinline__ int swz(int row, int c) {
    int q = row * kCPR + c, line = q >> 4, p = q & 15;
    return (line << 8) + ((p ^ (line & (kCPR - 1))) << 4);
}

// All LDS traffic of this wave has completed, then the workgroup barrier.  One asm statement with a memory
// clobber: the compiler must neither move LDS accesses across it nor add a wait for the global loads that are
// meant to stay in flight across the barrier.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// a ? x : y for a wave-uniform condition, as arithmetic: the slab loop must stay free of branches
__device__ __forceinline__ const bf16_t *pick(bool a, const bf16_t *x, const bf16_t *y) {
    const uintptr_t m = (uintptr_t)0 - (uintptr_t)a;
    return (const bf16_t *)(((uintptr_t)x & m) | ((uintptr_t)y & ~m));
}
__device__ __forceinline__ int pick(bool a, int x, int y) {
    const int m = -(int)a;
    return (x & m) | (y & ~m);
}

// Shape of the kernel for TM x TN MFMA tiles per wave: a tall wave tile puts the four waves side by side, else they
// sit 2 x 2; D = slabs of loads in flight = register sets = LDS stages (the loop below is written for 2 or 3).
template <int TM, int TN>
struct GdShape {
    static constexpr int WVM = TM > TN ? 1 : 2, WVN = 4 / WVM;
    static constexpr int BM = 32 * TM * WVM, BN = 32 * TN * WVN;
    static constexpr int kStage = (BM + BN) * kBK * 2;
    static constexpr int D = 2;
};

template <int TM, int TN>  // MFMA tiles of a wave
__global__ void __launch_bounds__(256) k_gemm_decode(GemmArgs g) {
    using Shape = GdShape<TM, TN>;
    constexpr int WVM = Shape::WVM, WVN = Shape::WVN, BM = Shape::BM, BN = Shape::BN, D = Shape::D;
    constexpr int WNR = BN / WVN;  // weight rows of a wave column
    constexpr int KS = kBK / 16;
    constexpr int NA = BM * kCPR / 256, NB = BN * kCPR / 256;  // 16-byte chunks of a slab per thread: activations, weights
    constexpr int kBOff = BM * kBK * 2, kStage = Shape::kStage;
    static_assert(TN % 2 == 0 && KS % 2 == 0 && BM * kCPR % 256 == 0 && BN * kCPR % 256 == 0, "tile shape");
    extern __shared__ __attribute__((aligned(1024))) char smem[];  // D stages of { X [BM][64], W [BN][64] }; then the epilogue's scratch

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = w / WVN, wc = w % WVN;
    const int cl = lane & 31, half = lane >> 5;
    int tile_n, row_blk;
    {   // consecutive workgroups of one XCD: the row blocks of one column tile
        const int id = blockIdx.x, s = id >> 3;
        row_blk = s % g.m_tiles;
        tile_n = (s / g.m_tiles) * 8 + (id & 7);
        if (tile_n >= g.n_tiles) return;
    }
    const int kz = blockIdx.y;
    const int row0 = row_blk * BM;
    const bool dual = g.mode == GEMM_DUAL;

    int seg = 0, t = tile_n, col_base = 0;
    if (!dual)
        while (seg + 1 < g.nseg && t >= g.tiles_seg[seg]) { t -= g.tiles_seg[seg]; col_base += g.n_seg[seg]; ++seg; }
    const int n_lim = g.n_seg[dual ? 0 : seg];
    const bf16_t *zero = (const bf16_t *)g_gd_zero;
    const int mr = g.M_models * g.r, lr = 31 - __clz(max(g.r, 1)), rmask = g.r - 1;
    const int model_stride = g.n_seg[0] * g.r;  // elements between consecutive models' B
    const bool has_adp = g.T && (dual ? (g.B[0] || g.B[1]) : (seg == 0 && g.B[0]));  // this tile has adapter columns

    // K range of this workgroup, in slabs: the base weights, then (where this tile has adapters) the columns of T
    const int base_slabs = g.K / kBK;
    const int t_cols = has_adp ? g.ldt : 0;  // a multiple of 8
    const int total = base_slabs + (t_cols + kBK - 1) / kBK;
    const int sl_begin = kz * g.slabs_per_split;
    const int sl_end = min(total, sl_begin + g.slabs_per_split);  // <= sl_begin: this slice is all zeros

    // Loader: chunk i of this thread is slab row (tid / 8 + 32 i), 16-byte column c = tid % 8, of either operand.
    // Weight-tile row b: PLAIN weight row t * BN + b of the segment; DUAL: the tile covers BN / 2 output columns,
    // a wave column of WNR tile rows holds the gate rows of its WNR / 2 output columns, then their up rows.
    const int c = tid & 7, lrow = tid >> 3;
    int offx[NA], offt[NA], offw[NB], offb[NB];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int grow = min(row0 + lrow + 32 * i, g.R - 1);  // clamped rows are never stored
        offx[i] = grow * g.ldx + 8 * c;
        offt[i] = grow * g.ldt;
    }
    // chunk i holds tile rows lrow + 32 i: in a DUAL tile an up row exactly when i % TN >= TN / 2 (a wave column is TN
    // chunks long), so the matrix a chunk reads is known per i: two base pointers per operand, wave-uniform
    const bf16_t *Wlo = dual ? g.W[0] : g.W[seg], *Whi = dual ? g.W[1] : Wlo;
    const bf16_t *Blo = dual ? g.B[0] : (seg == 0 ? g.B[0] : nullptr), *Bhi = dual ? g.B[1] : Blo;
    const bool adp_lo = g.T && Blo, adp_hi = g.T && Bhi;
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int b = lrow + 32 * i;
        int n = dual ? tile_n * (BN / 2) + (b / WNR) * (WNR / 2) + b % (WNR / 2) : t * BN + b;
        n = min(n, n_lim - 1);  // clamped columns are never stored
        offw[i] = n * g.K + 8 * c;
        offb[i] = n * g.r;
    }
    const int ldsw = swz(lrow, c);  // chunk i lands 32 rows = 4096 bytes further

    // Chunk u of a slab: u < NA activation chunk u, else weight chunk u - NA.  Any slab index, branch-free: base
    // range -> X / W at column sl * 64; past it -> T / Bcat; columns past T's last, whole slabs past the end, and
    // weight rows without an adapter: finite activations against zero weights.
    const bf16_t *x_past = t_cols ? g.T : g.X + (size_t)(base_slabs - 1) * kBK + 8 * c;
    u32x4 xr[D][NA + NB];
    auto issue_chunk = [&](int sl, int u, u32x4 &dst) {
        const bool past = sl >= sl_end;  // the slab that rounds an odd count up; it may belong to the next K slice
        const bool xbase = sl < base_slabs, base = !past && xbase;
        const int t0 = (sl - base_slabs) * kBK + 8 * c;          // this thread's 8 columns of T
        if (u < NA) {
            const int tcol = t_cols ? max(0, min(t0, t_cols - 8)) : 0;
            const bf16_t *pa = pick(xbase, g.X + (size_t)sl * kBK, x_past);
            dst = *(const u32x4 *)(pa + pick(xbase, offx[u], (t_cols ? offt[u] : offx[u] - 8 * c) + tcol));
        } else {
            const int i = u - NA;
            const bool up = dual && (i % TN) >= TN / 2;
            const int kk = t0 - (up ? mr : 0);  // column inside this row's adapter range
            const bool ok = !past && !xbase && (up ? adp_hi : adp_lo) && t0 < t_cols && kk >= 0 && kk < mr;
            const bf16_t *pw = (up ? Whi : Wlo) + (size_t)sl * kBK + offw[i];
            const bf16_t *pb = (up ? Bhi : Blo) + ((kk >> lr) * model_stride + (kk & rmask) + offb[i]);
            dst = *(const u32x4 *)pick(base, pw, pick(ok, pb, zero));
        }
    };
    // the same for a slab inside the base K range
    auto issue_chunk_base = [&](int sl, int u, u32x4 &dst) {
        if (u < NA) dst = *(const u32x4 *)(g.X + (size_t)sl * kBK + offx[u]);
        else dst = *(const u32x4 *)((((u - NA) % TN) >= TN / 2 ? Whi : Wlo) + (size_t)sl * kBK + offw[u - NA]);
    };
    auto park_chunk = [&](int stage, int u, const u32x4 &src) {
        *(u32x4 *)(smem + stage * kStage + ldsw + (u < NA ? u * 4096 : kBOff + (u - NA) * 4096)) = src;
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    bf16x8 fa[2][TM], fb[2][TN];
    // fragment f of K step ks of the slab in `stage`: f < TM activation rows, else weight rows
    auto read_frag = [&](int stage, int ks, int f, bf16x8 (&a)[TM], bf16x8 (&b)[TN]) {
        const char *sA = smem + stage * kStage, *sB = sA + kBOff;
        if (f < TM) a[f] = *(const bf16x8 *)(sA + swz(wr * (BM / WVM) + f * 32 + cl, 2 * ks + half));
        else b[f - TM] = *(const bf16x8 *)(sB + swz(wc * WNR + (f - TM) * 32 + cl, 2 * ks + half));
    };

    if (sl_end > sl_begin) {
        // prologue: slabs 0 .. D-1 requested, slab 0 parked in stage 0, slab D requested, first fragments read
#pragma unroll
        for (int d = 0; d < D; ++d)
#pragma unroll
            for (int u = 0; u < NA + NB; ++u) issue_chunk(sl_begin + d, u, xr[d][u]);
#pragma unroll
        for (int u = 0; u < NA + NB; ++u) {
            park_chunk(0, u, xr[0][u]);
            issue_chunk(sl_begin + D, u, xr[0][u]);
        }
        lds_barrier();
#pragma unroll
        for (int f = 0; f < TM + TN; ++f) read_frag(0, 0, f, fa[0], fb[0]);
        // One slab, P = its index mod D: LDS stage P holds it, register set N = (P + 1) % D the next one (requested
        // D slabs ago).  A wave issues in order, and an instruction that the LDS or the memory path cannot take yet
        // blocks the MFMAs behind it while the matrix pipe runs dry; so every memory instruction sits right behind
        // an MFMA, whose 8 passes cover it: after the first TM + TN MFMAs of a K step the fragment reads of the next
        // step (two fragment sets alternate), after the others chunks of the next slab are parked in stage N --
        // free since the barrier of the previous slab -- and their registers reloaded with the slab D slabs after
        // the next.  The barrier precedes the last K step, whose fragment reads are the next slab's.
        auto slab = [&](int sl, auto Pc, auto hot) {
            constexpr int P = decltype(Pc)::value, N = (P + 1) % D;
            constexpr int kFree = TM * TN - (TM + TN);  // MFMAs of a K step that carry no fragment read
            constexpr int kPer = (NA + NB + kFree * (KS - 1) - 1) / (kFree * (KS - 1));  // chunks behind each of them
            static_assert(kFree > 0 && kPer <= 2, "not enough MFMAs per slab to carry its loads");
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks == KS - 1) lds_barrier();
                const int set = ks & 1;
#pragma unroll
                for (int m = 0; m < TM * TN; ++m) {
                    const int i = m / TN, j = m % TN;
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
                    if (m < TM + TN) {
                        if (ks + 1 < KS) read_frag(P, ks + 1, m, fa[set ^ 1], fb[set ^ 1]);
                        else read_frag(N, 0, m, fa[set ^ 1], fb[set ^ 1]);
                    } else if (ks + 1 < KS) {
#pragma unroll
                        for (int e = 0; e < kPer; ++e) {
                            const int u = (ks * kFree + (m - (TM + TN))) * kPer + e;
                            if (u < NA + NB) {
                                park_chunk(N, u, xr[N][u]);
                                if constexpr (decltype(hot)::value) issue_chunk_base(sl + D + 1, u, xr[N][u]);
                                else issue_chunk(sl + D + 1, u, xr[N][u]);
                            }
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        // slabs whose loads (D + 1 slabs ahead) stay inside the base K range of this slice, D at a time
        int sl = sl_begin;
        const int hot_end = sl_begin + max(0, min(sl_end, base_slabs) - (D + 1) - sl_begin) / D * D;
        for (; sl < hot_end; sl += D) {
            slab(sl, std::integral_constant<int, 0>(), std::true_type());
            slab(sl + 1, std::integral_constant<int, 1>(), std::true_type());
            if constexpr (D > 2) slab(sl + 2, std::integral_constant<int, 2>(), std::true_type());
        }
        // the rest in the general form, also D at a time: a count that is not a multiple of D is rounded up by slabs
        // of zero weights
        for (; sl < sl_end; sl += D) {
            slab(sl, std::integral_constant<int, 0>(), std::false_type());
            slab(sl + 1, std::integral_constant<int, 1>(), std::false_type());
            if constexpr (D > 2) slab(sl + 2, std::integral_constant<int, 2>(), std::false_type());
        }
    }

    // Epilogue.  Accumulator register r of MFMA tile (i, j) is row 8(r/4) + 4(lane/32) + r%4, column lane%32: a
    // lane owns single columns.  Each wave turns 32 rows at a time through its own slice of the (now dead) slab
    // stages and reads them back row-major, 8 columns per lane, for 16- and 32-byte global accesses.  DUAL: column
    // tiles 0 .. TN/2-1 are the gate, TN/2 .. TN-1 the up projection of the same columns.
    lds_barrier();  // every wave has left the K loop
    constexpr int WN = 32 * TN, kEs = WN + 8;  // scratch row stride in floats
    static_assert(4 * 32 * kEs * 4 <= D * kStage, "epilogue scratch must fit the slab stages");
    float *scr = (float *)smem + w * 32 * kEs;
    const int row_l = half * 4;
    const int wcols = dual ? WN / 2 : WN;                                         // output columns of this wave
    const int n_wave = dual ? tile_n * (BN / 2) + wc * (WN / 2) : t * BN + wc * WN;  // first of them, inside the segment
    const int lpr = wcols / 8, rpp = 64 / lpr;  // lanes per row, rows per pass
    const int rr0 = lane / lpr, c8 = (lane % lpr) * 8;
    constexpr int kPasses = WN / 16;  // passes over a 32-row group when the wave's columns are all outputs
    const bool with_resid = !dual && g.epi != EPI_F32;
    uint4 rres[2][kPasses];
    auto load_resid = [&](int i, uint4 (&dst)[kPasses]) {
#pragma unroll
        for (int p = 0; p < kPasses; ++p) {
            const int rr = rr0 + p * rpp, row = row0 + wr * (BM / WVM) + i * 32 + rr, nc = n_wave + c8;
            dst[p] = (rr < 32 && row < g.R && nc < n_lim) ? *(const uint4 *)(g.resid + (size_t)row * g.ldr + col_base + nc)
                                                            : make_uint4(0u, 0u, 0u, 0u);
        }
    };
    const int n_rows = g.R, ldy = g.ldy, n_in = n_wave + c8, n_out = col_base + n_in;
    const bool f32_out = !dual && g.epi == EPI_F32;
    float *const y32 = (float *)g.Y + (size_t)kz * n_rows * ldy + n_out;
    bf16_t *const y16 = (bf16_t *)g.Y + n_out;
    const int wrow0 = row0 + wr * (BM / WVM);  // first row of this wave
    if (with_resid) load_resid(0, rres[0]);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        if (wrow0 + i * 32 < n_rows) {  // row tiles past the last row hold nothing
            if (with_resid && i + 1 < TM) load_resid(i + 1, rres[(i + 1) & 1]);
            if (dual) {
#pragma unroll
                for (int j = 0; j < TN / 2; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float gt = acc[i][j][r], up = acc[i][j + TN / 2][r];
                        scr[(8 * (r >> 2) + row_l + (r & 3)) * kEs + j * 32 + cl] = gt * __builtin_amdgcn_rcpf(1.f + __expf(-gt)) * up;  // 1 ulp reciprocal: the result is rounded to bf16
                    }
            } else {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) scr[(8 * (r >> 2) + row_l + (r & 3)) * kEs + j * 32 + cl] = acc[i][j][r];
            }
#pragma unroll
            for (int p = 0; p < kPasses; ++p) {
                const int rr = rr0 + p * rpp, row = wrow0 + i * 32 + rr;
                // the fused gate/up tile has half the output columns: half the passes; output widths are multiples of 8
                if (rr < 32 && row < n_rows && n_in < n_lim) {
                    const float4 a = *(const float4 *)(scr + rr * kEs + c8), b = *(const float4 *)(scr + rr * kEs + c8 + 4);
                    if (f32_out) {
                        float *yp = y32 + (size_t)row * ldy;
                        *(float4 *)yp = a;
                        *(float4 *)(yp + 4) = b;
                    } else {
                        float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
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
                        *(uint4 *)(y16 + (size_t)row * ldy) = o;
                    }
                }
            }
        }
    }
}

template <int TM, int TN>
hipError_t launch_gd(GemmArgs g, hipStream_t st) {
    using Shape = GdShape<TM, TN>;
    constexpr int BM = Shape::BM, BN = Shape::BN;
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
    const int total = g.K / kBK + ((g.T ? g.ldt : 0) + kBK - 1) / kBK;
    if (g.splits < 1) g.splits = 1;
    g.slabs_per_split = (total + g.splits - 1) / g.splits;
    const size_t shm = (size_t)Shape::D * Shape::kStage;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_gemm_decode<TM, TN>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((g.n_tiles + 7) / 8 * 8 * g.m_tiles, g.splits);
    hipLaunchKernelGGL((k_gemm_decode<TM, TN>), grid, dim3(256), shm, st, g);
    return hipGetLastError();
}

constexpr int kGdBM = 192, kGdBN = 256, kGdBMSmall = 160;  // row tile; the smaller one where it covers every row

}  // namespace

bool gemm_decode_supported(const GemmArgs &g) {
    if (g.R <= 0 || g.K % kBK || g.K < kBK) return false;
    if (g.mode == GEMM_DUAL && g.nseg != 1) return false;
    if (g.T && (g.r < 8 || (g.r & (g.r - 1)) || g.ldt % 8)) return false;
    // 32-bit element offsets from one base per operand
    const size_t lim = (size_t)1 << 30;
    if ((size_t)g.R * std::max(g.ldx, g.ldt) >= lim) return false;
    for (int sg = 0; sg < (g.mode == GEMM_DUAL ? 1 : g.nseg); ++sg)
        if ((size_t)g.n_seg[sg] * g.K >= lim) return false;
    if (g.T && (size_t)g.M_models * g.n_seg[0] * g.r >= lim) return false;
    return true;
}

// Workgroups of one K slice.
int gemm_decode_tiles(const GemmArgs &g) {
    const int m_tiles = (g.R + kGdBM - 1) / kGdBM;
    if (g.mode == GEMM_DUAL) return m_tiles * ((g.n_seg[0] + kGdBN / 2 - 1) / (kGdBN / 2));
    int n = 0;
    for (int s = 0; s < g.nseg; ++s) n += (g.n_seg[s] + kGdBN - 1) / kGdBN;
    return m_tiles * n;
}

int gemm_decode_slabs(const GemmArgs &g) { return g.K / kBK + ((g.T ? g.ldt : 0) + kBK - 1) / kBK; }

hipError_t launch_gemm_decode(GemmArgs g, hipStream_t st) {
    if (!gemm_decode_supported(g)) return hipErrorInvalidValue;
    if (!g.T || !(g.B[0] || g.B[1])) { g.T = nullptr; g.ldt = 0; }
    return g.R <= kGdBMSmall ? launch_gd<5, 2>(g, st) : launch_gd<3, 4>(g, st);
}

}  // namespace icarus

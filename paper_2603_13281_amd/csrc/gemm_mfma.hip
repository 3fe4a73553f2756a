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
// Tiling: 256 threads = 4 waves as 2 x 2; workgroup tile 128 rows x BN columns; MFMA 32x32x16 bf16
// on 64 x (BN/2) wave tiles.  K advances BK at a time: 16-byte coalesced global loads land in a ring
// of PF register stages (so PF-1 slabs are in flight while one is computed), go to double-buffered
// LDS, and are read back as MFMA fragments.  LDS rows are padded by 16 bytes so that fragment reads
// (16 bytes per lane, 32 consecutive rows) are bank-conflict free.
//
// MFMA 32x32x16 bf16 operand layout (lane l): A[row l%32][k 8(l/32)..+7], B[k 8(l/32)..+7][col l%32],
// C[row 8(r/4) + 4(l/32) + r%4][col l%32] for accumulator register r = 0..15.
#include <cstdio>
#include <cstdlib>

#include "device_util.h"
#include "kernels.h"

namespace icarus {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

namespace {

constexpr int kBM = 128;
constexpr int kKAlign = 64;  // K of every GEMM is a multiple of this

__device__ __forceinline__ uint4 ldg16(const bf16_t *p) { return *(const uint4 *)p; }

// Per-thread description of one 16-byte load of the weight (B) tile, fixed for the whole K loop.
// Every address the loop forms from it is valid memory (rows and columns past the matrix are
// clamped to its last row / column: they only feed outputs that are never stored), so that loads
// are unconditional and many can be in flight; chunks that must read as zeros are masked after
// the load.
struct BRow {
    const bf16_t *w;   // weight row + chunk offset: base-K loads are w + k
    const bf16_t *b;   // adapter B of this output column: &B[0][n][0] + chunk offset inside a model
    int kind;          // 0: no adapter columns; 1: adapter range [0, M*r); 2: range [M*r, 2*M*r) (up rows)
};

template <int BN>
__device__ __forceinline__ BRow b_row(const GemmArgs &g, int tile_n, int b) {
    BRow o;
    if (g.mode == GEMM_DUAL) {
        // tile covers BN/2 output columns: LDS row b -> wave column b / (BN/2), j = gate/up, nn
        constexpr int HW = BN / 2;          // rows per wave column
        int wn = b / HW, j = (b % HW) / (HW / 2), nn = b % (HW / 2);
        int n = min(tile_n * (BN / 2) + wn * (HW / 2) + nn, g.n_seg[0] - 1);
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

__device__ __forceinline__ uint4 masked(uint4 v, bool ok) {
    uint32_t m = ok ? 0xffffffffu : 0u;
    return uint4{v.x & m, v.y & m, v.z & m, v.w & m};
}

template <int BN, int BK, int PF>
__global__ void __launch_bounds__(256) k_gemm_mfma(GemmArgs g) {
    constexpr int WN = BN / 2;        // wave tile columns
    constexpr int TN = WN / 32;       // 32-col MFMA tiles per wave
    constexpr int CPR = BK / 8;       // 16-byte chunks per tile row
    constexpr int A_LD = kBM * CPR / 256;  // 16-byte loads per thread for the A tile
    constexpr int B_LD = BN * CPR / 256;
    constexpr int kLd = BK + 8;       // LDS row stride in elements
    static_assert(A_LD >= 1 && B_LD >= 1, "tile too small for 256 threads");
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
    bf16_t *As = smem;                         // [2][kBM][kLd]
    bf16_t *Bs = smem + 2 * kBM * kLd;         // [2][BN][kLd]

    // XCD-aware tile order: the 8 XCDs take workgroups round-robin, so consecutive ids on one XCD
    // walk the row tiles of the same weight tile (weights stay in that XCD's L2).
    const int Mt = g.m_tiles, Nt = g.n_tiles;
    int bid = blockIdx.x, tile_m, tile_n;
    {
        int grp = bid / (8 * Mt), rem = bid % (8 * Mt);
        int ncols = min(8, Nt - grp * 8);       // weight tiles in this group of 8
        tile_n = grp * 8 + rem % ncols;
        tile_m = rem / ncols;
    }
    const int kz = blockIdx.y;                  // split-K slice
    const int k_begin = kz * g.k_per_split;
    const int k_end = min(g.K_ext, k_begin + g.k_per_split);
    const int nk = (k_end - k_begin + BK - 1) / BK;

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wm = w >> 1, wn = w & 1;
    const int row0 = tile_m * kBM;

    f32x16 acc[2][TN];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // This thread's 16-byte loads: row sources fixed for the whole K loop.  Base-K slabs are
    // pointer + k; the few adapter slabs past K read T (activations side) and the models' B.
    const bf16_t *pa[A_LD], *pt[A_LD];
    BRow br[B_LD];
    int kca[A_LD], kcb[B_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        int e = tid + i * 256, row = min(row0 + e / CPR, g.R - 1);
        kca[i] = (e % CPR) * 8;
        pa[i] = g.X + (size_t)row * g.ldx + kca[i];
        pt[i] = g.T ? g.T + (size_t)row * g.ldt + kca[i] : pa[i];
    }
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        int e = tid + i * 256;
        kcb[i] = (e % CPR) * 8;
        br[i] = b_row<BN>(g, tile_n, e / CPR);
        br[i].w += kcb[i];
    }
    const int K_base = g.K, mr = g.M_models * g.r, lr = 31 - __clz(max(g.r, 1)), ldt = g.T ? g.ldt : 0;
    const size_t model_stride = (size_t)g.n_seg[0] * g.r;  // elements between consecutive models' B
    uint4 ra[PF][A_LD], rb[PF][B_LD];
    auto gload = [&](int kt, uint4 (&qa)[A_LD], uint4 (&qb)[B_LD]) {
        const int k0 = k_begin + kt * BK;
        if (k0 < K_base) {  // slab inside the base weights (K is a multiple of the slab)
#pragma unroll
            for (int i = 0; i < A_LD; ++i) qa[i] = ldg16(pa[i] + k0);
#pragma unroll
            for (int i = 0; i < B_LD; ++i) qb[i] = ldg16(br[i].w + k0);
            return;
        }
        const int k2 = k0 - K_base;  // adapter slab (r is a power of two)
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            bool ok = k2 + kca[i] < ldt && k0 + kca[i] < k_end;
            qa[i] = masked(ldg16(ok ? pt[i] + k2 : pa[i]), ok);
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            int kk = k2 + kcb[i] - (br[i].kind == 2 ? mr : 0);
            bool ok = br[i].kind != 0 && kk >= 0 && kk < mr && k0 + kcb[i] < k_end;
            const bf16_t *p = br[i].b + (size_t)(kk >> lr) * model_stride + (kk & (g.r - 1));
            qb[i] = masked(ldg16(ok ? p : br[i].w), ok);
        }
    };
    auto sstore = [&](int buf, const uint4 (&qa)[A_LD], const uint4 (&qb)[B_LD]) {
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            int e = tid + i * 256, rr = e / CPR, kc = (e % CPR) * 8;
            *(uint4 *)(As + ((size_t)buf * kBM + rr) * kLd + kc) = qa[i];
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            int e = tid + i * 256, rr = e / CPR, kc = (e % CPR) * 8;
            *(uint4 *)(Bs + ((size_t)buf * BN + rr) * kLd + kc) = qb[i];
        }
    };

    // slab t lives in register stage t % PF from its load until it is stored to LDS buffer t & 1
#pragma unroll
    for (int p = 0; p < PF; ++p)
        if (p < nk) gload(p, ra[p], rb[p]);
    if (nk > 0) sstore(0, ra[0], rb[0]);
    __syncthreads();
    const int fr = lane & 31, fk = (lane >> 5) * 8;
    for (int kt0 = 0; kt0 < nk; kt0 += PF) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int kt = kt0 + p;
            if (kt < nk) {
                const int buf = kt & 1;
                if (kt + PF < nk) gload(kt + PF, ra[p], rb[p]);  // stage p was emptied into LDS one step ago
                const bf16_t *Ab = As + ((size_t)buf * kBM + wm * 64 + fr) * kLd + fk;
                const bf16_t *Bb = Bs + ((size_t)buf * BN + wn * WN + fr) * kLd + fk;
#pragma unroll
                for (int ks = 0; ks < BK / 16; ++ks) {
                    bf16x8 a0 = *(const bf16x8 *)(Ab + ks * 16);
                    bf16x8 a1 = *(const bf16x8 *)(Ab + 32 * kLd + ks * 16);
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        bf16x8 b = *(const bf16x8 *)(Bb + (size_t)j * 32 * kLd + ks * 16);
                        acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b, acc[0][j], 0, 0, 0);
                        acc[1][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b, acc[1][j], 0, 0, 0);
                    }
                }
                if (kt + 1 < nk) sstore(buf ^ 1, ra[(p + 1) % PF], rb[(p + 1) % PF]);
            }
            __syncthreads();
        }
    }

    // epilogue: accumulator register r of tile (i, j) is row 8(r/4) + 4(lane/32) + r%4, column lane%32
    const int col_l = lane & 31, row_l = (lane >> 5) * 4;
    if (g.mode == GEMM_DUAL) {
        // wave columns: tile j = 0 gate, j = 1 up (TN == 2), same output column
        if constexpr (TN == 2) {
            int n = tile_n * (BN / 2) + wn * (WN / 2) + col_l;
            if (n < g.n_seg[0]) {
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        int row = row0 + wm * 64 + i * 32 + 8 * (r >> 2) + row_l + (r & 3);
                        if (row < g.R) {
                            float gt = acc[i][0][r], up = acc[i][1][r];
                            float hv = gt / (1.f + __expf(-gt)) * up;
                            ((bf16_t *)g.Y)[(size_t)row * g.ldy + n] = f32_to_bf16(hv);
                        }
                    }
            }
        }
        return;
    }
    int seg = 0, t = tile_n, col_base = 0;
    while (seg + 1 < g.nseg && t >= g.tiles_seg[seg]) { t -= g.tiles_seg[seg]; col_base += g.n_seg[seg]; ++seg; }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        int n_in = t * BN + wn * WN + j * 32 + col_l;
        if (n_in >= g.n_seg[seg]) continue;
        int n = col_base + n_in;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int row = row0 + wm * 64 + i * 32 + 8 * (r >> 2) + row_l + (r & 3);
                if (row >= g.R) continue;
                float v = acc[i][j][r];
                if (g.epi == EPI_F32) {
                    ((float *)g.Y)[((size_t)kz * g.R + row) * g.ldy + n] = v;
                } else {  // EPI_BF16_RESID
                    v += bf16_to_f32(g.resid[(size_t)row * g.ldr + n]);
                    ((bf16_t *)g.Y)[(size_t)row * g.ldy + n] = f32_to_bf16(v);
                }
            }
    }
}

// T[row, c] = bf16(scale * sum_z P[z][row][c]) if c / r == model(row) else 0   (shrink epilogue)
__global__ void __launch_bounds__(256) k_lora_mask(const float *__restrict__ P, int splits, int R, int C, int r,
                                                   const int32_t *__restrict__ row_model, float scale,
                                                   bf16_t *__restrict__ T, int n_targets) {
    // C = n_targets * M * r columns; target t occupies columns [t*M*r, (t+1)*M*r)
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)R * C) return;
    int row = (int)(idx / C), c = (int)(idx % C);
    int per = C / n_targets;
    int j = (c % per) / r;
    float v = 0.f;
    if (row_model[row] == j) {
        for (int z = 0; z < splits; ++z) v += P[((size_t)z * R + row) * C + c];
        v *= scale;
    }
    T[idx] = f32_to_bf16(v);
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

template <int BN, int BK, int PF>
hipError_t launch_cfg(const GemmArgs &g, hipStream_t st) {
    size_t shm = (size_t)2 * (kBM + BN) * (BK + 8) * sizeof(bf16_t);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_gemm_mfma<BN, BK, PF>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid(g.m_tiles * g.n_tiles, g.splits);
    hipLaunchKernelGGL((k_gemm_mfma<BN, BK, PF>), grid, dim3(256), shm, st, g);
    return hipGetLastError();
}

// Pipeline shape: K slab width and register prefetch depth.  ICARUS_GEMM_CFG = "bk,pf" overrides
// the default for experiments.
int gemm_cfg() {
    static int cfg = -1;
    if (cfg < 0) {
        cfg = 641;
        if (const char *e = getenv("ICARUS_GEMM_CFG")) {
            int bk = 0, pf = 0;
            if (sscanf(e, "%d,%d", &bk, &pf) == 2) cfg = bk * 10 + pf;
        }
    }
    return cfg;
}

}  // namespace

bool gemm_mfma_supported(const Dims &dm, int K) {
    bool r_ok = dm.r == 0 || (dm.r >= 8 && (dm.r & (dm.r - 1)) == 0);  // adapter rank: a power of two >= 8
    return dm.bf16 && K % kKAlign == 0 && r_ok;
}

int gemm_mfma_tiles(const GemmArgs &g) {
    const int BN = 128;
    int m_tiles = (g.R + kBM - 1) / kBM, n_tiles = 0;
    if (g.mode == GEMM_DUAL) return m_tiles * ((g.n_seg[0] + BN / 2 - 1) / (BN / 2));
    for (int s = 0; s < g.nseg; ++s) n_tiles += (g.n_seg[s] + BN - 1) / BN;
    return m_tiles * n_tiles;
}

hipError_t launch_gemm_mfma(GemmArgs g, hipStream_t st) {
    if (g.R <= 0) return hipSuccess;
    const int BN = 128;
    g.m_tiles = (g.R + kBM - 1) / kBM;
    g.n_tiles = 0;
    if (g.mode == GEMM_DUAL) {
        g.n_tiles = (g.n_seg[0] + BN / 2 - 1) / (BN / 2);
        g.K_ext = g.K + (g.T ? 2 * g.M_models * g.r : 0);
    } else {
        for (int s = 0; s < g.nseg; ++s) {
            g.tiles_seg[s] = (g.n_seg[s] + BN - 1) / BN;
            g.n_tiles += g.tiles_seg[s];
        }
        g.K_ext = g.K + ((g.T && g.B[0]) ? g.M_models * g.r : 0);
    }
    if (g.splits < 1) g.splits = 1;
    g.k_per_split = ((g.K_ext + g.splits - 1) / g.splits + kKAlign - 1) / kKAlign * kKAlign;
    switch (gemm_cfg()) {
    case 642: return launch_cfg<128, 64, 2>(g, st);
    case 322: return launch_cfg<128, 32, 2>(g, st);
    default: return launch_cfg<128, 64, 1>(g, st);
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

hipError_t launch_lora_mask(const float *P, int splits, int R, int C, int r, const int32_t *row_model, float scale,
                            void *T, int n_targets, hipStream_t st) {
    size_t total = (size_t)R * C;
    if (!total) return hipSuccess;
    hipLaunchKernelGGL(k_lora_mask, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, P, splits, R, C, r, row_model, scale,
                       (bf16_t *)T, n_targets);
    return hipGetLastError();
}

}  // namespace icarus

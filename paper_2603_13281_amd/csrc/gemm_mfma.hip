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
// Tiling: 256 threads = 4 waves as 2 x 2; workgroup tile 128 rows x BN columns, K staged 64 at a
// time through double-buffered LDS (16-byte coalesced global loads -> registers -> LDS), MFMA
// 32x32x16 bf16 on 64 x (BN/2) wave tiles.  LDS rows are padded to 144 bytes so that fragment reads
// (16 bytes per lane, 32 consecutive rows) are bank-conflict free.
//
// MFMA 32x32x16 bf16 operand layout (lane l): A[row l%32][k 8(l/32)..+7], B[k 8(l/32)..+7][col l%32],
// C[row 8(r/4) + 4(l/32) + r%4][col l%32] for accumulator register r = 0..15.
#include "device_util.h"
#include "kernels.h"

namespace icarus {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

namespace {

constexpr int kBM = 128, kBK = 64;
constexpr int kLd = kBK + 8;  // LDS row stride in elements (144 bytes)

__device__ __forceinline__ uint4 ldg16(const bf16_t *p) { return *(const uint4 *)p; }

// Source row of LDS B-row `b` of this tile at extended-K position k (multiple of 8):
// returns a pointer to 8 consecutive bf16, or nullptr for zeros.
template <int BN>
__device__ __forceinline__ const bf16_t *b_src(const GemmArgs &g, int tile_n, int b, int k) {
    if (g.mode == GEMM_DUAL) {
        // tile covers BN/2 output columns: LDS row b -> wave column b / (BN/2), j = gate/up, nn
        constexpr int HW = BN / 2;          // rows per wave column
        int wn = b / HW, j = (b % HW) / (HW / 2), nn = b % (HW / 2);
        int n = tile_n * (BN / 2) + wn * (HW / 2) + nn;
        if (n >= g.n_seg[0]) return nullptr;
        if (k < g.K) return g.W[j] + (size_t)n * g.K + k;
        int k2 = k - g.K;                   // [0, r*M): gate adapters, [r*M, 2*r*M): up adapters
        int mr = g.M_models * g.r;
        if (k2 >= 2 * mr || (k2 >= mr) != (j == 1)) return nullptr;
        k2 -= j * mr;
        return g.B[j] + ((size_t)(k2 / g.r) * g.n_seg[0] + n) * g.r + k2 % g.r;
    }
    // plain: up to three weight segments stacked along N; tiles never straddle segments
    int seg = 0, t = tile_n;
    while (seg + 1 < g.nseg && t >= g.tiles_seg[seg]) { t -= g.tiles_seg[seg]; ++seg; }
    int n = t * BN + b;
    if (n >= g.n_seg[seg]) return nullptr;
    if (k < g.K) return g.W[seg] + (size_t)n * g.K + k;
    int k2 = k - g.K;
    if (seg != 0 || !g.B[0] || k2 >= g.M_models * g.r) return nullptr;
    return g.B[0] + ((size_t)(k2 / g.r) * g.n_seg[0] + n) * g.r + k2 % g.r;
}

// Source of A-row (activation row) at extended-K position k.
__device__ __forceinline__ const bf16_t *a_src(const GemmArgs &g, int row, int k) {
    if (row >= g.R) return nullptr;
    if (k < g.K) return g.X + (size_t)row * g.ldx + k;
    int k2 = k - g.K;
    if (!g.T || k2 >= g.ldt) return nullptr;
    return g.T + (size_t)row * g.ldt + k2;
}

template <int BN>
__global__ void __launch_bounds__(256) k_gemm_mfma(GemmArgs g) {
    constexpr int WN = BN / 2;        // wave tile columns
    constexpr int TN = WN / 32;       // 32-col MFMA tiles per wave
    constexpr int A_LD = kBM * kBK / 8 / 256;  // 16-byte loads per thread for the A tile (4)
    constexpr int B_LD = BN * kBK / 8 / 256;
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
    const int nk = (k_end - k_begin + kBK - 1) / kBK;

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

    uint4 ra[A_LD], rb[B_LD];
    // Row pointers of this thread's 16-byte loads at k = 0 (null: the row is outside the matrix).
    // Inside the base-K range a load is pointer + k; only the few adapter slabs past K take the
    // general source functions.
    const bf16_t *pa[A_LD], *pb[B_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        int e = tid + i * 256;
        pa[i] = a_src(g, row0 + (e >> 3), (e & 7) * 8);
    }
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        int e = tid + i * 256;
        pb[i] = b_src<BN>(g, tile_n, e >> 3, (e & 7) * 8);
    }
    auto gload = [&](int kt) {
        int k0 = k_begin + kt * kBK;
        if (k0 + kBK <= g.K) {  // whole slab inside the base weights (K is a multiple of the slab)
#pragma unroll
            for (int i = 0; i < A_LD; ++i) ra[i] = pa[i] ? ldg16(pa[i] + k0) : uint4{0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < B_LD; ++i) rb[i] = pb[i] ? ldg16(pb[i] + k0) : uint4{0, 0, 0, 0};
            return;
        }
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            int e = tid + i * 256, rr = e >> 3, kc = (e & 7) * 8;
            const bf16_t *p = (k0 + kc < k_end) ? a_src(g, row0 + rr, k0 + kc) : nullptr;
            ra[i] = p ? ldg16(p) : uint4{0, 0, 0, 0};
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            int e = tid + i * 256, rr = e >> 3, kc = (e & 7) * 8;
            const bf16_t *p = (k0 + kc < k_end) ? b_src<BN>(g, tile_n, rr, k0 + kc) : nullptr;
            rb[i] = p ? ldg16(p) : uint4{0, 0, 0, 0};
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            int e = tid + i * 256, rr = e >> 3, kc = (e & 7) * 8;
            *(uint4 *)(As + ((size_t)buf * kBM + rr) * kLd + kc) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            int e = tid + i * 256, rr = e >> 3, kc = (e & 7) * 8;
            *(uint4 *)(Bs + ((size_t)buf * BN + rr) * kLd + kc) = rb[i];
        }
    };

    if (nk > 0) {
        gload(0);
        sstore(0);
    }
    __syncthreads();
    const int fr = lane & 31, fk = (lane >> 5) * 8;
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) gload(kt + 1);
        const bf16_t *Ab = As + ((size_t)buf * kBM + wm * 64 + fr) * kLd + fk;
        const bf16_t *Bb = Bs + ((size_t)buf * BN + wn * WN + fr) * kLd + fk;
#pragma unroll
        for (int ks = 0; ks < kBK / 16; ++ks) {
            bf16x8 a0 = *(const bf16x8 *)(Ab + ks * 16);
            bf16x8 a1 = *(const bf16x8 *)(Ab + 32 * kLd + ks * 16);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                bf16x8 b = *(const bf16x8 *)(Bb + (size_t)j * 32 * kLd + ks * 16);
                acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b, acc[0][j], 0, 0, 0);
                acc[1][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b, acc[1][j], 0, 0, 0);
            }
        }
        if (kt + 1 < nk) sstore(buf ^ 1);
        __syncthreads();
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

template <int BN>
hipError_t launch_bn(const GemmArgs &g, hipStream_t st) {
    size_t shm = (size_t)2 * (kBM + BN) * kLd * sizeof(bf16_t);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_gemm_mfma<BN>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid(g.m_tiles * g.n_tiles, g.splits);
    hipLaunchKernelGGL(k_gemm_mfma<BN>, grid, dim3(256), shm, st, g);
    return hipGetLastError();
}

}  // namespace

bool gemm_mfma_supported(const Dims &dm, int K) { return dm.bf16 && K % kBK == 0 && (dm.r % 8 == 0); }

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
    g.k_per_split = ((g.K_ext + g.splits - 1) / g.splits + kBK - 1) / kBK * kBK;
    return launch_bn<128>(g, st);
}

int gemm_mfma_tiles(const GemmArgs &g) {
    const int BN = 128;
    int m_tiles = (g.R + kBM - 1) / kBM, n_tiles = 0;
    if (g.mode == GEMM_DUAL) return m_tiles * ((g.n_seg[0] + BN / 2 - 1) / (BN / 2));
    for (int s = 0; s < g.nseg; ++s) n_tiles += (g.n_seg[s] + BN - 1) / BN;
    return m_tiles * n_tiles;
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

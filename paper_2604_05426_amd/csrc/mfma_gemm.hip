// Fused frozen-weight GEMM + LoRA expand for bf16 on gfx950 MFMA.
//
// Forward (paper Sec. 5.1 / App. A.1, "fused base-output addition"): the paper runs the
// base GEMM, then a second GEMM Y = S_i B_i + Y_base that reloads the base tile.  Here the
// expand is folded into the base GEMM itself: after the contraction over k, the same
// accumulators take a few more MFMA steps over the rank dimension with operands
// s_i S_i (rows of the tile that belong to adapter i, zero elsewhere) and B_i, so Y is
// written exactly once and Y_base never exists in memory.  Row tiles are not aligned to
// segments; a tile that straddles several adapters runs one masked extension per adapter.
// Backward input gradient is the mirror image: dX = dY W^T, extended with dS_i and A_i^T.
//
// Tile 256 x 256 x 64, 4 wavefronts (2 x 2), each 128 x 128 = 4 x 4 MFMA 32x32x16 blocks,
// fp32 accumulators, LDS double-buffered.  The forward's W tile is [k][n] in memory, i.e.
// column-contiguous; it is staged row-major and read with the transposing LDS load.
#include "mfma_common.h"

namespace mlora {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int A_LD = BK + 8;     // 144-byte rows: conflict-free 128-bit fragment reads
constexpr int BNT_LD = BK + 8;   // [col][contraction] layout
constexpr int BNN_LD = BN + 32;  // [contraction][col] layout, 576-byte rows for the transposing reads
constexpr int A_TILE = BM * A_LD;
constexpr int B_TILE = BN * BNT_LD;
static_assert(B_TILE == BK * BNN_LD, "both B layouts share one buffer size");
constexpr int STAGE = A_TILE + B_TILE;

struct GemmArgs {
    const u16* Aop; int64_t lda;   // X [T,k] (fwd) or dY [T,n] (bwd)
    const u16* Bop; int64_t ldb;   // W [k,n]
    u16* C; int64_t ldc;           // Y [T,n] or dX [T,k]
    const u16* E;                  // ragged S (fwd) or dS (bwd)
    int32_t M, Ncols, Kdim;
    int32_t tiles_m, tiles_n;
    int32_t skip_base, skip_lora, accumulate;
    PlanView pv;
};

template <bool NN>
__device__ __forceinline__ void compute_stage(const u16* As, const u16* Bs, f32x16 (&acc)[4][4], int ksteps,
                                              int wm, int wn, int lane) {
    const int lm = lane & 31, h = lane >> 5;
    const int g = lane >> 4, j = lane & 15;
    for (int ks = 0; ks < ksteps; ++ks) {
        bf16x8 a[4], b[4];
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
            a[mb] = lds_read_frag(As + (wm * 128 + mb * 32 + lm) * A_LD + ks * 16 + h * 8);
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
            if (NN) {
                const u16* p = Bs + (ks * 16 + 8 * (g >> 1) + (j >> 2)) * BNN_LD + wn * 128 + nb * 32 +
                               16 * (g & 1) + 4 * (j & 3);
                b[nb] = lds_read_frag_tr(p, p + 4 * BNN_LD);
            } else {
                b[nb] = lds_read_frag(Bs + (wn * 128 + nb * 32 + lm) * BNT_LD + ks * 16 + h * 8);
            }
        }
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) acc[mb][nb] = mfma32(a[mb], b[nb], acc[mb][nb]);
    }
}

template <bool NN>
__global__ __launch_bounds__(256, 1) void fused_gemm_kernel(GemmArgs g) {
    __shared__ __attribute__((aligned(16))) u16 lds[2 * STAGE];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous run of
    // tiles and walk it in bands of 8 row tiles so that co-resident tiles share W / X panels
    // in that XCD's L2.
    const int total = g.tiles_m * g.tiles_n;
    const int per_xcd = (total + 7) / 8;
    int L = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (L >= total) return;
    constexpr int GM = 8;
    const int band = L / (GM * g.tiles_n);
    const int band_rows = min(GM, g.tiles_m - band * GM);
    const int in_band = L - band * GM * g.tiles_n;
    const int tm = band * GM + in_band % band_rows;
    const int tn = in_band / band_rows;
    const int m0 = tm * BM, n0 = tn * BN;

    f32x16 acc[4][4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mb][nb][i] = 0.f;

    // ---- contraction over the frozen weight ------------------------------------------
    if (!g.skip_base) {
        const int nk = (g.Kdim + BK - 1) / BK;
        uint4 ra[8], rb[8];
        auto gload = [&](int kt) {
            const int k0 = kt * BK;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                const int row = (tid >> 3) + 32 * jj, kc = tid & 7;
                const int grow = m0 + row, gk = k0 + kc * 8;
                ra[jj] = (grow < g.M && gk < g.Kdim)
                             ? *reinterpret_cast<const uint4*>(g.Aop + (int64_t)grow * g.lda + gk) : zero4();
                if (NN) {
                    const int krow = (tid >> 5) + 8 * jj, nc = tid & 31;
                    const int gkb = k0 + krow, gcol = n0 + nc * 8;
                    rb[jj] = (gkb < g.Kdim && gcol < g.Ncols)
                                 ? *reinterpret_cast<const uint4*>(g.Bop + (int64_t)gkb * g.ldb + gcol) : zero4();
                } else {
                    const int gcol = n0 + row;
                    rb[jj] = (gcol < g.Ncols && gk < g.Kdim)
                                 ? *reinterpret_cast<const uint4*>(g.Bop + (int64_t)gcol * g.ldb + gk) : zero4();
                }
            }
        };
        auto lstore = [&](int stage) {
            u16* As = lds + stage * STAGE;
            u16* Bs = As + A_TILE;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                const int row = (tid >> 3) + 32 * jj, kc = tid & 7;
                *reinterpret_cast<uint4*>(As + row * A_LD + kc * 8) = ra[jj];
                if (NN) {
                    const int krow = (tid >> 5) + 8 * jj, nc = tid & 31;
                    *reinterpret_cast<uint4*>(Bs + krow * BNN_LD + nc * 8) = rb[jj];
                } else {
                    *reinterpret_cast<uint4*>(Bs + row * BNT_LD + kc * 8) = rb[jj];
                }
            }
        };
        gload(0);
        lstore(0);
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            const int cur = kt & 1;
            if (kt + 1 < nk) gload(kt + 1);
            compute_stage<NN>(lds + cur * STAGE, lds + cur * STAGE + A_TILE, acc, BK / 16, wm, wn, lane);
            if (kt + 1 < nk) lstore(cur ^ 1);
            __syncthreads();
        }
    }

    // ---- rank extension: one masked pass per adapter that owns rows of this tile -----------
    if (!g.skip_lora) {
        const Entry4 tile = g.pv.gemm_tiles[tm];
        u16* As = lds;
        u16* Bs = lds + A_TILE;
        for (int i = tile.c; i < tile.d; ++i) {
            const int r = g.pv.rank[i];
            if (r == 0) continue;
            const int seg0 = g.pv.off[i], seg1 = g.pv.off[i + 1];
            const int lo = max(seg0, m0), hi = min(seg1, m0 + BM);
            if (lo >= hi) continue;
            const int64_t so = g.pv.soff[i];
            const float s = NN ? g.pv.scale[i] : 1.0f;
            const u16* F = (const u16*)(NN ? g.pv.ptrs[i].B : g.pv.ptrs[i].A);
            const bool e_vec = ((r & 7) == 0) && ((so & 7) == 0);
            const bool f_vec = NN ? true : ((r & 7) == 0);
            for (int r0 = 0; r0 < r; r0 += BK) {
                const int rc = min(BK, r - r0);
                const int rpad = (rc + 15) & ~15;
                __syncthreads();
                {   // rows of s_i S_i (or dS_i) owned by adapter i, zero elsewhere
                    const int t = m0 + tid;
                    const bool own = (t >= lo && t < hi);
                    const u16* src = g.E + so + (int64_t)(t - seg0) * r + r0;
                    for (int cc = 0; cc < rpad / 8; ++cc) {
                        uint4 v = zero4();
                        if (own) {
                            v = load_chunk(src + cc * 8, min(8, rc - cc * 8), e_vec);
                            if (s != 1.0f) v = scale_chunk(v, s);
                        }
                        *reinterpret_cast<uint4*>(As + tid * A_LD + cc * 8) = v;
                    }
                }
                if (NN) {   // B_i rows r0.., columns of this tile
                    for (int jj = 0; jj < rpad / 8; ++jj) {
                        const int krow = (tid >> 5) + 8 * jj, nc = tid & 31;
                        const int gcol = n0 + nc * 8;
                        uint4 v = zero4();
                        if (krow < rc && gcol < g.Ncols)
                            v = *reinterpret_cast<const uint4*>(F + (int64_t)(r0 + krow) * g.Ncols + gcol);
                        *reinterpret_cast<uint4*>(Bs + krow * BNN_LD + nc * 8) = v;
                    }
                } else {    // A_i rows = output columns of this tile, contraction over the rank
                    const int gcol = n0 + tid;
                    const u16* src = F + (int64_t)gcol * r + r0;
                    for (int cc = 0; cc < rpad / 8; ++cc) {
                        uint4 v = zero4();
                        if (gcol < g.Ncols) v = load_chunk(src + cc * 8, min(8, rc - cc * 8), f_vec);
                        *reinterpret_cast<uint4*>(Bs + tid * BNT_LD + cc * 8) = v;
                    }
                }
                __syncthreads();
                compute_stage<NN>(As, Bs, acc, rpad / 16, wm, wn, lane);
            }
        }
    }

    // ---- store: one rounding from the fp32 accumulator ------------------------------------
    const int lm = lane & 31, h = lane >> 5;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
            const int col = n0 + wn * 128 + nb * 32 + lm;
            if (col >= g.Ncols) continue;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int row = m0 + wm * 128 + mb * 32 + (i >> 2) * 8 + h * 4 + (i & 3);
                if (row >= g.M) continue;
                u16* c = g.C + (int64_t)row * g.ldc + col;
                float v = acc[mb][nb][i];
                if (g.accumulate) v += bf2f(*c);
                *c = f2bf(v);
            }
        }
}

static int launch_gemm(mlora_plan* p, bool fwd, const void* Aop, const void* W, void* C, const void* E,
                       uint32_t flags, hipStream_t st) {
    if (p->T == 0) return MLORA_OK;
    GemmArgs g{};
    g.Aop = (const u16*)Aop;
    g.Bop = (const u16*)W;
    g.ldb = p->n;
    g.C = (u16*)C;
    g.E = (const u16*)E;
    g.M = (int32_t)p->T;
    if (fwd) { g.lda = p->k; g.ldc = p->n; g.Ncols = (int32_t)p->n; g.Kdim = (int32_t)p->k; }
    else     { g.lda = p->n; g.ldc = p->k; g.Ncols = (int32_t)p->k; g.Kdim = (int32_t)p->n; }
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.Ncols + BN - 1) / BN;
    g.skip_base = (flags & MLORA_FLAG_LORA_ONLY) ? 1 : 0;
    g.skip_lora = ((flags & MLORA_FLAG_BASE_ONLY) || p->N == 0) ? 1 : 0;
    g.accumulate = g.skip_base;
    g.pv = p->view;
    const int total = g.tiles_m * g.tiles_n;
    const int grid = ((total + 7) / 8) * 8;
    ProfScope prof(p, fwd ? MLORA_K_GEMM_FWD : MLORA_K_GEMM_BWD, st);
    if (fwd) hipLaunchKernelGGL(fused_gemm_kernel<true>, dim3(grid), dim3(256), 0, st, g);
    else     hipLaunchKernelGGL(fused_gemm_kernel<false>, dim3(grid), dim3(256), 0, st, g);
    MLORA_HIP_TRY(hipGetLastError());
    return MLORA_OK;
}

int mfma_gemm_fwd(mlora_plan* p, const void* X, const void* W, void* Y, const void* S, uint32_t flags,
                  hipStream_t st) {
    return launch_gemm(p, true, X, W, Y, S, flags, st);
}

int mfma_gemm_bwd(mlora_plan* p, const void* dY, const void* W, void* dX, const void* dS, uint32_t flags,
                  hipStream_t st) {
    return launch_gemm(p, false, dY, W, dX, dS, flags, st);
}

}  // namespace mlora

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
// Tile 256 x 256 x 64, 8 wavefronts (2 x 4; two per SIMD so that one wavefront's LDS and
// barrier waits hide under the other's MFMAs), each 128 x 64 = 4 x 2 MFMA 32x32x16 blocks
// with fp32 accumulators.  LDS is double-buffered; global loads run one whole tile ahead in
// registers; MFMA operands are read from LDS one 16-wide step ahead of their use.  The
// forward's W tile is [k][n] in memory (column index contiguous); it is staged row-major and
// read with the transposing LDS load.  The MFMA operands are swapped (C^T blocks) so that
// each lane ends up with 4 consecutive output columns, which lets the epilogue transpose each
// wavefront's sub-tile through LDS with 64-bit writes and store full 128-byte row segments.
#include "mfma_common.h"

namespace mlora {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int WM = 2, WN = 4;                 // wavefront grid
constexpr int NTHR = 64 * WM * WN;            // 512
constexpr int TM = BM / WM, TN = BN / WN;     // 128 x 64 per wavefront
constexpr int MB = TM / 32, NB = TN / 32;     // 4 x 2 MFMA blocks
constexpr int CH = (BM * BK / 8) / NTHR;      // 16-byte chunks per thread per operand tile (4)
constexpr int A_LD = BK + 8;     // 144-byte rows: conflict-free 128-bit fragment reads
constexpr int BNT_LD = BK + 8;   // [col][contraction] layout
constexpr int BNN_LD = BN + 32;  // [contraction][col] layout, 576-byte rows for the transposing reads
constexpr int A_TILE = BM * A_LD;
constexpr int B_TILE = BN * BNT_LD;
static_assert(B_TILE == BK * BNN_LD, "both B layouts share one buffer size");
constexpr int STAGE = A_TILE + B_TILE;
constexpr int E_LD = TN + 8;     // epilogue staging row
static_assert(WM * WN * TM * E_LD <= 2 * STAGE, "epilogue staging fits in the tile buffers");
static_assert(kGemmTileRows == BM && kGemmTileCols == BN, "plan geometry and kernel tile must agree");

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

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

// One masked operand pass staged into stage 0 of the tile buffers.  Used for the rank extension
// (rows owned by one adapter, contraction = rank) and for the tail of a contraction that is not a
// multiple of 64.  All arguments are uniform over the workgroup.
struct PassDesc {
    const u16* a_src; int64_t a_ld;   // element (row t, c) at a_src[(t - a_row_base) * a_ld + c]
    int a_row_base, a_row_lo, a_row_hi;
    bool a_vec;
    float scale;
    const u16* b_src; int64_t b_ld;   // NN: (c, col) at b_src[c * b_ld + col];  NT: at b_src[col * b_ld + c]
    bool b_vec;
    int kc;                            // valid contraction length, 1..64
};

template <bool NN>
__device__ __forceinline__ void stage_pass(u16* As, u16* Bs, const PassDesc& d, int m0, int n0, int ncols, int tid) {
    const int kpad = (d.kc + 15) & ~15;
    const int nch = kpad / 8;
    {
        const int row = tid & (BM - 1);
        const int t = m0 + row;
        const bool own = (t >= d.a_row_lo && t < d.a_row_hi);
        const u16* src = d.a_src + (int64_t)(t - d.a_row_base) * d.a_ld;
        for (int cc = tid >> 8; cc < nch; cc += NTHR / BM) {
            uint4 v = zero4();
            if (own) {
                v = load_chunk(src + cc * 8, min(8, d.kc - cc * 8), d.a_vec);
                if (d.scale != 1.0f) v = scale_chunk(v, d.scale);
            }
            *reinterpret_cast<uint4*>(As + row * A_LD + cc * 8) = v;
        }
    }
    if (NN) {
        const int nc = tid & 31;
        const int gcol = n0 + nc * 8;
        for (int krow = tid >> 5; krow < kpad; krow += NTHR / 32) {
            uint4 v = zero4();
            if (krow < d.kc && gcol < ncols)
                v = load_chunk(d.b_src + (int64_t)krow * d.b_ld + gcol, min(8, ncols - gcol), d.b_vec);
            *reinterpret_cast<uint4*>(Bs + krow * BNN_LD + nc * 8) = v;
        }
    } else {
        const int row = tid & (BN - 1);
        const int gcol = n0 + row;
        const u16* src = d.b_src + (int64_t)gcol * d.b_ld;
        for (int cc = tid >> 8; cc < nch; cc += NTHR / BN) {
            uint4 v = zero4();
            if (gcol < ncols) v = load_chunk(src + cc * 8, min(8, d.kc - cc * 8), d.b_vec);
            *reinterpret_cast<uint4*>(Bs + row * BNT_LD + cc * 8) = v;
        }
    }
}

template <bool NN>
__global__ __launch_bounds__(NTHR) void fused_gemm_kernel(GemmArgs g) {
    __shared__ __attribute__((aligned(16))) u16 lds[2 * STAGE];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lm = lane & 31, h = lane >> 5, gq = lane >> 4, j = lane & 15;

    // Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous run of
    // tiles and walk it in bands of 8 row tiles so that co-resident tiles share W / X panels
    // in that XCD's L2.
    const int total = g.tiles_m * g.tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int L = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (L >= total) return;
    constexpr int GM = 8;
    const int band = L / (GM * g.tiles_n);
    const int band_rows = min(GM, g.tiles_m - band * GM);
    const int in_band = L - band * GM * g.tiles_n;
    const int tm = band * GM + in_band % band_rows;
    const int tn = in_band / band_rows;
    const int m0 = tm * BM, n0 = tn * BN;

    f32x16 acc[MB][NB];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    // fragment read offsets (elements)
    const int a_off = (wm * TM + lm) * A_LD + h * 8;
    const int bnt_off = (wn * TN + lm) * BNT_LD + h * 8;
    const int bnn_off = (8 * (gq >> 1) + (j >> 2)) * BNN_LD + wn * TN + 16 * (gq & 1) + 4 * (j & 3);
    bf16x8 fa[2][MB], fb[2][NB];
    auto rfrag = [&](int stage, int ks, int buf) {
        const u16* As = lds + stage * STAGE;
        const u16* Bs = As + A_TILE;
#pragma unroll
        for (int a = 0; a < MB; ++a) fa[buf][a] = lds_read_frag(As + a_off + a * 32 * A_LD + ks * 16);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (NN) {
                const u16* p = Bs + bnn_off + ks * 16 * BNN_LD + b * 32;
                fb[buf][b] = lds_read_frag_tr(p, p + 4 * BNN_LD);
            } else {
                fb[buf][b] = lds_read_frag(Bs + bnt_off + b * 32 * BNT_LD + ks * 16);
            }
        }
    };
    // operands swapped: acc[a][b] holds the transposed 32x32 block (lane = output row, 4 consecutive columns per group)
    auto mma = [&](int buf, int a_lo, int a_hi) {
#pragma unroll
        for (int a = a_lo; a < a_hi; ++a)
#pragma unroll
            for (int b = 0; b < NB; ++b) acc[a][b] = mfma32(fb[buf][b], fa[buf][a], acc[a][b]);
    };
    // ask the scheduler to alternate LDS reads with MFMAs instead of issuing the reads in one burst
    auto interleave = [&]() {
        constexpr int NDS = NN ? (MB + 2 * NB) : (MB + NB);
#pragma unroll
        for (int i = 0; i < NDS; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
        }
    };

    // ---- contraction over the frozen weight: whole 64-wide tiles -------------------------------
    const int nk = g.skip_base ? 0 : g.Kdim / BK;
    if (nk > 0) {
        // per-thread global pointers; rows / columns past the edge are clamped to valid memory
        // (they only feed output rows / columns that are never stored)
        const u16* pa[CH];
        const u16* pb[CH];
        int sa[CH], sb[CH];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int row = (tid >> 3) + (NTHR / 8) * c, kc = tid & 7;
            pa[c] = g.Aop + (int64_t)min(m0 + row, g.M - 1) * g.lda + kc * 8;
            sa[c] = row * A_LD + kc * 8;
            if (NN) {
                const int krow = (tid >> 5) + (NTHR / 32) * c, nc = tid & 31;
                pb[c] = g.Bop + (int64_t)krow * g.ldb + min(n0 + nc * 8, g.Ncols - 8);
                sb[c] = krow * BNN_LD + nc * 8;
            } else {
                pb[c] = g.Bop + (int64_t)min(n0 + row, g.Ncols - 1) * g.ldb + kc * 8;
                sb[c] = row * BNT_LD + kc * 8;
            }
        }
        const int64_t bstep = NN ? (int64_t)BK * g.ldb : (int64_t)BK;
        u32x4 ra[CH], rb[CH];
        auto gload = [&](bool advance) {
            const int64_t da = advance ? (int64_t)BK : 0, db = advance ? bstep : 0;
#pragma unroll
            for (int c = 0; c < CH; ++c) { ra[c] = *reinterpret_cast<const u32x4*>(pa[c]); pa[c] += da; }
#pragma unroll
            for (int c = 0; c < CH; ++c) { rb[c] = *reinterpret_cast<const u32x4*>(pb[c]); pb[c] += db; }
        };
        auto lstore = [&](int stage) {
            u16* As = lds + stage * STAGE;
            u16* Bs = As + A_TILE;
#pragma unroll
            for (int c = 0; c < CH; ++c) *reinterpret_cast<u32x4*>(As + sa[c]) = ra[c];
#pragma unroll
            for (int c = 0; c < CH; ++c) *reinterpret_cast<u32x4*>(Bs + sb[c]) = rb[c];
        };

        gload(nk > 1);
        lstore(0);
        __syncthreads();
        rfrag(0, 0, 0);
        gload(nk > 2);   // tile 1 travels in registers for a whole iteration (a harmless reload if nk == 1)
        for (int kt = 0; kt < nk - 1; ++kt) {
            const int cur = kt & 1;
            lstore(cur ^ 1);          // tile kt+1; that stage was last read before the previous barrier
            gload(kt + 3 < nk);       // tile kt+2 (re-reads the last tile when past the end)
            __builtin_amdgcn_sched_barrier(0);
            rfrag(cur, 1, 1); mma(0, 0, MB); interleave();
            __builtin_amdgcn_sched_barrier(0);
            rfrag(cur, 2, 0); mma(1, 0, MB); interleave();
            __builtin_amdgcn_sched_barrier(0);
            rfrag(cur, 3, 1); mma(0, 0, MB); interleave();
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();          // tile kt+1 visible; nobody reads stage `cur` after this point
            rfrag(cur ^ 1, 0, 0); mma(1, 0, MB); interleave();
            __builtin_amdgcn_sched_barrier(0);
        }
        {
            const int cur = (nk - 1) & 1;
            rfrag(cur, 1, 1); mma(0, 0, MB);
            rfrag(cur, 2, 0); mma(1, 0, MB);
            rfrag(cur, 3, 1); mma(0, 0, MB);
            mma(1, 0, MB);
        }
    }

    // one masked pass: stage into buffer 0, then ceil(kc / 16) MFMA steps
    auto run_pass = [&](const PassDesc& d) {
        __syncthreads();
        stage_pass<NN>(lds, lds + A_TILE, d, m0, n0, g.Ncols, tid);
        __syncthreads();
        const int ksteps = (d.kc + 15) / 16;
        for (int ks = 0; ks < ksteps; ++ks) {
            rfrag(0, ks, 0);
            mma(0, 0, MB);
        }
    };

    // ---- tail of a contraction that is not a multiple of 64 -------------------------------------
    if (!g.skip_base && (g.Kdim % BK) != 0) {
        const int k0 = (g.Kdim / BK) * BK;
        PassDesc d;
        d.a_src = g.Aop + k0; d.a_ld = g.lda; d.a_row_base = 0; d.a_row_lo = m0; d.a_row_hi = min(g.M, m0 + BM);
        d.a_vec = true; d.scale = 1.0f;
        d.b_src = NN ? g.Bop + (int64_t)k0 * g.ldb : g.Bop + k0; d.b_ld = g.ldb; d.b_vec = true;
        d.kc = g.Kdim - k0;
        run_pass(d);
    }

    // ---- rank extension: one masked pass per adapter that owns rows of this tile -----------------
    if (!g.skip_lora) {
        const Entry4 tile = g.pv.gemm_tiles[tm];
        for (int i = tile.c; i < tile.d; ++i) {
            const int r = g.pv.rank[i];
            if (r == 0) continue;
            const int seg0 = g.pv.off[i], seg1 = g.pv.off[i + 1];
            const int lo = max(seg0, m0), hi = min(seg1, m0 + BM);
            if (lo >= hi) continue;
            const int64_t so = g.pv.soff[i];
            const u16* F = (const u16*)(NN ? g.pv.ptrs[i].B : g.pv.ptrs[i].A);
            for (int r0 = 0; r0 < r; r0 += BK) {
                PassDesc d;
                d.a_src = g.E + so + r0; d.a_ld = r; d.a_row_base = seg0; d.a_row_lo = lo; d.a_row_hi = hi;
                d.a_vec = ((r & 7) == 0) && ((so & 7) == 0);
                d.scale = NN ? g.pv.scale[i] : 1.0f;
                if (NN) { d.b_src = F + (int64_t)r0 * g.Ncols; d.b_ld = g.Ncols; d.b_vec = true; }
                else    { d.b_src = F + r0; d.b_ld = r; d.b_vec = ((r & 7) == 0); }
                d.kc = min(BK, r - r0);
                run_pass(d);
            }
        }
    }

    // ---- epilogue: each wavefront transposes its own sub-tile through LDS; one rounding from fp32 ----
    __syncthreads();
    {
        u16* Es = lds + wave * (TM * E_LD);
#pragma unroll
        for (int a = 0; a < MB; ++a)
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint2 v;
                    v.x = pack2(acc[a][b][4 * q + 0], acc[a][b][4 * q + 1]);
                    v.y = pack2(acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]);
                    *reinterpret_cast<uint2*>(Es + (a * 32 + lm) * E_LD + b * 32 + q * 8 + h * 4) = v;
                }
        // the same wavefront reads back what it wrote: only its own LDS writes must have landed
        __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
        constexpr int CPR = TN / 8;            // 16-byte chunks per row of the sub-tile
        constexpr int RPI = 64 / CPR;          // rows per wavefront-wide store
#pragma unroll
        for (int it = 0; it < TM / RPI; ++it) {
            const int rr = it * RPI + lane / CPR, c = lane % CPR;
            const int row = m0 + wm * TM + rr, col = n0 + wn * TN + c * 8;
            if (row >= g.M || col >= g.Ncols) continue;   // Ncols is a multiple of 8: chunks are all-in or all-out
            uint4 v = *reinterpret_cast<const uint4*>(Es + rr * E_LD + c * 8);
            u16* dst = g.C + (int64_t)row * g.ldc + col;
            if (g.accumulate) {   // in-place LoRA-only mode: add what the output already holds, round once more
                const uint4 old = *reinterpret_cast<const uint4*>(dst);
                const uint32_t nv[4] = {v.x, v.y, v.z, v.w}, ov[4] = {old.x, old.y, old.z, old.w};
                uint32_t res[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    res[e] = pack2(__uint_as_float(nv[e] << 16) + __uint_as_float(ov[e] << 16),
                                   __uint_as_float(nv[e] & 0xffff0000u) + __uint_as_float(ov[e] & 0xffff0000u));
                v = make_uint4(res[0], res[1], res[2], res[3]);
            }
            *reinterpret_cast<uint4*>(dst) = v;
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
    if (fwd) hipLaunchKernelGGL(fused_gemm_kernel<true>, dim3(grid), dim3(NTHR), 0, st, g);
    else     hipLaunchKernelGGL(fused_gemm_kernel<false>, dim3(grid), dim3(NTHR), 0, st, g);
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

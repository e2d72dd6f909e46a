// Fused frozen-weight GEMM + LoRA expand for bf16 on gfx950 MFMA.
//
// Forward (paper Sec. 5.1 / App. A.1, "fused base-output addition"): the paper runs the
// base GEMM, then a second GEMM Y = S_i B_i + Y_base that reloads the base tile.  Here the
// expand is folded into the base GEMM itself: ahead of the contraction over k, the same
// accumulators take a few MFMA steps over the rank dimension with operands S_i (rows of
// the tile that belong to adapter i, zero elsewhere) and B_i, and are scaled by s_i, so Y is
// written exactly once and Y_base never exists in memory.  Row tiles are not aligned to
// segments; a tile that straddles several adapters runs one masked extension per adapter.
// Backward input gradient is the mirror image: dX = dY W^T, extended with dS_i and A_i^T.
//
// Tile 256 x 256 x 64, 8 wavefronts (2 x 4; two per SIMD so that one wavefront's waits hide under the
// other's MFMAs), each 128 x 64 = 8 x 4 blocks of 16x16x32 MFMAs with fp32 accumulators (on this chip a
// GEMM of this size runs into the board power limit, and the 16x16x32 form needs measurably less energy
// per FLOP than 32x32x16).  Operand tiles go from global memory straight into LDS (no staging registers,
// no LDS store instructions).  The 160 KB of LDS hold five 32 KB tile buffers: two stages for the row
// operand (X / dY), which runs one tile ahead, and three slots for the weight operand, which runs two
// tiles ahead.  The eight direct loads a wavefront owes per tile are issued one at a time between groups
// of 8 MFMAs: issued back to back after the barrier they fill the memory pipeline's queue and every
// wavefront of the workgroup sits blocked on load issue, with no MFMA in flight, for ~20 % of the tile.
// With the weight tile two tiles ahead, each barrier only waits for loads issued at least half a tile
// earlier.  LDS tiles are unpadded and
// XOR-swizzled so that both the 1 KB-contiguous direct loads and the fragment reads are conflict free:
//   X / dY tile and the [col][contraction] weight tile: 256 rows of 128 bytes; the 16-byte chunk c of
//     row r sits at chunk position c ^ (r & 7);
//   the forward's W tile is [k][n] in memory (column index contiguous): 64 rows of 512 bytes, chunk c
//     (8 columns) of row k sits at position c ^ (v(k) << 1), v(k) = (k & 3) | (((k >> 3) & 1) << 2); it
//     is read with the transposing LDS load.
// The MFMA operands are swapped (C^T blocks) so that each lane ends up with 4 consecutive output columns,
// which lets the epilogue transpose each wavefront's sub-tile through LDS with 64-bit writes and store
// full 128-byte row segments.
#include "mfma_common.h"

namespace mlora {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int WM = 2, WN = 4;                 // wavefront grid
constexpr int NTHR = 64 * WM * WN;            // 512
constexpr int TM = BM / WM, TN = BN / WN;     // 128 x 64 per wavefront
constexpr int TILE_BYTES = 32768;             // one operand tile
constexpr int B_SLOT0 = 2;                    // tile buffers 0, 1: row-operand stages; 2, 3, 4: weight-operand slots
constexpr int E_LD = TN + 8;                  // epilogue staging row (elements)
constexpr int EPI_BYTES = WM * WN * TM * E_LD * 2;
constexpr int LDS_BYTES = 5 * TILE_BYTES;     // all of a CU's LDS
static_assert(EPI_BYTES <= LDS_BYTES, "epilogue staging must fit the tile buffers");
static_assert(kGemmTileRows == BM && kGemmTileCols == BN, "plan geometry and kernel tile must agree");

typedef f32x4 f32x4v;

// all of this wavefront's direct loads and LDS accesses have completed; then the workgroup barrier
__device__ __forceinline__ void wait_all_and_barrier() {
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

struct GemmArgs {
    const u16* Aop; int64_t lda;   // X [T,k] (fwd) or dY [T,n] (bwd)
    const u16* Bop; int64_t ldb;   // W [k,n]
    u16* C; int64_t ldc;           // Y [T,n] or dX [T,k]
    const u16* E;                  // ragged S (fwd) or dS (bwd)
    int32_t M, Ncols, Kdim;
    int32_t tiles_m, tiles_n;
    int32_t skip_lora;             // MLORA_FLAG_BASE_ONLY, or a plan without adapters (the LoRA-only mode has a kernel of its own)
    int32_t stream_out;            // write the output with streaming stores (see launch_gemm)
    int32_t band_group;            // bands whose column groups are interleaved (see the tile order)
    PlanView pv;
};

// One masked operand pass staged into the first row-operand stage and the first weight slot.  Used for the rank extension
// (rows owned by one adapter, contraction = rank) and for the tail of a contraction that is not a
// multiple of 64.  All arguments are uniform over the workgroup.
struct PassDesc {
    const u16* a_src; int64_t a_ld;   // element (row t, c) at a_src[(t - a_row_base) * a_ld + c]
    int a_row_base, a_row_lo, a_row_hi;
    bool a_vec;
    const u16* b_src; int64_t b_ld;   // NN: (c, col) at b_src[c * b_ld + col];  NT: at b_src[col * b_ld + c]
    bool b_vec;
    int kc;                            // valid contraction length, 1..64
    bool isolate;                      // rows of other adapters share the tile: see stage_pass
};

// Isolation of co-located jobs.  A rank-extension pass masks the rows of other adapters by staging zeros for them, and
// then multiplies those zeros with adapter j's B_j (A_j^T in the backward).  If job j has diverged and its matrices hold
// Inf or NaN, 0 x Inf = NaN would land in its neighbours' rows of every tile that straddles the segment boundary.  So in
// such tiles the staged copy of adapter j's operand has its non-finite values replaced by zero, the columns they sat in
// are flagged, and after the pass's MFMAs the accumulators of adapter j's own rows in flagged columns are set to NaN
// (the plain definition gives Inf or NaN there).  Flags: one byte per tile column and one "any" word behind them, in a
// tile buffer the pass does not use.
constexpr int FLAG_OFF = TILE_BYTES;          // row stage 1 is free during a pass
constexpr int FLAG_ANY = FLAG_OFF + BN;       // uint32 behind the BN column bytes

// zeroes the non-finite bf16 values of a chunk; bit e of the result is set if element e was non-finite
__device__ __forceinline__ unsigned drop_nonfinite(uint4& v) {
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
    unsigned mask = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if ((w[e] & 0x7f80u) == 0x7f80u) { w[e] &= 0xffff0000u; mask |= 1u << (2 * e); }
        if ((w[e] & 0x7f800000u) == 0x7f800000u) { w[e] &= 0x0000ffffu; mask |= 2u << (2 * e); }
    }
    v = make_uint4(w[0], w[1], w[2], w[3]);
    return mask;
}

// Writes the pass operands into tile buffers 0 and B_SLOT0 in the same swizzled layouts the main loop uses, zero-filled
// up to a multiple of 32 in the contraction and outside the rows / columns the pass owns.
template <bool NN>
__device__ __forceinline__ void stage_pass(unsigned char* lds, const PassDesc& d, int m0, int n0, int ncols, int tid) {
    const int kpad = (d.kc + 31) & ~31;
    const int nch = kpad / 8;
    {
        const int row = tid & (BM - 1);
        const int t = m0 + row;
        const bool own = (t >= d.a_row_lo && t < d.a_row_hi);
        const u16* src = d.a_src + (int64_t)(t - d.a_row_base) * d.a_ld;
        for (int cc = tid >> 8; cc < nch; cc += NTHR / BM) {
            uint4 v = zero4();
            if (own) v = load_chunk(src + cc * 8, min(8, d.kc - cc * 8), d.a_vec);
            *reinterpret_cast<uint4*>(lds + row * 128 + ((cc ^ (row & 7)) << 4)) = v;
        }
    }
    unsigned char* Bs = lds + B_SLOT0 * TILE_BYTES;
    if (NN) {
        const int nc = tid & 31;
        const int gcol = n0 + nc * 8;
        for (int krow = tid >> 5; krow < kpad; krow += NTHR / 32) {
            uint4 v = zero4();
            if (krow < d.kc && gcol < ncols)
                v = load_chunk(d.b_src + (int64_t)krow * d.b_ld + gcol, min(8, ncols - gcol), d.b_vec);
            if (d.isolate) {
                const unsigned bad = drop_nonfinite(v);
                if (bad) {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (bad >> e & 1) lds[FLAG_OFF + nc * 8 + e] = 1;
                    *reinterpret_cast<uint32_t*>(lds + FLAG_ANY) = 1u;
                }
            }
            *reinterpret_cast<uint4*>(Bs + krow * 512 + ((nc ^ (nn_swz(krow) << 1)) << 4)) = v;
        }
    } else {
        const int row = tid & (BN - 1);
        const int gcol = n0 + row;
        const u16* src = d.b_src + (int64_t)gcol * d.b_ld;
        for (int cc = tid >> 8; cc < nch; cc += NTHR / BN) {
            uint4 v = zero4();
            if (gcol < ncols) v = load_chunk(src + cc * 8, min(8, d.kc - cc * 8), d.b_vec);
            if (d.isolate && drop_nonfinite(v)) {
                lds[FLAG_OFF + row] = 1;
                *reinterpret_cast<uint32_t*>(lds + FLAG_ANY) = 1u;
            }
            *reinterpret_cast<uint4*>(Bs + row * 128 + ((cc ^ (row & 7)) << 4)) = v;
        }
    }
}

#define MLORA_SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)

template <bool NN>
__global__ __launch_bounds__(NTHR) void fused_gemm_kernel(GemmArgs g) {
    __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS_BYTES];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int l16 = lane & 15, g4 = lane >> 4;

    // Tile order.  Tiles are numbered band by band (a band = 8 row tiles x all column tiles, numbered down the rows first),
    // so 32 consecutive numbers are 8 row tiles x 4 column tiles: 12 operand panels for 32 tiles.  Workgroups are handed to
    // the 8 XCDs round-robin (XCD = blockIdx % 8), and each XCD has its own L2: the 32 workgroups an XCD runs at a time take
    // one such group, so that they share those panels in its L2.  Consecutive groups go to consecutive XCDs, i.e. all
    // eight XCDs work on the same band at the same time, on different columns: the band's row panels are then fetched
    // from HBM once and served to the other XCDs, and to later rounds, by the Infinity Cache (with one band per XCD the
    // eight bands of a large layer did not fit there together; this order measured 1.5 to 4.5 % faster on every workload).
    const int total = g.tiles_m * g.tiles_n;
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const int L = ((slot / 32) * 8 + xcd) * 32 + (slot % 32);
    if (L >= total) return;
    // The bands themselves run in the order the plan's scheduler table gives (most rank-extension work first; a last,
    // shorter band stays last, so every band before position `ord` is a full one).  `band_group` = H consecutive full
    // bands of that order run interleaved by 32-tile groups (band 0 columns 0-3, band 1 columns 0-3, ..., band 0 columns
    // 4-7, ...): the eight XCDs then cover H bands x 8/H column groups at a time, and one sweep over the weight's column
    // panels serves H bands.  What is left over (a short last band, fewer than H bands, the columns past the last whole
    // group of four) is numbered band by band.
    constexpr int GM = kGemmBandTiles;
    const int per_band = GM * g.tiles_n;
    const int H = g.band_group;
    const int nfull = g.pv.band_order[g.pv.n_bands - 1].c == GM ? g.pv.n_bands : g.pv.n_bands - 1;
    const int nsup = nfull / H;
    int ord, in_band;
    if (L < nsup * H * per_band) {
        const int P = L / (H * per_band), within = L - P * (H * per_band);
        const int full_cg = g.tiles_n / 4;
        if (within < H * full_cg * 32) {
            const int c = within / 32;
            ord = P * H + c % H; in_band = (c / H) * 32 + within % 32;
        } else {
            const int rem = within - H * full_cg * 32, rem_per = per_band - full_cg * 32;
            ord = P * H + rem / rem_per; in_band = full_cg * 32 + rem % rem_per;
        }
    } else {
        const int Lr = L - nsup * H * per_band;
        ord = nsup * H + Lr / per_band; in_band = Lr % per_band;
    }
    const Entry4 band = g.pv.band_order[ord];          // (band, first row tile, row tiles, cost)
    const int band_rows = band.c;
    const int tm = band.b + in_band % band_rows;
    const int tn = in_band / band_rows;
    const int m0 = tm * BM, n0 = tn * BN;

    // acc[a][b][i] = C[m0 + wm*128 + a*16 + l16][n0 + wn*64 + b*16 + 4*g4 + i]
    f32x4v acc[8][4];
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[a][b][i] = 0.f;

    // ---- fragment reads (k32 = 32-wide half of the 64-wide tile, half = upper / lower 64 rows of the wave tile) ----
    const int a_off0 = (wm * TM + l16) * 128 + ((g4 ^ (l16 & 7)) << 4);
    const int a_off1 = (wm * TM + l16) * 128 + (((4 + g4) ^ (l16 & 7)) << 4);
    const int bnt_off0 = (wn * TN + l16) * 128 + ((g4 ^ (l16 & 7)) << 4);
    const int bnt_off1 = (wn * TN + l16) * 128 + (((4 + g4) ^ (l16 & 7)) << 4);
    const int vq = ((l16 >> 2) & 3) | ((g4 & 1) << 2);    // nn_swz of the rows this lane reads
    const int bnn_off = (8 * g4 + (l16 >> 2)) * 512 + (l16 & 3) * 8;
    bf16x8 fa[2][4], fb[2][4];
    auto rfa = [&](int stage, int k32, int half, int buf) {
        const unsigned char* base = lds + stage * TILE_BYTES + (k32 ? a_off1 : a_off0);
#pragma unroll
        for (int a = 0; a < 4; ++a) fa[buf][a] = lds_read_frag(reinterpret_cast<const u16*>(base + (half * 4 + a) * 16 * 128));
    };
    auto rfb = [&](int slot, int k32, int buf) {
        const unsigned char* bbase = lds + (B_SLOT0 + slot) * TILE_BYTES;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            if (NN) {
                const unsigned char* p = bbase + bnn_off + k32 * 32 * 512 + (((wn * 4 + b) ^ vq) << 5);
                fb[buf][b] = lds_read_frag_tr(reinterpret_cast<const u16*>(p), reinterpret_cast<const u16*>(p + 4 * 512));
            } else {
                fb[buf][b] = lds_read_frag(reinterpret_cast<const u16*>(bbase + (k32 ? bnt_off1 : bnt_off0) + b * 16 * 128));
            }
        }
    };
    auto rfbh = [&](int slot, int k32, int buf, int h) {     // half of rfb: column blocks 2 h, 2 h + 1
        const unsigned char* bbase = lds + (B_SLOT0 + slot) * TILE_BYTES;
#pragma unroll
        for (int b = 2 * h; b < 2 * h + 2; ++b) {
            if (NN) {
                const unsigned char* p = bbase + bnn_off + k32 * 32 * 512 + (((wn * 4 + b) ^ vq) << 5);
                fb[buf][b] = lds_read_frag_tr(reinterpret_cast<const u16*>(p), reinterpret_cast<const u16*>(p + 4 * 512));
            } else {
                fb[buf][b] = lds_read_frag(reinterpret_cast<const u16*>(bbase + (k32 ? bnt_off1 : bnt_off0) + b * 16 * 128));
            }
        }
    };
    // operands swapped: each accumulator block holds the transposed 16x16 block (lane = output row, 4 consecutive columns)
    auto mma = [&](int half, int abuf, int bbuf) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) acc[half * 4 + a][b] = mfma16(fb[bbuf][b], fa[abuf][a], acc[half * 4 + a][b]);
    };
    // two of the four 16-row blocks of one half: 8 MFMAs
    auto mma8 = [&](int half, int abuf, int bbuf, int alo) {
#pragma unroll
        for (int a = alo; a < alo + 2; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) acc[half * 4 + a][b] = mfma16(fb[bbuf][b], fa[abuf][a], acc[half * 4 + a][b]);
    };
    // ask the scheduler to spread nds LDS reads over the 8 MFMAs issued with them instead of one burst
    constexpr int NDSB = NN ? 8 : 4;
    auto interleave = [&](int nds) {
        if (nds > 8) { for (int i = 0; i < 8; ++i) { MLORA_SGB(0x008, 1); if (2 * i < nds) MLORA_SGB(0x100, 2); } }
        else { for (int i = 0; i < 8; ++i) { MLORA_SGB(0x008, 1); if (i < nds) MLORA_SGB(0x100, 1); } }
        __builtin_amdgcn_sched_barrier(0);
    };

    // Direct loads of the contraction over the frozen weight: 4 instructions per wave per operand, each fills 1 KB of LDS.
    // Address = uniform base (advances one tile per step) + constant per-lane byte offset.  Rows / columns past the edge are
    // clamped to valid memory (they only feed outputs that are never stored).
    const int nk = g.Kdim / BK;
    unsigned oa[4], ob[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int ii = wave * 4 + c;
        const int row = ii * 8 + (lane >> 3), ch = (lane & 7) ^ (lane >> 3);
        oa[c] = (unsigned)((int64_t)(min(m0 + row, g.M - 1) - m0) * g.lda + ch * 8) * 2u;
        if (NN) {
            const int k = ii * 2 + (lane >> 5);
            const int chn = (lane & 31) ^ (nn_swz(k) << 1);
            ob[c] = (unsigned)((int64_t)k * g.ldb + min(n0 + chn * 8, g.Ncols - 8)) * 2u;
        } else {
            ob[c] = (unsigned)((int64_t)(min(n0 + row, g.Ncols - 1) - n0) * g.ldb + ch * 8) * 2u;
        }
    }
    const char* baseA = uniform_ptr(g.Aop + (int64_t)m0 * g.lda);
    const char* baseB = NN ? uniform_ptr(g.Bop) : uniform_ptr(g.Bop + (int64_t)n0 * g.ldb);
    const int64_t astep = (int64_t)BK * 2, bstep = NN ? (int64_t)BK * g.ldb * 2 : (int64_t)BK * 2;
    const unsigned ldsw = (unsigned)(uintptr_t)lds + wave * 4096;
    auto dmaA = [&](int stage, int c) { dma16(oa[c], baseA, ldsw + stage * TILE_BYTES + c * 1024); };
    auto dmaB = [&](int slot, int c) { dma16(ob[c], baseB, ldsw + (B_SLOT0 + slot) * TILE_BYTES + c * 1024); };

    // one masked pass: stage (through registers) into the first row stage and weight slot, then one or two 32-wide MFMA steps
    auto run_pass = [&](const PassDesc& d) {
        wait_all_and_barrier();          // outstanding direct loads have landed; nobody reads the buffers any more
        if (d.isolate) {                 // (uniform) clear the column flags before anybody sets one
            if (tid <= BN / 4) reinterpret_cast<uint32_t*>(lds + FLAG_OFF)[tid] = 0u;
            __syncthreads();
        }
        stage_pass<NN>(lds, d, m0, n0, g.Ncols, tid);
        __syncthreads();
        const int ksteps = (d.kc + 31) / 32;
        for (int ks = 0; ks < ksteps; ++ks) {
            rfa(0, ks, 0, 0); rfa(0, ks, 1, 1); rfb(0, ks, 0);
            mma(0, 0, 0); mma(1, 1, 0);
        }
        if (d.isolate && *reinterpret_cast<const uint32_t*>(lds + FLAG_ANY) != 0u) {
            // the adapter's operand held Inf / NaN in some columns: its own rows of those columns are NaN
            const float qnan = __uint_as_float(0x7fc00000u);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const uint32_t f4 = *reinterpret_cast<const uint32_t*>(lds + FLAG_OFF + wn * TN + b * 16 + 4 * g4);
                if (f4 == 0u) continue;
#pragma unroll
                for (int a = 0; a < 8; ++a) {
                    const int row = m0 + wm * TM + a * 16 + l16;
                    if (row < d.a_row_lo || row >= d.a_row_hi) continue;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if ((f4 >> (8 * i)) & 0xffu) acc[a][b][i] = qnan;
                }
            }
        }
    };

    // ---- rank extension: the LoRA term goes into the accumulators first ------------------------------
    // acc = s_i (S_i B_i) here, the contraction over the frozen weight is added afterwards: the scale is applied to the fp32
    // accumulators (rows of S_i reach the MFMAs as stored, one rounding fewer than scaling them in bf16), and the operands of
    // the passes can be fetched like any other operand tile:
    //  * A tile whose rows all belong to one adapter with a rank that is a multiple of 8 (nearly every tile of a training
    //    batch) takes its one or two 64-rank passes as extra K-steps of the main loop's own form: rows of S_i and the
    //    64 x 256 piece of B_i (backward: dS_i, A_i) come by direct loads into tile buffers in the main loop's layouts -
    //    no staging registers, no LDS stores - and, for ranks up to 64, together with tile 0 of the frozen weight's
    //    contraction, so that their latency costs nothing.  Chunks past the rank are fetched from a valid address and
    //    overwritten with zeros before any MFMA reads them.
    //  * Any other tile (several adapters, a rank that is not a multiple of 8) stages each adapter's pass through registers
    //    with the rows of other adapters zeroed (run_pass).
    // Both forms feed the same values to the same MFMAs in the same order, so a row's bits do not depend on which one its
    // tile took.
    bool tile0_requested = false;
    if (!g.skip_lora) {
        const Entry4 tile = g.pv.gemm_tiles[tm];
        const int row_end = min(g.M, m0 + BM);
        int owners = 0, one = -1;
        for (int i = tile.c; i < tile.d; ++i) {
            if (g.pv.rank[i] == 0) continue;
            if (max(g.pv.off[i], m0) >= min(g.pv.off[i + 1], m0 + BM)) continue;
            ++owners; one = i;
        }
        bool direct = false;
        if (owners == 1) {
            const int r = g.pv.rank[one];
            direct = g.pv.off[one] <= m0 && g.pv.off[one + 1] >= row_end && (r & 7) == 0 && (g.pv.soff[one] & 7) == 0;
        }
        if (direct) {
            const int i = one;
            const int r = g.pv.rank[i];
            const int npass = (r + BK - 1) / BK;                       // 1 or 2
            const char* sb = reinterpret_cast<const char*>(g.E + g.pv.soff[i] + (int64_t)(m0 - g.pv.off[i]) * r);
            const u16* F = (const u16*)(NN ? g.pv.ptrs[i].B : g.pv.ptrs[i].A);
            // pass 0 goes to row stage 1 / weight slot 2, pass 1 to row stage 0 / weight slot 0 (the buffers tile 0 of the main
            // loop uses: with two passes it is requested after them)
            if (npass == 1 && nk > 0) {
#pragma unroll
                for (int c = 0; c < 4; ++c) dmaA(0, c);
#pragma unroll
                for (int c = 0; c < 4; ++c) dmaB(0, c);
                tile0_requested = true;
            }
            for (int p = 0; p < npass; ++p) {
                const int kc = min(BK, r - p * BK);
                const int stage = p == 0 ? 1 : 0, slot = p == 0 ? 2 : 0;
                const char* sbp = uniform_ptr(sb + p * BK * 2);
                const char* fbp = uniform_ptr(NN ? F + (int64_t)p * BK * g.Ncols : F + (int64_t)n0 * r + p * BK);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int ii = wave * 4 + c;
                    const int row = ii * 8 + (lane >> 3), ch = (lane & 7) ^ (lane >> 3);
                    const int chv = ch * 8 < kc ? ch : 0;
                    const unsigned va = (unsigned)((min(m0 + row, g.M - 1) - m0) * r + chv * 8) * 2u;
                    dma16(va, sbp, ldsw + stage * TILE_BYTES + c * 1024);
                    unsigned vb;
                    if (NN) {
                        const int k = ii * 2 + (lane >> 5);
                        const int chn = (lane & 31) ^ (nn_swz(k) << 1);
                        vb = (unsigned)((int64_t)(k < kc ? k : 0) * g.ldb + min(n0 + chn * 8, g.Ncols - 8)) * 2u;
                    } else {
                        vb = (unsigned)((min(n0 + row, g.Ncols - 1) - n0) * r + chv * 8) * 2u;
                    }
                    dma16(vb, fbp, ldsw + (B_SLOT0 + slot) * TILE_BYTES + c * 1024);
                }
            }
            wait_all_and_barrier();
            // ranks that are not multiples of 32: zeros over the chunks between the rank and the end of its 32-wide MFMA step
            bool zeroed = false;
            for (int p = 0; p < npass; ++p) {
                const int kc = min(BK, r - p * BK), kpad = (kc + 31) & ~31;
                if (kc == kpad) continue;
                zeroed = true;
                const int stage = p == 0 ? 1 : 0, slot = p == 0 ? 2 : 0;
                unsigned char* As = lds + stage * TILE_BYTES;
                unsigned char* Bs = lds + (B_SLOT0 + slot) * TILE_BYTES;
                const int c0 = kc / 8, nc = (kpad - kc) / 8;
                for (int idx = tid; idx < BM * nc; idx += NTHR) {
                    const int row = idx & (BM - 1), cc = c0 + idx / BM;
                    *reinterpret_cast<uint4*>(As + row * 128 + ((cc ^ (row & 7)) << 4)) = zero4();
                    if (!NN) *reinterpret_cast<uint4*>(Bs + row * 128 + ((cc ^ (row & 7)) << 4)) = zero4();
                }
                if (NN)
                    for (int idx = tid; idx < (kpad - kc) * 32; idx += NTHR)
                        *reinterpret_cast<uint4*>(Bs + (kc + idx / 32) * 512 + ((idx & 31) << 4)) = zero4();
            }
            if (zeroed) __syncthreads();
            for (int p = 0; p < npass; ++p) {
                const int kc = min(BK, r - p * BK);
                const int stage = p == 0 ? 1 : 0, slot = p == 0 ? 2 : 0;
                const int ksteps = (kc + 31) / 32;
                for (int ks = 0; ks < ksteps; ++ks) {
                    rfa(stage, ks, 0, 0); rfa(stage, ks, 1, 1); rfb(slot, ks, 0);
                    mma(0, 0, 0); mma(1, 1, 0);
                }
            }
            if (NN) {
                const float sc = g.pv.scale[i];
                if (sc != 1.0f) {
#pragma unroll
                    for (int a = 0; a < 8; ++a)
#pragma unroll
                        for (int b = 0; b < 4; ++b)
#pragma unroll
                            for (int q = 0; q < 4; ++q) acc[a][b][q] *= sc;
                }
            }
            wait_all_and_barrier();      // every wavefront is done with the pass buffers before the main loop's loads reuse them
        } else if (owners > 0) {
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
                    if (NN) { d.b_src = F + (int64_t)r0 * g.Ncols; d.b_ld = g.Ncols; d.b_vec = true; }
                    else    { d.b_src = F + r0; d.b_ld = r; d.b_vec = ((r & 7) == 0); }
                    d.kc = min(BK, r - r0);
                    d.isolate = lo > m0 || hi < row_end;
                    run_pass(d);
                }
                if (NN) {   // this adapter's rows hold nothing but its own term so far: scale them
                    const float sc = g.pv.scale[i];
                    if (sc != 1.0f) {
#pragma unroll
                        for (int a = 0; a < 8; ++a) {
                            const int row = m0 + wm * TM + a * 16 + l16;
                            if (row < lo || row >= hi) continue;
#pragma unroll
                            for (int b = 0; b < 4; ++b)
#pragma unroll
                                for (int q = 0; q < 4; ++q) acc[a][b][q] *= sc;
                        }
                    }
                }
            }
            wait_all_and_barrier();      // as above
        }
    }

    // ---- contraction over the frozen weight: whole 64-wide tiles -------------------------------
    if (nk > 0) {
        // tile 0 of both operands, then the weight tile 1 and the first half of the row tile 1: from here on the
        // order of this wavefront's loads is ... A(t+1) x4, B(t+2) x4, A(t+2) x4, B(t+3) x4 ...  Past the last tile the
        // base pointers stop advancing and the loads fetch the last tile again into buffers nobody reads.
        if (!tile0_requested) {
#pragma unroll
            for (int c = 0; c < 4; ++c) dmaA(0, c);
#pragma unroll
            for (int c = 0; c < 4; ++c) dmaB(0, c);
        }
        if (nk > 1) { baseA += astep; baseB += bstep; }
        if (!tile0_requested) wait_all_and_barrier();
#pragma unroll
        for (int c = 0; c < 4; ++c) dmaB(1, c);
        if (nk > 2) baseB += bstep;
        dmaA(1, 0); dmaA(1, 1);
        rfa(0, 0, 0, 0); rfb(0, 0, 0);
        int bs = 0;                      // weight slot of tile kt
        for (int kt = 0; kt < nk - 1; ++kt) {
            const int cur = kt & 1;
            const int bn = bs == 2 ? 0 : bs + 1, bp = bs == 0 ? 2 : bs - 1;
            // Since the last barrier row stage cur^1 and weight slot bp are free.  Row tile kt+1 is completed here,
            // the weight tile kt+2 follows; one load per 8 MFMAs.
            __builtin_amdgcn_sched_barrier(0);
            dmaA(cur ^ 1, 2);
            __builtin_amdgcn_sched_barrier(0);
            rfa(cur, 0, 1, 1); mma8(0, 0, 0, 0); interleave(4);
            dmaA(cur ^ 1, 3); baseA += (kt + 2 < nk) ? astep : 0;
            __builtin_amdgcn_sched_barrier(0);
            mma8(0, 0, 0, 2); __builtin_amdgcn_sched_barrier(0);
            dmaB(bp, 0);
            __builtin_amdgcn_sched_barrier(0);
            rfa(cur, 1, 0, 0); rfbh(bs, 1, 1, 0); mma8(1, 1, 0, 0); interleave(4 + NDSB / 2);
            dmaB(bp, 1);
            __builtin_amdgcn_sched_barrier(0);
            rfbh(bs, 1, 1, 1); mma8(1, 1, 0, 2); interleave(NDSB / 2);
            dmaB(bp, 2);
            __builtin_amdgcn_sched_barrier(0);
            // Last quarter before the barrier: this wavefront steps back behind the one it shares the SIMD with.  The two run
            // the same instruction stream and the issue arbiter prefers the older one, so without this one of them reaches the barrier
            // half a tile early and the other finishes alone, with nobody to fill the gaps behind its own LDS reads and load
            // issue.  With the priority dropped here the one that is behind gets the matrix pipe first and both arrive
            // together (backward GEMM 1.7-2 % faster, forward unchanged).
            __builtin_amdgcn_s_setprio(0);
            rfa(cur, 1, 1, 1); mma8(0, 0, 1, 0); interleave(4);
            dmaB(bp, 3); baseB += (kt + 3 < nk) ? bstep : 0;
            __builtin_amdgcn_sched_barrier(0);
            mma8(0, 0, 1, 2); __builtin_amdgcn_sched_barrier(0);
            // Everything but this iteration's four weight loads has landed: row tile kt+1 and weight tile kt+1 are
            // complete (this wavefront's share; the barrier covers the rest), and every wavefront has finished reading
            // row stage cur and weight slot bs, which the next loads overwrite.
            asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            __builtin_amdgcn_s_setprio(3);
            dmaA(cur, 0);
            __builtin_amdgcn_sched_barrier(0);
            // (the fragments of the weight operand are read in two halves, one with each group of 8 MFMAs: the forward's
            // transposing reads are two instructions per fragment, and sixteen of them in one group held the MFMAs up)
            rfa(cur ^ 1, 0, 0, 0); rfbh(bn, 0, 0, 0); mma8(1, 1, 1, 0); interleave(4 + NDSB / 2);
            dmaA(cur, 1);
            __builtin_amdgcn_sched_barrier(0);
            rfbh(bn, 0, 0, 1); mma8(1, 1, 1, 2); interleave(NDSB / 2);
            bs = bn;
        }
        {
            const int cur = (nk - 1) & 1;
            rfa(cur, 0, 1, 1); mma(0, 0, 0);
            rfa(cur, 1, 0, 0); rfb(bs, 1, 1); mma(1, 1, 0);
            rfa(cur, 1, 1, 1); mma(0, 0, 1);
            mma(1, 1, 1);
        }
    }

    // ---- tail of a contraction that is not a multiple of 64 -------------------------------------
    if ((g.Kdim % BK) != 0) {
        const int k0 = (g.Kdim / BK) * BK;
        PassDesc d;
        d.a_src = g.Aop + k0; d.a_ld = g.lda; d.a_row_base = 0; d.a_row_lo = m0; d.a_row_hi = min(g.M, m0 + BM);
        d.a_vec = true;
        d.b_src = NN ? g.Bop + (int64_t)k0 * g.ldb : g.Bop + k0; d.b_ld = g.ldb; d.b_vec = true;
        d.kc = g.Kdim - k0;
        d.isolate = false;
        run_pass(d);
    }

    // ---- epilogue: each wavefront transposes its own sub-tile through LDS; one rounding from fp32 ----
    wait_all_and_barrier();
    {
        u16* Es = reinterpret_cast<u16*>(lds) + wave * (TM * E_LD);
#pragma unroll
        for (int a = 0; a < 8; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                uint2 v;
                v.x = pack2hw(acc[a][b][0], acc[a][b][1]);
                v.y = pack2hw(acc[a][b][2], acc[a][b][3]);
                *reinterpret_cast<uint2*>(Es + (a * 16 + l16) * E_LD + b * 16 + g4 * 4) = v;
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
            const uint4 v = *reinterpret_cast<const uint4*>(Es + rr * E_LD + c * 8);
            u16* dst = g.C + (int64_t)row * g.ldc + col;
            if (g.stream_out) store_streaming(dst, v);
            else *reinterpret_cast<uint4*>(dst) = v;
        }
    }
}

static int launch_gemm(mlora_plan* p, bool fwd, const void* Aop, const void* W, void* C, const void* E,
                       uint32_t flags, hipStream_t st) {
    if (p->T == 0) return MLORA_OK;
    // the direct tile loads address a tile with 32-bit byte offsets from its first row: 256 rows of k or n elements
    if (p->k > (int64_t(1) << 22) || p->n > (int64_t(1) << 22)) {
        set_error("bf16 MFMA path supports k, n up to 4194304");
        return MLORA_ERR_SHAPE;
    }
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
    g.skip_lora = ((flags & MLORA_FLAG_BASE_ONLY) || p->N == 0) ? 1 : 0;
    // Streaming stores: an output written with ordinary stores sits dirty in the caches when the kernel ends and is
    // written back underneath the next kernel, which is always a memory-bound one (dShrink after the forward and the
    // weight gradients after the backward ran up to a third slower).
    g.stream_out = 1;
    // Row bands that share the sweep over the weight (see the tile order).  A weight that fits half of the 256 MB Infinity
    // Cache stays there from band to band and nothing is gained (Llama-8B MLP: 1-2 % lost); a larger one streams from HBM
    // once per group of bands, and as many bands are grouped as keep their row panels (2048 rows x contraction each) in
    // the other half of the cache.  Llama-70B MLP forward (448 MiB weight, 32 MiB of rows per band): 4 bands, the launch
    // 3.3 % faster; its backward (117 MB of rows per band) stays at one band.
    constexpr int64_t kHalfCache = int64_t(128) << 20;
    g.band_group = 1;
    if (flags & MLORA_FLAG_GROUP_BANDS) g.band_group = 4;
    else if (p->k * p->n * 2 > kHalfCache)
        while (g.band_group < 4 && int64_t(2 * g.band_group) * kGemmBandTiles * BM * g.Kdim * 2 <= kHalfCache) g.band_group *= 2;
    g.pv = p->view;
    const int total = g.tiles_m * g.tiles_n;
    const int grid = ((total + 255) / 256) * 256;    // whole groups of 32 tiles for each of the 8 XCDs
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

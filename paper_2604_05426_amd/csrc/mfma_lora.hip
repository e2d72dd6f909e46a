// Grouped low-rank kernels for bf16 on gfx950 MFMA: shrink, gradient shrink, weight gradients.
//
// Paper Sec. 5.1: the LoRA GEMMs are memory-bandwidth bound (r << k, n); all adapters run in
// one launch over a schedule table of (adapter, block) entries and only the diagonal blocks
// S_i = X_i A_i are computed.  App. A.1: blocks map to token ranges through the per-adapter
// offsets, the boundary block is masked at the segment end, ranks are masked (columns beyond
// r_i contribute zero).
#include "mfma_common.h"

namespace mlora {

// =========================================================================================
// Shrink:   S_i  = X_i A_i            (FWD: A_i is [k][r], column index contiguous -> transposing reads)
// dShrink:  dS_i = s_i dY_i B_i^T     (!FWD: B_i is [r][n], contraction contiguous)
// One workgroup per row block (64 rows of one adapter), 8 wavefronts.  Two bodies: the GEMM-tiled one further down
// (shrink_tiled_body) serves contractions that are multiples of 64 and, in the forward form, ranks that are multiples
// of 4; the register-staged one below takes everything else.  Register-staged body: the
// work is a pure stream of X (or dY), so it is built for bytes in flight: every wavefront owns a
// contiguous slice of the contraction and runs its own register-prefetch -> private LDS tile
// -> MFMA pipeline with no workgroup barrier in the loop, so eight independent streams per
// CU keep loads outstanding.  The eight partial tiles are added in LDS in wavefront order
// (deterministic) and rounded once.
// =========================================================================================
constexpr int SR = 64;             // rows per block == kBlockRows
constexpr int SNW = 8;             // wavefronts per workgroup
static_assert(kBlockRows == SR, "row-block table and shrink kernel must agree");

struct ShrinkArgs {
    const u16* src; int64_t ld;   // X (ld k) or dY (ld n)
    u16* out;                     // ragged S or dS
    int32_t Kdim;                 // k or n
    PlanView pv;                  // one workgroup per entry of pv.class_blocks (wide rank class first: its blocks run longest)
};

// MAXNB: rank blocks of 32 the kernel is built for (2: every rank <= 64, 4: ranks up to 128).
// SKS: contraction elements per wavefront step.  64 (ranks <= 64): every load instruction takes whole 128-byte lines,
//      which halves the number of outstanding line requests per byte (the L1's pending-miss capacity is what limits this
//      kernel); the X / dY tile is then unpadded and XOR-swizzled (chunk c of row r at c ^ ((r >> 1) & 7)), which keeps
//      the private LDS of the eight wavefronts at exactly 160 KB.  32 (wide ranks): 80-byte padded rows.
// DX / DF: register prefetch depth in steps for the streamed operand (X or dY, comes from HBM) and for
// the adapter matrix (cache resident).
template <bool FWD, int MAXNB, int SKS, int DX, int DF>
__device__ __forceinline__ void shrink_body(const ShrinkArgs& g, const Entry4 e, u16* lds) {
    constexpr bool SWZ = SKS == 64;
    constexpr int SX_LD = SWZ ? SKS : SKS + 8;                    // X / dY tile row (elements)
    constexpr int SX_TILE = SR * SX_LD;
    constexpr int SF_LD = SKS + 8;                                // !FWD small tile [rank][LD]: 80 / 144-byte rows
    constexpr int SBN_LD = MAXNB == 2 ? 96 : 160;                 // FWD small tile [SKS contraction][LD] (192 / 320-byte rows)
    constexpr int SB_TILE = (SKS * SBN_LD > MAXNB * 32 * SF_LD) ? SKS * SBN_LD : MAXNB * 32 * SF_LD;
    constexpr int S_WAVE = SX_TILE + SB_TILE;                     // per-wavefront private LDS (elements)
    constexpr int XC = SKS / 8;                                   // 16-byte chunks per X row per step
    constexpr int NX = SR * XC / 64;                              // X chunks per lane per step
    constexpr int NF = MAXNB * 32 * XC / 64;                      // small-tile chunks per lane per step
    constexpr int CPRF = MAXNB * 4;                               // FWD: 16-byte chunks per small-tile row
    static_assert(SNW * S_WAVE * 2 <= 163840, "private tiles fit in LDS");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = e.a, row0 = e.c, rows = e.d;
    const int r = g.pv.rank[i];
    const int rpad = (r + 31) & ~31;
    const int nblk = rpad / 32;
    const u16* F = (const u16*)(FWD ? g.pv.ptrs[i].A : g.pv.ptrs[i].B);
    const bool f_vec = FWD ? ((r & 7) == 0) : true;
    const float s = FWD ? 1.0f : g.pv.scale[i];
    u16* Xs = lds + wave * S_WAVE;
    u16* Fs = Xs + SX_TILE;
    // element offset of 16-byte chunk c of row `row` in the X tile
    auto xs_off = [&](int row, int c) { return SWZ ? row * SX_LD + ((c ^ ((row >> 1) & 7)) << 3) : row * SX_LD + c * 8; };

    f32x16 acc[2][MAXNB];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < MAXNB; ++nb)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[mb][nb][q] = 0.f;

    // this wavefront's share of the contraction: steps of SKS, dealt round-robin to the wavefronts so that at any
    // time the eight streams of a workgroup read neighbouring pieces of the same rows
    const int steps = (g.Kdim + SKS - 1) / SKS;
    const int s_begin = 0, s_end = wave < steps ? (steps - wave + SNW - 1) / SNW : 0;

    uint4 rx[DX][NX], rf[DF][NF];
    auto gloadX = [&](int lstep, int set) {
        const int k0 = (lstep * SNW + wave) * SKS;
#pragma unroll
        for (int jj = 0; jj < NX; ++jj) {
            const int row = (lane / XC) + (64 / XC) * jj, gk = k0 + (lane % XC) * 8;
            rx[set][jj] = (row < rows && gk < g.Kdim)
                              ? *reinterpret_cast<const uint4*>(g.src + (int64_t)(row0 + row) * g.ld + gk) : zero4();
        }
    };
    auto gloadF = [&](int lstep, int set) {
        const int k0 = (lstep * SNW + wave) * SKS;
#pragma unroll
        for (int jj = 0; jj < NF; ++jj) {
            const int idx = lane + 64 * jj;
            rf[set][jj] = zero4();
            if (FWD) {   // A_i[k0 + kr][cc * 8 ..]
                const int kr = idx / CPRF, cc = idx % CPRF;
                if (cc * 8 < rpad && k0 + kr < g.Kdim)
                    rf[set][jj] = load_chunk(F + (int64_t)(k0 + kr) * r + cc * 8, min(8, r - cc * 8), f_vec);
            } else {     // B_i[rho][k0 + c * 8 ..]
                const int rho = idx / XC, gk = k0 + (idx % XC) * 8;
                if (rho < r && gk < g.Kdim)
                    rf[set][jj] = *reinterpret_cast<const uint4*>(F + (int64_t)rho * g.ld + gk);
            }
        }
    };
    auto lstoreX = [&](int set) {
#pragma unroll
        for (int jj = 0; jj < NX; ++jj) {
            const int row = (lane / XC) + (64 / XC) * jj;
            *reinterpret_cast<uint4*>(Xs + xs_off(row, lane % XC)) = rx[set][jj];
        }
    };
    auto lstoreF = [&](int set) {
#pragma unroll
        for (int jj = 0; jj < NF; ++jj) {
            const int idx = lane + 64 * jj;
            if (FWD) {
                const int kr = idx / CPRF, cc = idx % CPRF;
                if (cc * 8 < rpad) *reinterpret_cast<uint4*>(Fs + kr * SBN_LD + cc * 8) = rf[set][jj];
            } else {
                const int rho = idx / XC;
                if (rho < rpad) *reinterpret_cast<uint4*>(Fs + rho * SF_LD + (idx % XC) * 8) = rf[set][jj];
            }
        }
    };
    const int lm = lane & 31, h = lane >> 5, gq = lane >> 4, j = lane & 15;
    auto compute = [&]() {
#pragma unroll
        for (int ks = 0; ks < SKS / 16; ++ks) {
            bf16x8 a[2];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) a[mb] = lds_read_frag(Xs + xs_off(mb * 32 + lm, ks * 2 + h));
#pragma unroll
            for (int nb = 0; nb < MAXNB; ++nb) {
                if (nb < nblk) {
                    bf16x8 b;
                    if (FWD) {
                        const u16* p = Fs + (ks * 16 + 8 * (gq >> 1) + (j >> 2)) * SBN_LD + nb * 32 + 16 * (gq & 1) + 4 * (j & 3);
                        b = lds_read_frag_tr(p, p + 4 * SBN_LD);
                    } else {
                        b = lds_read_frag(Fs + (nb * 32 + lm) * SF_LD + ks * 16 + h * 8);
                    }
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb) acc[mb][nb] = mfma32(a[mb], b, acc[mb][nb]);
                }
            }
        }
    };

    // LDS tiles are private to the wavefront and LDS operations of one wavefront execute in order,
    // so the loop needs no workgroup barrier: write the tile, start the next loads, compute.
    if (s_begin < s_end) {
        gloadX(s_begin, 0);
        if (DX == 2 && s_begin + 1 < s_end) gloadX(s_begin + 1, DX - 1);
        gloadF(s_begin, 0);
        if (DF == 2 && s_begin + 1 < s_end) gloadF(s_begin + 1, DF - 1);
        for (int st = s_begin; st < s_end; st += 2) {
            lstoreX(0);
            lstoreF(0);
            if (st + DX < s_end) gloadX(st + DX, 0);
            if (st + DF < s_end) gloadF(st + DF, 0);
            compute();
            if (st + 1 < s_end) {
                lstoreX(DX - 1);
                lstoreF(DF - 1);
                if (st + 1 + DX < s_end) gloadX(st + 1 + DX, DX - 1);
                if (st + 1 + DF < s_end) gloadF(st + 1 + DF, DF - 1);
                compute();
            }
        }
    }
    __syncthreads();

    // Add the eight partial tiles: NBUF wavefronts at a time write / add into NBUF fp32 buffers (SNW / NBUF
    // barrier rounds instead of SNW), then every thread sums the buffers in index order.  Fixed order, no atomics.
    constexpr int RLD = MAXNB * 32 + 4;                       // fp32 row of one buffer
    constexpr int NBUF = MAXNB == 2 ? 4 : 2;
    static_assert(NBUF * SR * RLD * 4 <= SNW * S_WAVE * 2, "reduction buffers fit in the staging area");
    float* red = reinterpret_cast<float*>(lds);
    for (int round = 0; round < SNW / NBUF; ++round) {
        if (wave / NBUF == round) {
            float* buf = red + (wave % NBUF) * (SR * RLD);
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int nb = 0; nb < MAXNB; ++nb) {
                    if (nb >= nblk) continue;
#pragma unroll
                    for (int q = 0; q < 16; ++q) {
                        const int row = mb * 32 + (q >> 2) * 8 + h * 4 + (q & 3);
                        float* d = buf + row * RLD + nb * 32 + lm;
                        *d = (round == 0) ? acc[mb][nb][q] : (*d + acc[mb][nb][q]);
                    }
                }
        }
        __syncthreads();
    }
    const int64_t so = g.pv.soff[i];
    const int seg0 = g.pv.off[i];
    u16* out = g.out + so + (int64_t)(row0 - seg0) * r;
    for (int idx = tid; idx < rows * r; idx += 64 * SNW) {
        const int row = idx / r, col = idx - row * r;
        float v = 0.f;
#pragma unroll
        for (int b = 0; b < NBUF; ++b) v += red[b * (SR * RLD) + row * RLD + col];
        out[idx] = f2bf(s * v);
    }
}

// WIDE: the launch may contain row blocks of adapters with ranks above 64; those take the wide-rank build, all others
// the narrow one (the branch is uniform over the workgroup).  The list puts the wide blocks first: they run longest.
template <bool FWD, bool WIDE>
__global__ __launch_bounds__(64 * SNW) void shrink_kernel(ShrinkArgs g) {
    __shared__ __attribute__((aligned(16))) u16 lds[163840 / 2];
    const Entry4 e = g.pv.row_blocks[blockIdx.x];      // the canonical 64-row blocks
    if (WIDE && g.pv.rank[e.a] > 64) shrink_body<FWD, 4, 32, 2, 1>(g, e, lds);
    else shrink_body<FWD, 2, 64, 2, 1>(g, e, lds);
}

// GEMM-tiled shrink / dShrink, used when the contraction is a multiple of 64 (shrink: for adapters whose rank is a multiple of 4).
// Per 64-wide contraction step the work group shares one X / dY tile [64 rows][64] and one adapter tile (of A_i, read
// with the transposing load, or of B_i), both brought in by direct global -> LDS loads into a ring of stages (no staging
// registers, no LDS stores, the loads of all but the current step in flight), one barrier per step.  Every output block
// is accumulated by one wavefront over the whole contraction, so there is no cross-wavefront reduction and the result is
// deterministic.  RB16 = 16-wide rank blocks the body is built for:
//   4 (ranks <= 64): adapter tile 8 KB, nine 16 KB stages; wavefront w owns row block w & 3 and rank blocks 2 (w >> 2) + {0, 1};
//   8 (ranks <= 128): adapter tile 16 KB, six 24 KB stages; wavefront w owns row block w & 3 and rank blocks 4 (w >> 2) + {0..3}.
// Against the register-staged builds above it keeps more bytes in flight with an eighth of the registers, has no LDS stores
// and no reduction epilogue: 8 x 2048 tokens, k = 4096: rank 16 forward 41 -> 33 us, rank 128 68 -> 51 us.
// Tiles are unpadded and XOR-swizzled as in the fused GEMM: 128-byte rows of a tile read along its rows keep chunk c of row t
// at c ^ (t & 7); the A_i tile [k][ranks], read with the transposing load, keeps 32-byte unit u of row k at u ^ nn_swz(k)
// (256-byte rows) or u ^ (((k >> 1) & 1) | (((k >> 3) & 1) << 1)) (128-byte rows).  Rows past the block and ranks past r_i
// are clamped to valid addresses; they only feed outputs that are not stored.
//   8 with ROWS = 128 (ranks 65..128, the wide rank class, whose row blocks are 128 rows): X / dY tile 16 KB, adapter tile 16 KB,
//     five 32 KB stages; wavefront w owns row block w (of eight) and all eight rank blocks.  With 64-row blocks the adapter tile was
//     twice the X tile and both go through the same load path of the CU; 128 rows halve that traffic per X byte.
template <bool FWD, int RB16, bool DENSE = false, int ROWS = 64>
__device__ __forceinline__ void shrink_tiled_body(const ShrinkArgs& g, const Entry4 e, unsigned char* lds) {
    static_assert(FWD || !DENSE, "the dense adapter tile is a layout of A_i");
    static_assert(ROWS == 64 || (ROWS == 128 && RB16 == 8 && !DENSE), "128-row blocks: wide rank class, swizzled adapter tile");
    constexpr int ST_XT = ROWS * 128;               // X / dY tile bytes
    constexpr int FT = RB16 * 2048;                 // adapter tile bytes
    constexpr int STAGE = ST_XT + FT;
    constexpr int NST = ROWS == 128 ? 5 : RB16 == 8 ? 6 : 9;   // ring stages (144 KB; 160 KB with 128-row blocks)
    constexpr int NX = ROWS / 64;                   // X-tile loads per wavefront per step
    constexpr int NF = RB16 / 4;                    // adapter-tile loads per wavefront per step
    constexpr int NCB = ROWS == 128 ? RB16 : RB16 / 2;   // rank blocks per wavefront
    constexpr int FROW = RB16 * 32;                 // FWD: bytes per contraction row of the A_i tile
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g4 = lane >> 4;
    const int i = e.a, row0 = e.c, rows = e.d;
    const int r = g.pv.rank[i];
    const u16* F = (const u16*)(FWD ? g.pv.ptrs[i].A : g.pv.ptrs[i].B);
    const float s = FWD ? 1.0f : g.pv.scale[i];
    // swizzle key of contraction row k of the A_i tile
    auto fkey = [](int k) { return RB16 == 8 ? nn_swz(k) : (((k >> 1) & 1) | (((k >> 3) & 1) << 1)); };

    // per-lane byte offsets of the direct loads this wavefront issues per step
    unsigned voffX[NX], voffF[NF];
    {
#pragma unroll
        for (int j = 0; j < NX; ++j) {
            const int row = 8 * (NX * wave + j) + (lane >> 3);
            voffX[j] = (unsigned)(((int64_t)min(row, rows - 1) * g.ld + (((lane & 7) ^ (lane >> 3)) << 3)) * 2);
        }
#pragma unroll
        for (int j = 0; j < NF; ++j) {
            const int kb = NF * wave + j;        // 1 KB piece of the adapter tile
            if (DENSE) {   // the step's 64 rows of A_i are 128 r contiguous bytes: copied as they are
                voffF[j] = (unsigned)min(kb * 1024 + lane * 16, 128 * r - 16);
            } else if (FWD) {     // piece = 1024 / FROW contraction rows of FROW bytes
                constexpr int LPR = FROW / 16;   // lanes (16-byte chunks) per row
                const int krow = kb * (64 / LPR) + lane / LPR, pos = lane % LPR;
                const int chunk = min((((pos >> 1) ^ fkey(krow)) << 1) | (pos & 1), r / 8 - 1);
                voffF[j] = (unsigned)((krow * r + chunk * 8) * 2);
            } else {       // piece = 8 rank rows of 128 bytes
                const int rho = 8 * kb + (lane >> 3);
                voffF[j] = (unsigned)(((int64_t)min(rho, r - 1) * g.ld + (((lane & 7) ^ (lane >> 3)) << 3)) * 2);
            }
        }
    }
    const int steps = g.Kdim / 64;
    const char* baseX = uniform_ptr(g.src + (int64_t)row0 * g.ld);
    const char* baseF = uniform_ptr(F);
    const int64_t stepF = FWD ? (int64_t)64 * __builtin_amdgcn_readfirstlane(r) * 2 : 128;
    const unsigned lds0 = (unsigned)(uintptr_t)lds;
    int issued = 0, slot_in = 0;          // next step to load and the ring slot it goes to
    auto issue = [&]() {                  // past the last step the last one is loaded again (keeps the wait counts uniform)
        const int t = min(issued, steps - 1);
        const unsigned dst = lds0 + slot_in * STAGE;
#pragma unroll
        for (int j = 0; j < NX; ++j) dma16(voffX[j], baseX + (int64_t)t * 128, dst + (NX * wave + j) * 1024);
#pragma unroll
        for (int j = 0; j < NF; ++j) dma16(voffF[j], baseF + t * stepF, dst + ST_XT + (NF * wave + j) * 1024);
        ++issued;
        slot_in = slot_in == NST - 1 ? 0 : slot_in + 1;
    };

    const int rb = ROWS == 128 ? wave : (wave & 3), ch = ROWS == 128 ? 0 : (wave >> 2);
    f32x4 acc[NCB];
#pragma unroll
    for (int j = 0; j < NCB; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int xrow = 16 * rb + l16;
    const int vq = fkey(8 * g4 + (l16 >> 2));      // key of the A_i tile rows this lane reads (rows +4, +32 share it)
    auto compute = [&](int slot) {
        const unsigned char* Xs = lds + slot * STAGE;
        const unsigned char* Fs = Xs + ST_XT;
#pragma unroll
        for (int k32 = 0; k32 < 2; ++k32) {
            const bf16x8 a = lds_read_frag(reinterpret_cast<const u16*>(Xs + xrow * 128 + (((k32 * 4 + g4) ^ (l16 & 7)) << 4)));
#pragma unroll
            for (int j = 0; j < NCB; ++j) {
                const int cb = ch * NCB + j;
                if (cb * 16 >= r) continue;
                bf16x8 b;
                if (DENSE) {   // rows of 2 r bytes, unswizzled; a lane past r_i reads ranks 0..3 again (output not stored)
                    const int rk = 16 * cb + (l16 & 3) * 4;
                    const unsigned char* p = Fs + (k32 * 32 + 8 * g4 + (l16 >> 2)) * (2 * r) + (rk < r ? rk * 2 : 0);
                    b = lds_read_frag_tr(reinterpret_cast<const u16*>(p), reinterpret_cast<const u16*>(p + 8 * r));
                } else if (FWD) {
                    const unsigned char* p = Fs + (k32 * 32 + 8 * g4 + (l16 >> 2)) * FROW + ((cb ^ vq) << 5) + (l16 & 3) * 8;
                    b = lds_read_frag_tr(reinterpret_cast<const u16*>(p), reinterpret_cast<const u16*>(p + 4 * FROW));
                } else {
                    const int rho = 16 * cb + l16;
                    b = lds_read_frag(reinterpret_cast<const u16*>(Fs + rho * 128 + (((k32 * 4 + g4) ^ (l16 & 7)) << 4)));
                }
                acc[j] = mfma16(a, b, acc[j]);
            }
        }
    };

    for (int t = 0; t < NST - 1; ++t) issue();
    int slot = 0;
    for (int t = 0; t < steps; ++t) {
        // step t has landed (only the loads of the NST - 2 later steps may be in flight) and every wavefront is past
        // step t-1, whose slot the next load overwrites
        if (RB16 == 8) asm volatile("s_waitcnt vmcnt(12)\n\ts_barrier" ::: "memory");
        else           asm volatile("s_waitcnt vmcnt(14)\n\ts_barrier" ::: "memory");
        static_assert((NX + NF) * (NST - 2) == (RB16 == 8 ? 12 : 14), "wait count = loads of the steps that may still be in flight");
        issue();
        compute(slot);
        slot = slot == NST - 1 ? 0 : slot + 1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // no load may still be writing LDS when the work group ends

    // lane (l16, g4) holds rows 16 rb + 4 g4 + q, rank 16 cb + l16
    const int64_t so = g.pv.soff[i];
    const int seg0 = g.pv.off[i];
    u16* out = g.out + so + (int64_t)(row0 - seg0) * r;
#pragma unroll
    for (int j = 0; j < NCB; ++j) {
        const int rank = 16 * (ch * NCB + j) + l16;
        if (rank >= r) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int row = 16 * rb + 4 * g4 + q;
            if (row < rows) out[(int64_t)row * r + rank] = f2bf(s * acc[j][q]);
        }
    }
}

// WIDE: the launch may contain row blocks of adapters with ranks above 64.  MIXED: it may contain adapters whose rank is
// not a multiple of 8 (forward form only): a rank that is a multiple of 4 takes the tiled body with the adapter tile kept
// dense in LDS (rows of 2 r bytes: 8-byte granules, which is what one lane of the transposing load reads), any other rank
// the register-staged body.  Uniform branches per work group.
// Row blocks of the wide class have 128 rows (kBlockRowsWide); the bodies built for 64 rows take such a block as two halves.
template <bool FWD, bool WIDE, bool MIXED>
__global__ __launch_bounds__(64 * SNW) void shrink_tiled_kernel(ShrinkArgs g) {
    __shared__ __attribute__((aligned(1024))) unsigned char lds[(MIXED || WIDE) ? 163840 : 147456];
    const Entry4 e = g.pv.class_blocks[blockIdx.x];
    const int r = g.pv.rank[e.a];
    if (WIDE && r > 64) {
        if (!MIXED || (r & 7) == 0) {
            shrink_tiled_body<FWD, 8, false, kBlockRowsWide>(g, e, lds);
        } else {
            for (int h = 0; h < e.d; h += SR) {       // (uniform)
                const Entry4 half{e.a, e.b, e.c + h, min(SR, e.d - h)};
                if (h) __syncthreads();               // every wavefront is done with the first half's tiles
                if (FWD && (r & 7) == 4) shrink_tiled_body<FWD, 8, FWD>(g, half, lds);
                else shrink_body<FWD, 4, 32, 2, 1>(g, half, reinterpret_cast<u16*>(lds));
            }
        }
    } else if (MIXED && FWD && (r & 7) == 4) {
        shrink_tiled_body<FWD, 4, FWD>(g, e, lds);
    } else if (MIXED && (r & 7) != 0) {
        shrink_body<FWD, 2, 64, 2, 1>(g, e, reinterpret_cast<u16*>(lds));
    } else {
        shrink_tiled_body<FWD, 4>(g, e, lds);
    }
}

template <bool FWD>
static void launch_shrink(mlora_plan* p, ShrinkArgs a, hipStream_t st) {
    const dim3 block(64 * SNW);
    // the tiled kernels address rows with 32-bit lane offsets: rows of at most 2^22 elements
    const bool tiled = a.Kdim >= 64 && a.Kdim % 64 == 0 && a.ld <= ((int64_t)1 << 22);
    const bool wide = p->n_blocks_wide != 0;
    // (the forward form reads A_i in 16-byte chunks of a rank row: row blocks of adapters whose rank is not a multiple of 8
    // keep the register-staged body; B_i is read along its rows, any rank will do)
    const bool mixed = FWD && !p->ranks_mult8;
    // the tiled kernels walk the class table (wide class first, 128-row blocks); the register-staged ones the canonical 64-row blocks
    const dim3 grid(tiled ? p->n_blocks_wide + p->n_blocks_narrow : p->n_row_blocks);
    if (tiled && !mixed) {
        if (!wide) hipLaunchKernelGGL((shrink_tiled_kernel<FWD, false, false>), grid, block, 0, st, a);
        else       hipLaunchKernelGGL((shrink_tiled_kernel<FWD, true, false>), grid, block, 0, st, a);
    } else if (tiled) {
        if (!wide) hipLaunchKernelGGL((shrink_tiled_kernel<FWD, false, true>), grid, block, 0, st, a);
        else       hipLaunchKernelGGL((shrink_tiled_kernel<FWD, true, true>), grid, block, 0, st, a);
    } else {
        if (!wide) hipLaunchKernelGGL((shrink_kernel<FWD, false>), grid, block, 0, st, a);
        else       hipLaunchKernelGGL((shrink_kernel<FWD, true>), grid, block, 0, st, a);
    }
}

// =========================================================================================
// Weight gradients (token reductions):
//   dA_i[kappa][rho] = sum_t X[t][kappa] dS[t][rho]          out [k][r]
//   dB_i[rho][nu]    = s_i sum_t S[t][rho] dY[t][nu]         out [r][n]  (stored transposed)
// Work item = (token chunk of one adapter, 128-column panel of X or dY).  Both MFMA operands
// have the token index as the row index in memory, so both are read with transposing loads.
// A chunk that covers its whole segment stores the result directly; otherwise fp32 partials go
// to the workspace and a second kernel adds them in chunk order (no atomics, deterministic).
// The kernel is a stream of X / dY, and what it sustains depends on the bytes a CU keeps in flight, i.e. on how
// many workgroups fit a CU: it is built per rank class MAXNB (32-wide rank blocks: 1, 2 or 4, chosen per plan from
// the largest rank), which sizes the accumulators, the prefetch registers and the S / dS tile.  LDS tiles are
// unpadded and XOR-swizzled in 64-byte units so that the transposing reads (4 token rows x 64 bytes per half
// wavefront) are conflict free: the panel tile [64 tokens][128] and a 128-wide S tile keep unit u of token row t at
// u ^ (t & 3), a 64-wide S tile at u ^ ((t >> 1) & 1), a 32-wide one needs none.  Two stages: 40 / 48 / 64 KB.
// =========================================================================================
constexpr int WP = kWgradPanelCols;   // panel columns (128)
constexpr int WT = 64;           // tokens per step
constexpr int WX_TILE = WT * 128;     // panel tile (elements)

struct WgradArgs {
    const u16* X; const u16* dY; const u16* S; const u16* dS;
    float* partials;
    int32_t panels_k, panels_n;
    PlanView pv;
    int32_t accumulate;        // dA_i, dB_i += result (MLORA_FLAG_ACCUM_GRADS)
    int32_t chunk_base;        // first entry of the chunk table this launch covers (the table is ordered by rank class)
};

// One work item; isA: a dA_i item (panel of X against dS_i), else a dB_i item (panel of dY against S_i).  The two forms
// are separate instantiations (the kernel branches once, uniformly): they use the MFMA operands the other way round.
// NW: wavefronts per work group: 4, or 8 for the wide build (64 columns x 32 ranks per wavefront: half the accumulators and half
// the prefetch registers per wavefront, 128 registers instead of 240, so twice the wavefronts per CU hide the latency of the
// same two work groups' loads; weight gradients of 4 x 2048 tokens at rank 128, 8192 + 28672 wide: 190 -> 173 us)
template <int MAXNB, bool isA, int NW = 4>
__device__ __forceinline__ void wgrad_body(const WgradArgs& g, u16* lds, const int ce, const int panel) {
    constexpr int NTHW = 64 * NW;
    static_assert(NW == 4 || (NW == 8 && MAXNB == 4), "8 wavefronts: wide build only");
    constexpr int SW = MAXNB * 32;                 // S / dS tile width (elements)
    constexpr int CPRS = SW / 8;                   // 16-byte chunks per S tile row
    constexpr int W_STAGE = WX_TILE + WT * SW;     // elements per stage
    // byte offset of element column c (multiple of 4) of token row t
    auto x_off = [](int t, int c) { return t * 256 + ((((c >> 5) ^ (t & 3)) << 6) | ((c & 31) << 1)); };
    auto s_off = [](int t, int c) {
        const int u = c >> 5;
        const int us = MAXNB == 4 ? (u ^ (t & 3)) : MAXNB == 2 ? (u ^ ((t >> 1) & 1)) : u;
        return t * (SW * 2) + ((us << 6) | ((c & 31) << 1));
    };
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const Entry4 e = g.pv.wgrad_chunks[ce];
    const int i = e.a, chunk = e.b, row0 = e.c, rows = e.d;
    const int r = g.pv.rank[i];
    const int rpad = (r + 31) & ~31;
    const int nblk = rpad / 32;
    const int64_t so = g.pv.soff[i];
    const int seg0 = g.pv.off[i];
    const int width = (int)(isA ? g.pv.k : g.pv.n);
    const u16* big = isA ? g.X : g.dY;
    const u16* small = (isA ? g.dS : g.S) + so + (int64_t)(row0 - seg0) * r;
    const int col0 = panel * WP;
    const bool s_vec = ((r & 7) == 0) && ((so & 7) == 0);
    // ranks that are multiples of 4 but not of 8: 8-byte halves of a chunk, loaded straight into the prefetch registers
    // (the element-wise path combines what it loads at once, which would make every step wait for its own loads)
    const bool s_v8 = !s_vec && ((r & 3) == 0) && ((so & 3) == 0) && ((reinterpret_cast<uintptr_t>(isA ? g.dS : g.S) & 7) == 0);

    // Accumulator blocks of a wavefront: NCB 32-column blocks x NRB 32-rank blocks.  Up to 64 ranks every wavefront takes
    // 32 panel columns against all ranks; the widest build splits the work group 2 x 4 (64 columns x 32 ranks per wavefront;
    // with four wavefronts it was 2 x 2 with 64 x 64 each),
    // which reads a fifth less from LDS for the same MFMAs - that build is bound by LDS bandwidth.
    constexpr int NCB = MAXNB == 4 ? 2 : 1;
    constexpr int NRB = MAXNB == 4 ? (NW == 8 ? 1 : 2) : MAXNB;
    const int cwave = MAXNB == 4 ? (wave & 1) * 64 : wave * 32;      // first panel column of this wavefront
    const int rb0 = MAXNB == 4 ? (wave >> 1) * NRB : 0;              // its first rank block
    f32x16 acc[NCB * NRB];
#pragma unroll
    for (int nb = 0; nb < NCB * NRB; ++nb)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[nb][q] = 0.f;

    const int nt = (rows + WT - 1) / WT;
    constexpr int NRA = 1024 / NTHW, NRS = MAXNB * 256 / NTHW;      // 16-byte chunks per thread: panel tile, S tile
    uint4 ra[2][NRA], rb[2][NRS];   // two register sets: tiles of even / odd index, two steps of loads in flight
    auto gload = [&](int tt, int set) {
        const int t0 = tt * WT;
#pragma unroll
        for (int jj = 0; jj < NRA; ++jj) {
            const int trow = (tid >> 4) + (NTHW / 16) * jj, cc = tid & 15;
            const int col = col0 + cc * 8;
            ra[set][jj] = (t0 + trow < rows && col < width)
                              ? load_streaming(big + (int64_t)(row0 + t0 + trow) * width + col) : zero4();
        }
#pragma unroll
        for (int jj = 0; jj < NRS; ++jj) {
            const int idx = tid + NTHW * jj, trow = idx / CPRS, cc = idx % CPRS;
            rb[set][jj] = zero4();
            if (t0 + trow < rows && cc * 8 < r) {
                const u16* ps = small + (int64_t)(t0 + trow) * r + cc * 8;
                if (s_v8) {
                    const uint2 lo = *reinterpret_cast<const uint2*>(ps);
                    rb[set][jj].x = lo.x; rb[set][jj].y = lo.y;
                    if (r - cc * 8 >= 8) {
                        const uint2 hi = *reinterpret_cast<const uint2*>(ps + 4);
                        rb[set][jj].z = hi.x; rb[set][jj].w = hi.y;
                    }
                } else {
                    rb[set][jj] = load_chunk(ps, min(8, r - cc * 8), s_vec);
                }
            }
        }
    };
    auto lstore = [&](int stage, int set) {
        unsigned char* Xs = reinterpret_cast<unsigned char*>(lds + stage * W_STAGE);
        unsigned char* Ss = Xs + WX_TILE * 2;
#pragma unroll
        for (int jj = 0; jj < NRA; ++jj) {
            const int trow = (tid >> 4) + (NTHW / 16) * jj, cc = tid & 15;
            *reinterpret_cast<uint4*>(Xs + x_off(trow, cc * 8)) = ra[set][jj];
        }
#pragma unroll
        for (int jj = 0; jj < NRS; ++jj) {
            const int idx = tid + NTHW * jj, trow = idx / CPRS, cc = idx % CPRS;
            *reinterpret_cast<uint4*>(Ss + s_off(trow, cc * 8)) = rb[set][jj];
        }
    };
    const int lm = lane & 31, h = lane >> 5, gq = lane >> 4, j = lane & 15;
    auto compute = [&](int stage) {
        const unsigned char* Xs = reinterpret_cast<const unsigned char*>(lds + stage * W_STAGE);
        const unsigned char* Ss = Xs + WX_TILE * 2;
#pragma unroll
        for (int ks = 0; ks < WT / 16; ++ks) {
            const int trow = ks * 16 + 8 * (gq >> 1) + (j >> 2);    // token rows trow and trow + 4 share their swizzle keys
            const int coff = 16 * (gq & 1) + 4 * (j & 3);
            bf16x8 a[NCB];
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                const unsigned char* pa = Xs + x_off(trow, cwave + cb * 32 + coff);
                a[cb] = lds_read_frag_tr(reinterpret_cast<const u16*>(pa), reinterpret_cast<const u16*>(pa + 4 * 256));
            }
#pragma unroll
            for (int rbl = 0; rbl < NRB; ++rbl) {
                if (rb0 + rbl < nblk) {
                    const unsigned char* pb = Ss + s_off(trow, (rb0 + rbl) * 32 + coff);
                    const bf16x8 b = lds_read_frag_tr(reinterpret_cast<const u16*>(pb), reinterpret_cast<const u16*>(pb + 4 * SW * 2));
                    // dA_i items compute the transposed block (ranks down the accumulator rows), so that for both outputs a
                    // lane ends up with 4 consecutive elements of an output row
#pragma unroll
                    for (int cb = 0; cb < NCB; ++cb)
                        acc[cb * NRB + rbl] = isA ? mfma32(b, a[cb], acc[cb * NRB + rbl]) : mfma32(a[cb], b, acc[cb * NRB + rbl]);
                }
            }
        }
    };
    // Tile u travels in register set u & 1 and is computed from LDS stage u & 1.  At the top of step t
    // tile t+1 is written to the other stage (last read before the previous barrier) and the loads
    // of tile t+3 start, so every tile's loads have two whole steps to land.
    if (nt > 0) {
        gload(0, 0);
        if (nt > 1) gload(1, 1);
        lstore(0, 0);
        if (nt > 2) gload(2, 0);
    }
    __syncthreads();
    for (int tt = 0; tt < nt; tt += 2) {
        if (tt + 1 < nt) lstore(1, 1);
        if (tt + 3 < nt) gload(tt + 3, 1);
        compute(0);
        __syncthreads();
        if (tt + 1 < nt) {
            if (tt + 2 < nt) lstore(0, 0);
            if (tt + 4 < nt) gload(tt + 4, 0);
            compute(1);
            __syncthreads();
        }
    }

    const int nchunks = g.pv.wgrad_chunk_start[i + 1] - g.pv.wgrad_chunk_start[i];
    const float s = isA ? 1.0f : g.pv.scale[i];
    const int64_t kk = g.pv.k, nn = g.pv.n;
    // Accumulator element q of lane (lm, h) of block nb is at (row 8 (q >> 2) + 4 h + (q & 3), column lm) of a 32 x 32 block.
    //   dB_i item: rows = panel columns, lane column = rank: out[rho][c], 4 consecutive c per (lane, q >> 2)
    //   dA_i item (transposed block): rows = ranks, lane column = panel column: out[c][rho], 4 consecutive rho
    // so every lane stores 8-byte (bf16) or 16-byte (fp32 partial) pieces; ranks that are not multiples of 4 and
    // the ragged edge go element by element.
    u16* out = (u16*)(isA ? g.pv.ptrs[i].dA : g.pv.ptrs[i].dB);
    float* part = nchunks == 1 ? nullptr
                               : g.partials + g.pv.part_off[i] + (int64_t)chunk * (kk + nn) * r + (isA ? 0 : kk * r);
    const bool vec = isA ? ((r & 3) == 0) : ((nn & 3) == 0);
    const bool part_vec = vec && ((reinterpret_cast<uintptr_t>(part) & 15) == 0);
#pragma unroll
    for (int ab = 0; ab < NCB * NRB; ++ab) {
        const int nb = rb0 + ab % NRB, cbase = cwave + (ab / NRB) * 32;
        if (nb >= nblk) continue;
#pragma unroll
        for (int qg = 0; qg < 4; ++qg) {
            const int inner = 8 * qg + 4 * h;
            const int c = col0 + cbase + (isA ? lm : inner);
            const int rho = nb * 32 + (isA ? inner : lm);
            if (c >= width || rho >= r) continue;
            const int64_t idx0 = isA ? ((int64_t)c * r + rho) : ((int64_t)rho * nn + c);
            const int nvalid = min(4, isA ? r - rho : width - c);
            float v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = s * acc[ab][4 * qg + q];
            if (part) {
                if (part_vec && nvalid == 4) {
                    *reinterpret_cast<float4*>(part + idx0) = make_float4(v[0], v[1], v[2], v[3]);
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (q < nvalid) part[idx0 + q] = v[q];
                }
            } else if (vec && nvalid == 4) {
                uint2* dst = reinterpret_cast<uint2*>(out + idx0);
                if (g.accumulate) {
                    const uint2 old = *dst;
                    v[0] += __uint_as_float(old.x << 16); v[1] += __uint_as_float(old.x & 0xffff0000u);
                    v[2] += __uint_as_float(old.y << 16); v[3] += __uint_as_float(old.y & 0xffff0000u);
                }
                *dst = make_uint2(pack2(v[0], v[1]), pack2(v[2], v[3]));
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (q < nvalid) out[idx0 + q] = f2bf(g.accumulate ? v[q] + bf2f(out[idx0 + q]) : v[q]);
            }
        }
    }
}

// (the register budget is stated per build: the work groups per CU that its LDS footprint allows, one wavefront of each per SIMD)
template <int MAXNB, int NW = 4>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(NW == 8 ? 4 : MAXNB == 4 ? 2 : MAXNB == 2 ? 3 : 4)))
void wgrad_kernel(WgradArgs g) {
    __shared__ __attribute__((aligned(16))) u16 lds[2 * (WX_TILE + WT * MAXNB * 32)];
    const int panels = g.panels_k + g.panels_n;
    const int ce = g.chunk_base + blockIdx.x / panels;
    const int panel = blockIdx.x % panels;
    if (panel < g.panels_k) wgrad_body<MAXNB, true, NW>(g, lds, ce, panel);
    else wgrad_body<MAXNB, false, NW>(g, lds, ce, panel - g.panels_k);
}

// Adds the chunk partials of one adapter in chunk order and rounds once.  blockIdx.y walks the adapters that have
// partials; a thread owns 4 consecutive elements (k, n are multiples of 8 on this path, so a group never straddles
// the dA_i / dB_i boundary and every access is 16- resp. 8-byte aligned).
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(WgradArgs g, const int32_t* list) {
    const int i = list[blockIdx.y];
    const int nchunks = g.pv.wgrad_chunk_start[i + 1] - g.pv.wgrad_chunk_start[i];
    const int r = g.pv.rank[i];
    const int64_t kk = g.pv.k, nn = g.pv.n;
    const int64_t per = (kk + nn) * r;
    const int64_t idx = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (idx >= per) return;
    const float* part = g.partials + g.pv.part_off[i] + idx;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int c = 0; c < nchunks; ++c) {
        const float4 t = *reinterpret_cast<const float4*>(part + (int64_t)c * per);
        v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
    }
    uint2* out = reinterpret_cast<uint2*>(idx < kk * r ? (u16*)g.pv.ptrs[i].dA + idx : (u16*)g.pv.ptrs[i].dB + (idx - kk * r));
    if (g.accumulate) {
        const uint2 old = *out;
        v.x += __uint_as_float(old.x << 16); v.y += __uint_as_float(old.x & 0xffff0000u);
        v.z += __uint_as_float(old.y << 16); v.w += __uint_as_float(old.y & 0xffff0000u);
    }
    *out = make_uint2(pack2(v.x, v.y), pack2(v.z, v.w));
}

// Zero-fills dA_i, dB_i of adapters that have a rank but no tokens (no work item reaches them).
__global__ void wgrad_zero_empty_kernel(PlanView pv) {
    const int i = blockIdx.y;
    const int r = pv.rank[i];
    if (r == 0 || pv.off[i + 1] != pv.off[i]) return;
    const int64_t kk = pv.k, nn = pv.n;
    const int64_t per = (kk + nn) * r;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < per; idx += (int64_t)gridDim.x * 256) {
        if (idx < kk * r) ((u16*)pv.ptrs[i].dA)[idx] = 0;
        else ((u16*)pv.ptrs[i].dB)[idx - kk * r] = 0;
    }
}

// =========================================================================================
// Expand-add (MLORA_FLAG_LORA_ONLY; the paper's decoupled "fused GEMM-add", Sec. 5.1 / App. A.1):
//   fwd  Y_i  += s_i S_i B_i        bwd  dX_i += dS_i A_i^T        in place, one rounding.
// A pure read-modify-write stream of the output with a small contraction on top.  Work item = (64-row block of
// one adapter, 128 or 256 columns); 4 or 8 wavefronts (2 x 2 / 2 x 4), each 32 rows x 64 columns = 2 x 4 blocks of 16x16x32 MFMAs.
// The old output tile is not added after the fact: it is loaded in 16-byte row chunks, which is exactly the MFMA
// operand layout of a [row][32 columns] fragment, and multiplied by a constant identity operand into the fp32
// accumulators (bf16 x 1.0 is exact), so the accumulators start as the old tile and the rank steps add on top.
// That leaves no separate fp32 add, no second register copy of the tile and a bf16-only transpose in the
// epilogue (operands are swapped so that a lane holds 4 consecutive columns, as in the fused GEMM).
// fwd: B_i is [r][n] (contraction index outermost), so the work group stages its [r][128] tile in LDS once
// (256-byte rows, 16-byte chunk c of row k at c ^ (nn_swz(k) << 1)) and reads it with the transposing load;
// bwd: A_i is [k][r], contraction contiguous: the work group stages its 128 rows in LDS (padded pitch) and reads plain fragments.
// =========================================================================================
constexpr int XE_LD = 64 + 8;         // epilogue staging row of one wavefront (elements)

struct ExpandArgs {
    u16* C; int64_t ldc;     // Y [T,n] or dX [T,k]
    const u16* E;            // ragged S or dS
    int32_t Ncols, col_tiles;
    int32_t stream_out;      // streaming stores for the output
    int32_t stream_in;       // non-temporal loads for the old output tile
    const Entry4* blocks;    // the row blocks this launch covers: one rank class of pv.class_blocks
    PlanView pv;
};

// MAXKS: 32-wide rank steps the kernel is built for (2: every rank <= 64, 4: ranks up to 128).
// All loads of a work item (old output tile, S fragments, B_i / A_i^T operands) are issued before the
// first MFMA, so a wavefront pays the memory latency once; many small work items per CU overlap each other.
// XCW: 64-column wavefront columns of a work item (2: 128 output columns, 4 wavefronts; 4: 256 columns, 8 wavefronts - every
// work item fetches its 64 rows of S_i / dS_i again, so a strip twice as wide halves that traffic; used for the narrow rank class,
// whose adapter tile stays small enough for two work groups per CU: expand-add of configs 3-5 4-6 % faster; the wide class with
// 256 columns fits one work group per CU and is 10-20 % slower).
template <bool FWD, int MAXKS, int XCW>
__global__ __launch_bounds__(128 * XCW) void expand_add_kernel(ExpandArgs g) {
    constexpr int XC = 64 * XCW;                                 // output columns per work item
    constexpr int NTH = 128 * XCW;                               // threads
    constexpr int BROW = XC * 2;                                 // fwd: bytes per rank row of the staged B_i tile
    constexpr int AT_PITCH = MAXKS * 64 + 16;                    // bwd: bytes per column of the staged A_i rows (padded: bank spread)
    constexpr int BT_BYTES = FWD ? MAXKS * 32 * BROW : XC * AT_PITCH;   // staged B_i tile / A_i rows
    constexpr int EP_WAVE = 32 * XE_LD * 2;                      // bytes of epilogue staging per wavefront
    // 256-column forward strips stage the work item's 64 rows of S_i in LDS once (one 16-byte load per thread) instead of every
    // wavefront fetching the fragments of its rows itself (four wavefronts share each row)
    constexpr bool SLDS = FWD && XCW == 4;
    constexpr int ST_PITCH = MAXKS * 64 + 16;                    // bytes per staged row of S_i (padded: bank spread)
    constexpr int ST_BYTES = SLDS ? 64 * ST_PITCH : 0;
    __shared__ __attribute__((aligned(16))) unsigned char lds[BT_BYTES + ST_BYTES + 2 * XCW * EP_WAVE];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave / XCW, wc = wave % XCW;
    const int l16 = lane & 15, g4 = lane >> 4;
    // row-block-major: consecutive workgroups cover adjacent column tiles of the same 64 rows
    constexpr int PARTS = (MAXKS == 4 ? kBlockRowsWide : kBlockRows) / 64;   // 64-row work items per block of this class's table
    const int bsel = blockIdx.x / g.col_tiles;
    const Entry4 e = g.blocks[bsel / PARTS];
    const int ct = blockIdx.x % g.col_tiles;
    const int part = bsel % PARTS;
    const int i = e.a, row0 = e.c + 64 * part, rows = min(64, e.d - 64 * part);
    if (PARTS > 1 && rows <= 0) return;          // a last block of at most 64 rows has no second part (uniform)
    const int r = g.pv.rank[i];
    const int ksteps = (r + 31) / 32;
    const int64_t so = g.pv.soff[i];
    const int seg0 = g.pv.off[i];
    const float s = FWD ? g.pv.scale[i] : 1.0f;
    const u16* F = (const u16*)(FWD ? g.pv.ptrs[i].B : g.pv.ptrs[i].A);
    const int colw = ct * XC + wc * 64;          // first column of this wavefront
    const bool stream_in = g.stream_in != 0;

    // 1. old output tile as MFMA operand fragments: [16 rows][32 columns], lane = (row l16, 8 columns at 8 g4)
    uint4 old[2][2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int kg = 0; kg < 2; ++kg) {
            const int row = wr * 32 + rb * 16 + l16, col = colw + kg * 32 + g4 * 8;
            old[rb][kg] = (row < rows && col < g.Ncols)
                              ? (stream_in ? load_streaming(g.C + (int64_t)(row0 + row) * g.ldc + col) : *reinterpret_cast<const uint4*>(g.C + (int64_t)(row0 + row) * g.ldc + col)) : zero4();
        }
    // 2. S / dS fragments: [16 rows][32 ranks]
    const bool e_vec = ((r & 7) == 0) && ((so & 7) == 0);
    uint4 sv[2][MAXKS];
    constexpr int SCH = (64 * MAXKS * 4) / NTH;          // staged S chunks per thread
    uint4 sst[SCH > 0 ? SCH : 1];
    if (SLDS) {
#pragma unroll
        for (int jj = 0; jj < SCH; ++jj) {
            const int idx = tid + NTH * jj, row = idx / (MAXKS * 4), cc = idx % (MAXKS * 4);
            sst[jj] = zero4();
            if (row < rows && cc * 8 < r)
                sst[jj] = load_chunk_a8(g.E + so + (int64_t)(row0 + row - seg0) * r + cc * 8, min(8, r - cc * 8), e_vec);
        }
    } else {
#pragma unroll
        for (int ks = 0; ks < MAXKS; ++ks)
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                const int row = wr * 32 + rb * 16 + l16, rho = ks * 32 + g4 * 8;
                sv[rb][ks] = zero4();
                if (ks < ksteps && row < rows && rho < r)
                    sv[rb][ks] = load_chunk_a8(g.E + so + (int64_t)(row0 + row - seg0) * r + rho, min(8, r - rho), e_vec);
            }
    }
    // 3. the adapter matrix: fragments [16 columns][32 ranks], lane = (column l16, 8 ranks at 8 g4)
    uint4 fv[4][MAXKS];
    if (FWD) {
        // the work group's [32 ksteps][128] piece of B_i -> LDS (each thread 2 * MAXKS chunks), then transposing reads
        uint4 st[2 * MAXKS];
#pragma unroll
        for (int jj = 0; jj < 2 * MAXKS; ++jj) {
            const int idx = tid + NTH * jj, kr = idx / (XC / 8), c = idx % (XC / 8);
            const int col = ct * XC + c * 8;
            st[jj] = (kr < r && col < g.Ncols) ? *reinterpret_cast<const uint4*>(F + (int64_t)kr * g.Ncols + col) : zero4();
        }
#pragma unroll
        for (int jj = 0; jj < 2 * MAXKS; ++jj) {
            const int idx = tid + NTH * jj, kr = idx / (XC / 8), c = idx % (XC / 8);
            if (kr < ksteps * 32) *reinterpret_cast<uint4*>(lds + kr * BROW + ((c ^ (nn_swz(kr) << 1)) << 4)) = st[jj];
        }
        if (SLDS) {
#pragma unroll
            for (int jj = 0; jj < SCH; ++jj) {
                const int idx = tid + NTH * jj, row = idx / (MAXKS * 4), cc = idx % (MAXKS * 4);
                *reinterpret_cast<uint4*>(lds + BT_BYTES + row * ST_PITCH + cc * 16) = sst[jj];
            }
        }
        __syncthreads();
        if (SLDS) {
#pragma unroll
            for (int ks = 0; ks < MAXKS; ++ks)
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) {
                    sv[rb][ks] = zero4();
                    if (ks < ksteps)
                        sv[rb][ks] = *reinterpret_cast<const uint4*>(lds + BT_BYTES + (wr * 32 + rb * 16 + l16) * ST_PITCH + (ks * 32 + g4 * 8) * 2);
                }
        }
        const int vq = ((l16 >> 2) & 3) | ((g4 & 1) << 2);   // nn_swz of the rows this lane reads
#pragma unroll
        for (int ks = 0; ks < MAXKS; ++ks)
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) {
                fv[cb][ks] = zero4();
                if (ks < ksteps) {
                    const unsigned char* p = lds + (ks * 32 + 8 * g4 + (l16 >> 2)) * BROW + (((wc * 4 + cb) ^ vq) << 5) + (l16 & 3) * 8;
                    fv[cb][ks] = __builtin_bit_cast(uint4, lds_read_frag_tr(reinterpret_cast<const u16*>(p),
                                                                            reinterpret_cast<const u16*>(p + 4 * BROW)));
                }
            }
    } else {
        // the work group's 128 rows of A_i (one per output column; r contiguous elements each, the rows contiguous too)
        // -> LDS with a padded pitch, then plain 16-byte fragment reads.  Straight from memory every wavefront fetched
        // the fragments of its 64 columns itself: twice the bytes, in 64-byte pieces.
        constexpr int CPR = MAXKS * 4;          // 16-byte chunks per staged row
        const bool f_vec = (r & 7) == 0;
        uint4 st[2 * MAXKS];
#pragma unroll
        for (int jj = 0; jj < 2 * MAXKS; ++jj) {
            const int idx = tid + NTH * jj, c = idx / CPR, cc = idx % CPR;
            const int col = ct * XC + c;
            st[jj] = zero4();
            if (col < g.Ncols && cc * 8 < r) st[jj] = load_chunk_a8(F + (int64_t)col * r + cc * 8, min(8, r - cc * 8), f_vec);
        }
#pragma unroll
        for (int jj = 0; jj < 2 * MAXKS; ++jj) {
            const int idx = tid + NTH * jj, c = idx / CPR, cc = idx % CPR;
            if (cc < ksteps * 4) *reinterpret_cast<uint4*>(lds + c * AT_PITCH + cc * 16) = st[jj];
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < MAXKS; ++ks)
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) {
                fv[cb][ks] = zero4();
                if (ks < ksteps)
                    fv[cb][ks] = *reinterpret_cast<const uint4*>(lds + (wc * 64 + cb * 16 + l16) * AT_PITCH + (ks * 32 + g4 * 8) * 2);
            }
    }

    // accumulators start as the old tile: identity operand I_j[m][k] = (k == 16 j + m), j = column block parity
    f32x4 acc[2][4];
    {
        uint4 idn[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t one = (g4 == 2 * j + (l16 >> 3)) ? (0x3f80u << (16 * (l16 & 1))) : 0u;
            const int w = (l16 & 7) >> 1;
            idn[j] = make_uint4(w == 0 ? one : 0u, w == 1 ? one : 0u, w == 2 ? one : 0u, w == 3 ? one : 0u);
        }
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) {
                const f32x4 z = {0.f, 0.f, 0.f, 0.f};
                acc[rb][cb] = mfma16(__builtin_bit_cast(bf16x8, idn[cb & 1]), __builtin_bit_cast(bf16x8, old[rb][cb >> 1]), z);
            }
    }
#pragma unroll
    for (int ks = 0; ks < MAXKS; ++ks) {
        if (ks < ksteps) {
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                const bf16x8 a = __builtin_bit_cast(bf16x8, s != 1.0f ? scale_chunk(sv[rb][ks], s) : sv[rb][ks]);
#pragma unroll
                for (int cb = 0; cb < 4; ++cb)
                    acc[rb][cb] = mfma16(__builtin_bit_cast(bf16x8, fv[cb][ks]), a, acc[rb][cb]);   // transposed block
            }
        }
    }

    // epilogue: one rounding, transpose through this wavefront's private LDS, 128-byte row segments
    u16* Es = reinterpret_cast<u16*>(lds + BT_BYTES + ST_BYTES + wave * EP_WAVE);
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) {
            uint2 v;
            v.x = pack2hw(acc[rb][cb][0], acc[rb][cb][1]);
            v.y = pack2hw(acc[rb][cb][2], acc[rb][cb][3]);
            *reinterpret_cast<uint2*>(Es + (rb * 16 + l16) * XE_LD + cb * 16 + g4 * 4) = v;
        }
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): the same wavefront reads back what it wrote
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int rr = it * 8 + (lane >> 3), c = lane & 7;
        const int row = wr * 32 + rr, col = colw + c * 8;
        if (row >= rows || col >= g.Ncols) continue;
        const uint4 v = *reinterpret_cast<const uint4*>(Es + rr * XE_LD + c * 8);
        u16* dst = g.C + (int64_t)(row0 + row) * g.ldc + col;
        if (g.stream_out) store_streaming(dst, v);
        else *reinterpret_cast<uint4*>(dst) = v;
    }
}

// ---- host launchers ---------------------------------------------------------------------

int mfma_gemm_fwd(mlora_plan* p, const void* X, const void* W, void* Y, const void* S, uint32_t flags, hipStream_t st);
int mfma_gemm_bwd(mlora_plan* p, const void* dY, const void* W, void* dX, const void* dS, uint32_t flags, hipStream_t st);

static int launch_expand(mlora_plan* p, bool fwd, void* C, const void* E, hipStream_t st) {
    if (p->n_row_blocks == 0) return MLORA_OK;
    ExpandArgs a{};
    a.C = (u16*)C; a.E = (const u16*)E; a.pv = p->view;
    a.Ncols = (int32_t)(fwd ? p->n : p->k);
    a.ldc = a.Ncols;
    a.stream_out = 1;
    // An output that is larger than the Infinity Cache (256 MB) cannot stay there until anybody reads it again: its old
    // tile is then loaded with the non-temporal hint as well, so that it does not evict X / dY, which the next kernels
    // read (LoRA-only path of a 268 MB output: 0.48 -> 0.51 of the HBM peak).  A smaller output is loaded normally: it is
    // usually still there from whoever wrote it, and stays for whoever reads it next (134 MB output: 0.64 against 0.60).
    a.stream_in = (int64_t)p->T * a.Ncols * 2 > ((int64_t)192 << 20) ? 1 : 0;
    ProfScope prof(p, fwd ? MLORA_K_GEMM_FWD : MLORA_K_GEMM_BWD, st);
    auto go = [&](bool narrow, int32_t nblocks, const Entry4* blocks) {
        if (nblocks <= 0) return;
        a.blocks = blocks;
        const int parts = (narrow ? kBlockRows : kBlockRowsWide) / 64;     // 64-row work items per block of the class table
        const int xcw = narrow ? 4 : 2;                                    // narrow class: 256-column strips, 8 wavefronts
        a.col_tiles = (a.Ncols + 64 * xcw - 1) / (64 * xcw);
        const dim3 grid((unsigned)((int64_t)nblocks * parts * a.col_tiles)), block(128 * xcw);
        if (fwd && narrow)      hipLaunchKernelGGL((expand_add_kernel<true, 2, 4>), grid, block, 0, st, a);
        else if (fwd)           hipLaunchKernelGGL((expand_add_kernel<true, 4, 2>), grid, block, 0, st, a);
        else if (narrow)        hipLaunchKernelGGL((expand_add_kernel<false, 2, 4>), grid, block, 0, st, a);
        else                    hipLaunchKernelGGL((expand_add_kernel<false, 4, 2>), grid, block, 0, st, a);
    };
    // each rank class through the build made for it (the class table holds the wide class first)
    go(false, p->n_blocks_wide, p->view.class_blocks);
    go(true, p->n_blocks_narrow, p->view.class_blocks + p->n_blocks_wide);
    MLORA_HIP_TRY(hipGetLastError());
    return MLORA_OK;
}

int mfma_forward(mlora_plan* p, const void* X, const void* W, void* Y, void* S, uint32_t flags, hipStream_t st) {
    const bool lora = !(flags & MLORA_FLAG_BASE_ONLY) && p->N > 0;
    if (lora && p->n_row_blocks > 0) {
        ShrinkArgs a{};
        a.src = (const u16*)X; a.ld = p->k; a.out = (u16*)S; a.Kdim = (int32_t)p->k; a.pv = p->view;
        ProfScope prof(p, MLORA_K_SHRINK, st);
        launch_shrink<true>(p, a, st);
        MLORA_HIP_TRY(hipGetLastError());
    }
    if (flags & MLORA_FLAG_LORA_ONLY) return launch_expand(p, true, Y, S, st);
    return mfma_gemm_fwd(p, X, W, Y, S, flags, st);
}

int mfma_backward(mlora_plan* p, const void* dY, const void* X, const void* W, const void* S, void* dX, void* dS,
                  float* partials, uint32_t flags, hipStream_t st) {
    const bool lora = !(flags & MLORA_FLAG_BASE_ONLY) && p->N > 0;
    if (lora && p->n_row_blocks > 0) {
        ShrinkArgs a{};
        a.src = (const u16*)dY; a.ld = p->n; a.out = (u16*)dS; a.Kdim = (int32_t)p->n; a.pv = p->view;
        ProfScope prof(p, MLORA_K_DSHRINK, st);
        launch_shrink<false>(p, a, st);
        MLORA_HIP_TRY(hipGetLastError());
    }
    int rc = (flags & MLORA_FLAG_LORA_ONLY) ? launch_expand(p, false, dX, dS, st) : mfma_gemm_bwd(p, dY, W, dX, dS, flags, st);
    if (rc != MLORA_OK) return rc;
    if (lora) {
        WgradArgs w{};
        w.X = (const u16*)X; w.dY = (const u16*)dY; w.S = (const u16*)S; w.dS = (const u16*)dS;
        w.partials = partials;
        w.panels_k = (int32_t)((p->k + WP - 1) / WP);
        w.panels_n = (int32_t)((p->n + WP - 1) / WP);
        w.pv = p->view;
        w.accumulate = (flags & MLORA_FLAG_ACCUM_GRADS) ? 1 : 0;
        const DevGeo& geo = p->geo;
        if (geo.n_chunks > 0) {
            const int64_t panels = w.panels_k + w.panels_n;
            {
                // One launch per rank class over that class's part of the item table (wide class first), each through
                // the build - and so at the work groups per CU - its class allows, one after the other (overlapping them
                // on two streams was measured and is slower: the classes then share the CUs, and neither runs at its own
                // occupancy).
                ProfScope prof(p, MLORA_K_WGRAD, st);
                const int32_t n_wide = geo.n_chunks_wide, n_narrow = geo.n_chunks - geo.n_chunks_wide;
                if (n_wide > 0) {
                    w.chunk_base = 0;
                    hipLaunchKernelGGL((wgrad_kernel<4, 8>), dim3((unsigned)(n_wide * panels)), dim3(512), 0, st, w);
                }
                if (n_narrow > 0) {
                    w.chunk_base = n_wide;
                    const dim3 grid((unsigned)(n_narrow * panels));
                    if (p->max_rank_narrow <= 32) hipLaunchKernelGGL(wgrad_kernel<1>, grid, dim3(256), 0, st, w);
                    else                          hipLaunchKernelGGL(wgrad_kernel<2>, grid, dim3(256), 0, st, w);
                }
            }
            if (geo.n_reduce > 0) {
                const int64_t per = (p->k + p->n) * (int64_t)p->max_rank;
                ProfScope prof(p, MLORA_K_WGRAD_REDUCE, st);
                hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((per + 1023) / 1024), (unsigned)geo.n_reduce),
                                   dim3(256), 0, st, w, (const int32_t*)p->d_reduce_list);
            }
        }
        if (p->has_empty_ranked && !w.accumulate) {   // adapters without tokens add nothing when accumulating
            ProfScope prof(p, MLORA_K_OTHER, st);
            hipLaunchKernelGGL(wgrad_zero_empty_kernel, dim3(64, p->N), dim3(256), 0, st, p->view);
        }
        MLORA_HIP_TRY(hipGetLastError());
    }
    return MLORA_OK;
}

}  // namespace mlora

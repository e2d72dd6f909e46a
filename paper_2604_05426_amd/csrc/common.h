// Internal declarations shared by the translation units of libmultilora (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <memory>
#include <vector>

#include "multi_lora.h"

namespace mlora {

// ---- tiling constants (reported through multi_lora_plan_geometry) ------------------
constexpr int kBlockRows = 64;       // rows per LoRA block of the shrink kernels
constexpr int kBlockRowsWide = 128;  // the same for adapters of the wide rank class (their adapter tiles are the larger operand)
constexpr int kGemmBandTiles = 8;    // row tiles per band of the fused GEMM's tile order
constexpr int kGemmTileRows = 256;   // fused GEMM macro tile
constexpr int kGemmTileCols = 256;
constexpr int kWgradMinChunkRows = 512;  // smallest token chunk one weight-gradient work item reduces
constexpr int kNarrowMaxRank = 64;       // ranks above it form the wide rank class (their own kernel builds)
constexpr int kMaxSortedChunks = 16384;  // larger weight-gradient tables keep the canonical order
constexpr int kWgradPanelCols = 128;     // columns of X / dY one weight-gradient work item covers

// One entry of any plan table: 4 x int32 (meaning depends on the table).
struct Entry4 {
    int32_t a, b, c, d;
};

// Per-adapter pointers, refreshed by every fwd/bwd call (device resident).
struct AdapterPtrs {
    const void* A;
    const void* B;
    void* dA;
    void* dB;
};

// Owner of one hipMalloc'd block.
struct DeviceBlock {
    void* ptr = nullptr;
    ~DeviceBlock() {
        if (ptr) (void)hipFree(ptr);
    }
};

// Device-resident view of a plan, passed by value to kernels.
struct PlanView {
    int32_t N;
    int64_t T, k, n;
    const int32_t* off;     // [N+1] segment offsets (rows)
    const int32_t* rank;    // [N]
    const float* scale;     // [N]
    const int64_t* soff;    // [N+1] element offsets of S_i / dS_i in the ragged buffers
    const AdapterPtrs* ptrs; // [N]
    const Entry4* row_blocks;  int32_t n_row_blocks;      // canonical order (adapter, block)
    const Entry4* class_blocks; int32_t n_class_blocks;   // the same blocks, wide rank class first: what the kernels walk
    const Entry4* gemm_tiles;  int32_t n_gemm_tiles;
    const Entry4* band_order;  int32_t n_bands;           // launch order of the fused GEMM's row bands
    const Entry4* wgrad_chunks; int32_t n_wgrad_chunks;
    const int32_t* wgrad_chunk_start; // [N+1] canonical prefix: adapter i has start[i+1] - start[i] chunks
    const int64_t* part_off;   // [N] float offset of adapter i's partial weight-gradient block (adapters with > 1 chunk)
};

// What the device-side scheduler chose and counted; read back once by plan creation (sizes of the chunk table and of
// the workspace, launch grids).
struct DevGeo {
    int32_t chunk_rows, chunk_rows_wide;      // token chunk of the weight-gradient items per rank class
    int32_t n_chunks, n_chunks_wide;          // entries of the chunk table; the first n_chunks_wide are the wide class
    int32_t max_chunks_per_adapter, n_reduce; // n_reduce adapters have their tokens split over several chunks
    int64_t partial_floats;                   // fp32 partial sums those adapters need
    int64_t R1;                               // cross-checks of the sizes the host derived from the same offsets
    int32_t n_row_blocks, n_blocks_wide;
};

}  // namespace mlora

struct mlora_plan {
    int dtype = 0;
    int64_t T = 0, k = 0, n = 0;
    int32_t N = 0;
    std::vector<int32_t> ranks;
    std::vector<float> scales;
    std::vector<int64_t> off;
    std::vector<int32_t> off32;      // N+1, upload source
    int64_t R1 = 0;
    bool use_mfma = false;
    int32_t n_row_blocks = 0, n_gemm_tiles = 0, n_bands = 0;
    int32_t max_rank = 0;
    // Row blocks by rank class (<= 64 / wider): the class table puts the wide class first (its blocks run longest); plans
    // that mix narrow and wide ranks run each class through the kernel build made for it.
    int32_t n_blocks_narrow = 0, n_blocks_wide = 0;
    // Weight-gradient items: chosen, counted and ordered on the device (DevGeo).  Plans that mix ranks <= 64 and wider
    // ones launch the items of the two classes as two launches over their own parts of the table, each through the
    // kernel build - and so at the workgroups per CU - its class allows, and chunk the tokens per class.
    mlora::DevGeo geo{};
    int32_t max_rank_narrow = 0;      // largest rank <= 64 among adapters with tokens
    bool ranks_mult8 = true;          // every rank of an adapter with tokens is a multiple of 8
    // Device allocations: the plan's own blocks, and every block of other plans its view points into (a plan made by
    // multi_lora_plan_create_like uses the segmentation tables of its base in place - and through it those of the
    // base's base -, so plans may be destroyed in any order).
    std::vector<std::shared_ptr<mlora::DeviceBlock>> blocks;
    std::vector<std::shared_ptr<mlora::DeviceBlock>> shared_blocks;
    bool shares_tables = false;
    mlora::PlanView view{};
    mlora::AdapterPtrs* d_ptrs = nullptr;
    // host mirror of the device pointer table: a call whose pointers match what the same stream uploaded last skips the
    // upload.  Once an upload has been recorded into a captured graph the mirror is never trusted again: a replay
    // rewrites the table behind the host's back.
    std::vector<mlora::AdapterPtrs> ptr_mirror;
    bool ptr_mirror_valid = false;
    bool ptr_upload_captured = false;
    hipStream_t ptr_mirror_stream = nullptr;
    void* d_probs = nullptr;          // descriptor scratch of the FMA grouped GEMM
    void* d_adamw = nullptr;          // [N] optimizer entries (pointers + hyper-parameters), refreshed per call
    int32_t* d_reduce_list = nullptr; // adapters whose tokens are split over several weight-gradient chunks
    bool has_empty_ranked = false;    // some adapter has a rank but no tokens (its dA, dB are zero-filled)
    size_t ws_ds_bytes = 0;           // workspace: dS
    size_t ws_partial_bytes = 0;      // workspace: fp32 partial weight gradients
    hipStream_t build_stream = nullptr;
    int num_cus = 256;
    // per-kernel event timing (multi_lora_profile_begin / _end)
    bool prof_on = false;
    int32_t prof_used = 0;
    std::vector<int32_t> prof_kernel;
    std::vector<hipEvent_t> prof_start, prof_stop;
};

namespace mlora {

void set_error(const std::string& msg);
int hip_fail(hipError_t e, const char* what);

#define MLORA_HIP_TRY(expr)                                   \
    do {                                                      \
        hipError_t e__ = (expr);                              \
        if (e__ != hipSuccess) return ::mlora::hip_fail(e__, #expr); \
    } while (0)

// Brackets one kernel launch with events while profiling is on (no-op otherwise).
struct ProfScope {
    mlora_plan* p;
    hipStream_t st;
    int32_t idx = -1;
    ProfScope(mlora_plan* plan, int kernel, hipStream_t stream) : p(plan), st(stream) {
        if (p->prof_on && p->prof_used < (int32_t)p->prof_start.size()) {
            idx = p->prof_used++;
            p->prof_kernel[idx] = kernel;
            (void)hipEventRecord(p->prof_start[idx], st);
        }
    }
    ~ProfScope() {
        if (idx >= 0) (void)hipEventRecord(p->prof_stop[idx], st);
    }
};

// api.hip : looks up the static workspace of multi_lora_bwd_static on the current device (idempotent)
void prepare_static_workspace();

// plan.hip
int upload_ptrs(mlora_plan* p, const void* const* A, const void* const* B, void* const* dA,
                void* const* dB, hipStream_t st);

// grouped_fma.hip : descriptor-driven grouped GEMM on the vector ALUs (fp32 accumulate)
int fma_forward(mlora_plan* p, const void* X, const void* W, void* Y, void* S, uint32_t flags,
                hipStream_t st);
int fma_backward(mlora_plan* p, const void* dY, const void* X, const void* W, const void* S,
                 void* dX, void* dS, uint32_t flags, hipStream_t st);

// mfma_*.hip : bf16 MFMA kernels
int mfma_forward(mlora_plan* p, const void* X, const void* W, void* Y, void* S, uint32_t flags,
                 hipStream_t st);
int mfma_backward(mlora_plan* p, const void* dY, const void* X, const void* W, const void* S,
                  void* dX, void* dS, float* partials, uint32_t flags, hipStream_t st);

}  // namespace mlora

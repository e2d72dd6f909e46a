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
    const Entry4* row_blocks;  int32_t n_row_blocks;
    const Entry4* gemm_tiles;  int32_t n_gemm_tiles;
    const Entry4* wgrad_chunks; int32_t n_wgrad_chunks;
    const int32_t* wgrad_chunk_start; // [N+1] first chunk of each adapter
};

}  // namespace mlora

struct mlora_plan {
    int dtype = 0;
    int64_t T = 0, k = 0, n = 0;
    int32_t N = 0;
    std::vector<int32_t> ranks;
    std::vector<float> scales;
    std::vector<int64_t> off;
    std::vector<int64_t> soff;       // N+1
    std::vector<int32_t> wchunk_start; // N+1
    std::vector<int32_t> off32;      // N+1, upload source (kept alive for the async copy)
    std::vector<int64_t> part_off;   // N+1, upload source
    int64_t R1 = 0;
    bool use_mfma = false;
    int32_t n_row_blocks = 0, n_gemm_tiles = 0, n_wgrad_chunks = 0;
    int32_t max_rank = 0;
    int32_t max_chunks_per_adapter = 0;
    // row blocks split by rank class (<= 64 / wider): indices into the row-block table, wide class first (its blocks run longest).  Plans that
    // mix narrow and wide ranks run each class through the kernel build made for it.
    std::vector<int32_t> block_lists;   // upload source
    int32_t n_blocks_narrow = 0, n_blocks_wide = 0;
    int32_t* d_block_lists = nullptr;
    int32_t wgrad_chunk_rows = 0;     // token chunk of the weight-gradient items (chosen per plan)
    int32_t wgrad_chunk_rows_wide = 0;   // the same for adapters of the wide rank class (differs only when the plan mixes the classes)
    // Plans that mix ranks <= 64 and wider ones run the weight-gradient items of the two classes as two launches, each
    // through the kernel build - and so at the workgroups per CU - its class allows, and chunk the tokens per class.
    int32_t max_rank_narrow = 0;      // largest rank <= 64 among adapters with tokens
    bool ranks_mult8 = true;          // every rank of an adapter with tokens is a multiple of 8
    bool wgrad_two_classes = false;
    // one device allocation carved into the tables below; a plan made by multi_lora_plan_create_like also holds the
    // allocation of the plan whose segmentation tables it uses, so the two may be destroyed in any order
    std::shared_ptr<mlora::DeviceBlock> d_block, d_shared_block;
    size_t d_block_bytes = 0;
    bool shares_tables = false, shares_wgrad_table = false;
    mlora::PlanView view{};
    mlora::AdapterPtrs* d_ptrs = nullptr;
    // host mirror of the device pointer table: a call whose pointers match what the same stream uploaded last skips the upload
    std::vector<mlora::AdapterPtrs> ptr_mirror;
    bool ptr_mirror_valid = false;
    hipStream_t ptr_mirror_stream = nullptr;
    void* d_probs = nullptr;          // descriptor scratch of the FMA grouped GEMM
    void* d_adamw = nullptr;          // [N] optimizer entries (pointers + hyper-parameters), refreshed per call
    int64_t* d_part_off = nullptr;    // [N] float offset of each adapter's partial weight-gradient block
    std::vector<int32_t> reduce_list; // adapters whose tokens are split over several weight-gradient chunks
    int32_t* d_reduce_list = nullptr;
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

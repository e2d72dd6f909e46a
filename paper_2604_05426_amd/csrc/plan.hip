// Plan: argument validation, device-built schedule tables, per-call pointer upload.
//
// The paper builds a table of (adapter_idx, block_idx) pairs on the CPU before each
// forward pass and maps each block to a token range through per-adapter start/end
// offsets, masking the boundary block (App. A.1, "schedule-driven dispatch").  Here the
// host only validates and sizes; the tables themselves are built by device kernels from
// the offsets and ranks, once per segmentation, and shared by every layer of a step.
#include <cmath>
#include <cstring>

#include "common.h"

namespace mlora {

static thread_local std::string g_last_error;

void set_error(const std::string& msg) { g_last_error = msg; }

int hip_fail(hipError_t e, const char* what) {
    set_error(std::string("HIP error: ") + hipGetErrorString(e) + " in " + what);
    return MLORA_ERR_HIP;
}

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- device kernels -----------------------------------------------------------------

// Sequential prefix sums over the adapters (N <= 4096, done by one thread).  soff / rb_start may be NULL (not wanted).
__global__ void plan_scan_kernel(int32_t N, const int32_t* off, const int32_t* rank, int64_t* soff,
                                 int32_t* rb_start, int32_t* wc_start, int block_rows,
                                 int chunk_rows, int chunk_rows_wide) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    int64_t s = 0;
    int32_t rb = 0, wc = 0;
    for (int32_t i = 0; i < N; ++i) {
        if (soff) soff[i] = s;
        if (rb_start) rb_start[i] = rb;
        wc_start[i] = wc;
        const int32_t Ti = off[i + 1] - off[i];
        const int32_t r = rank[i];
        s += (int64_t)Ti * r;
        if (Ti > 0 && r > 0) {
            rb += (Ti + block_rows - 1) / block_rows;
            const int cr = r > kNarrowMaxRank ? chunk_rows_wide : chunk_rows;
            wc += (Ti + cr - 1) / cr;
        }
    }
    if (soff) soff[N] = s;
    if (rb_start) rb_start[N] = rb;
    wc_start[N] = wc;
}

// index of the adapter whose [start[i], start[i+1]) holds e  (start non-decreasing)
__device__ inline int32_t find_owner(const int32_t* start, int32_t N, int32_t e) {
    int32_t lo = 0, hi = N;  // invariant: start[lo] <= e < start[hi]
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if (start[mid] <= e) lo = mid; else hi = mid;
    }
    return lo;
}

// Fills a block table: entry e of adapter i = (i, b, off[i] + b*rows_per, min(rows_per, rest)).  With `rank` given,
// adapters of the wide rank class take `rows_per_wide` rows per entry instead.
__global__ void plan_fill_blocks_kernel(int32_t N, const int32_t* off, const int32_t* start,
                                        int rows_per_narrow, Entry4* out, int32_t count,
                                        const int32_t* rank, int rows_per_wide) {
    const int32_t e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= count) return;
    // adapters without entries have start[i] == start[i+1]; the owner is the last i with start[i] <= e
    // that also has start[i+1] > e, which the search below finds because start is non-decreasing.
    int32_t lo = 0, hi = N;
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if (start[mid] <= e) lo = mid; else hi = mid;
    }
    const int32_t i = lo;
    const int32_t b = e - start[i];
    const int rows_per = (rank && rank[i] > kNarrowMaxRank) ? rows_per_wide : rows_per_narrow;
    const int32_t row0 = off[i] + b * rows_per;
    const int32_t rest = off[i + 1] - row0;
    out[e] = Entry4{i, b, row0, rest < rows_per ? rest : rows_per};
}

// Device-side balancing of the weight-gradient items: entries are reordered by decreasing cost
// (tokens x (64 + rank): the stream of X / dY dominates, the MFMA work grows with the rank), ties in
// canonical order.  Workgroups are dispatched in index order, so the long items start first and the short
// ones fill the CUs as they drain (longest-processing-time-first).  Position = number of entries that
// sort before this one (counting, no atomics: the result is unique).
__global__ void plan_sort_chunks_kernel(const Entry4* in, const int32_t* rank, Entry4* out, int32_t count) {
    const int32_t e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= count) return;
    const Entry4 me = in[e];
    const int64_t key = (int64_t)me.d * (64 + rank[me.a]);
    int32_t pos = 0;
    for (int32_t o = 0; o < count; ++o) {
        const Entry4 other = in[o];
        const int64_t ok = (int64_t)other.d * (64 + rank[other.a]);
        if (ok > key || (ok == key && o < e)) ++pos;
    }
    out[pos] = me;
}

// Row tiles of the flat buffer and the adapters they touch.
__global__ void plan_fill_gemm_tiles_kernel(int32_t N, const int32_t* off, int32_t T, int tile_rows,
                                            Entry4* out, int32_t count) {
    const int32_t e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= count) return;
    const int32_t row0 = e * tile_rows;
    const int32_t rows = (T - row0) < tile_rows ? (T - row0) : tile_rows;
    int32_t lo = 0, hi = 0;
    if (N > 0) {
        lo = find_owner(off, N, row0);
        hi = find_owner(off, N, row0 + rows - 1) + 1;
    }
    out[e] = Entry4{row0, rows, lo, hi};
}

struct PtrBatch {
    AdapterPtrs p[32];
};

__global__ void upload_ptrs_kernel(AdapterPtrs* dst, PtrBatch batch, int32_t base, int32_t count) {
    const int32_t i = threadIdx.x;
    if (i < count) dst[base + i] = batch.p[i];
}

// Refreshes the device table of per-adapter pointers.  The forward passes no gradient pointers and leaves the ones in
// the table alone.  The table is left as it is when the same stream already uploaded exactly these pointers (the usual
// case: the same buffers every training step); a stream under graph capture always records the upload.
int upload_ptrs(mlora_plan* p, const void* const* A, const void* const* B, void* const* dA,
                void* const* dB, hipStream_t st) {
    if (p->N == 0) return MLORA_OK;
    const bool grads = dA != nullptr || dB != nullptr;
    if (p->ptr_mirror.size() != (size_t)p->N) {
        p->ptr_mirror.assign((size_t)p->N, AdapterPtrs{nullptr, nullptr, nullptr, nullptr});
        p->ptr_mirror_valid = false;
    }
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cap) != hipSuccess) { (void)hipGetLastError(); cap = hipStreamCaptureStatusNone; }
    const bool capturing = cap != hipStreamCaptureStatusNone;
    bool same = p->ptr_mirror_valid && p->ptr_mirror_stream == st && !capturing;
    for (int32_t i = 0; i < p->N; ++i) {
        AdapterPtrs& m = p->ptr_mirror[i];
        const void* a = A ? A[i] : nullptr;
        const void* b = B ? B[i] : nullptr;
        if (m.A != a || m.B != b) { same = false; m.A = a; m.B = b; }
        if (grads) {
            void* da = dA ? dA[i] : nullptr;
            void* db = dB ? dB[i] : nullptr;
            if (m.dA != da || m.dB != db) { same = false; m.dA = da; m.dB = db; }
        }
    }
    if (same) return MLORA_OK;
    for (int32_t base = 0; base < p->N; base += 32) {
        PtrBatch batch;
        std::memset(&batch, 0, sizeof(batch));
        const int32_t cnt = (p->N - base) < 32 ? (p->N - base) : 32;
        for (int32_t j = 0; j < cnt; ++j) batch.p[j] = p->ptr_mirror[base + j];
        ProfScope prof(p, MLORA_K_OTHER, st);
        hipLaunchKernelGGL(upload_ptrs_kernel, dim3(1), dim3(32), 0, st, p->d_ptrs, batch, base, cnt);
    }
    MLORA_HIP_TRY(hipGetLastError());
    p->ptr_mirror_valid = !capturing;
    p->ptr_mirror_stream = st;
    return MLORA_OK;
}

}  // namespace mlora

using namespace mlora;

// ---- C ABI -----------------------------------------------------------------------------

extern "C" const char* multi_lora_last_error(void) { return g_last_error.c_str(); }

extern "C" const char* multi_lora_version(void) { return "0.1"; }

extern "C" int multi_lora_validate(int dtype, int64_t T, int64_t k, int64_t n, int32_t N,
                                   const int32_t* ranks, const float* scales,
                                   const int64_t* seg_offsets) {
    if (dtype != MLORA_F32 && dtype != MLORA_BF16) {
        set_error("dtype must be MLORA_F32 or MLORA_BF16");
        return MLORA_ERR_DTYPE;
    }
    const int64_t kMaxDim = (int64_t)1 << 30;
    if (T < 0 || T > kMaxDim || k < 1 || k > kMaxDim || n < 1 || n > kMaxDim) {
        set_error("T must be in [0, 2^30] and k, n in [1, 2^30]");
        return MLORA_ERR_SHAPE;
    }
    if (N < 0 || N > MLORA_MAX_ADAPTERS) {
        set_error("N must be in [0, MLORA_MAX_ADAPTERS]");
        return MLORA_ERR_SHAPE;
    }
    if (N == 0) return MLORA_OK;   // no adapters: every row is a plain X W row; the metadata arrays are not read
    if (!seg_offsets) {
        set_error("seg_offsets is NULL");
        return MLORA_ERR_NULL;
    }
    if (!ranks || !scales) {
        set_error("ranks / scales is NULL");
        return MLORA_ERR_NULL;
    }
    if (seg_offsets[0] != 0) {
        set_error("seg_offsets[0] must be 0");
        return MLORA_ERR_SEGMENTS;
    }
    for (int32_t i = 0; i < N; ++i) {
        if (seg_offsets[i + 1] < seg_offsets[i]) {
            set_error("seg_offsets must be non-decreasing (segments may not overlap)");
            return MLORA_ERR_SEGMENTS;
        }
    }
    if (seg_offsets[N] != T) {
        set_error("seg_offsets[N] must equal T (every row belongs to exactly one adapter)");
        return MLORA_ERR_SEGMENTS;
    }
    for (int32_t i = 0; i < N; ++i) {
        if (ranks[i] < 0 || ranks[i] > MLORA_MAX_RANK) {
            set_error("rank outside [0, MLORA_MAX_RANK]");
            return MLORA_ERR_RANK;
        }
        if (!std::isfinite(scales[i])) {
            set_error("scale is not finite");
            return MLORA_ERR_SCALE;
        }
    }
    return MLORA_OK;
}

// `like`: a plan over the same segmentation (same T, N, ranks, scales, offsets) whose device tables the new plan
// uses instead of building its own; only what depends on the layer shape or on the caller's buffers is new.
static int plan_create_impl(mlora_plan** out, int dtype, int64_t T, int64_t k, int64_t n,
                            int32_t N, const int32_t* ranks, const float* scales,
                            const int64_t* seg_offsets, void* stream, const mlora_plan* like) {
    if (!out) {
        set_error("out is NULL");
        return MLORA_ERR_NULL;
    }
    *out = nullptr;
    const int rc = multi_lora_validate(dtype, T, k, n, N, ranks, scales, seg_offsets);
    if (rc != MLORA_OK) return rc;

    mlora_plan* p = new mlora_plan();
    p->dtype = dtype;
    p->T = T; p->k = k; p->n = n; p->N = N;
    if (N > 0) {
        p->ranks.assign(ranks, ranks + N);
        p->scales.assign(scales, scales + N);
        p->off.assign(seg_offsets, seg_offsets + N + 1);
    } else {
        p->off.assign(1, 0);
    }
    p->soff.resize(N + 1);
    p->wchunk_start.resize(N + 1);
    p->build_stream = (hipStream_t)stream;
    // bf16 with 16-byte row granularity goes to the MFMA kernels, everything else to the FMA kernels
    p->use_mfma = (dtype == MLORA_BF16) && (k % 8 == 0) && (n % 8 == 0);

    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            p->num_cus = cus;
    }
    // Weight-gradient work items are (token chunk, 128-column panel).  Balance heterogeneous segment
    // lengths across the CUs: keep whole segments when that already yields two items per CU (no
    // partial sums at all), otherwise halve the chunk until it does or the minimum is reached.
    // A plan that mixes the two rank classes launches them as two kernels that overlap; the rule then holds for
    // each launch by itself (a few long wide-rank segments would otherwise run on after everything else has ended).
    {
        bool wide = false, narrow = false;
        for (int32_t i = 0; i < N; ++i) {
            if (seg_offsets[i + 1] == seg_offsets[i] || ranks[i] == 0) continue;
            (ranks[i] > kNarrowMaxRank ? wide : narrow) = true;
        }
        const bool two = wide && narrow;
        const int64_t panels = ceil_div(k, kWgradPanelCols) + ceil_div(n, kWgradPanelCols);
        auto choose = [&](int cls) {      // 0: every adapter, 1: narrow ranks only, 2: wide ranks only
            int64_t chunk = (int64_t)1 << 30;
            for (;;) {
                int64_t items = 0;
                for (int32_t i = 0; i < N; ++i) {
                    const int64_t Ti = seg_offsets[i + 1] - seg_offsets[i];
                    if (Ti <= 0 || ranks[i] <= 0) continue;
                    if ((cls == 1 && ranks[i] > kNarrowMaxRank) || (cls == 2 && ranks[i] <= kNarrowMaxRank)) continue;
                    items += ceil_div(Ti, chunk) * panels;
                }
                if (items >= 2 * (int64_t)p->num_cus || chunk <= kWgradMinChunkRows) break;
                chunk /= 2;
            }
            return (int32_t)chunk;
        };
        p->wgrad_chunk_rows = choose(two ? 1 : 0);
        p->wgrad_chunk_rows_wide = two ? choose(2) : p->wgrad_chunk_rows;
    }
    p->shares_tables = like != nullptr;
    // the weight-gradient item table depends on the layer shape only through the token chunk
    p->shares_wgrad_table = like != nullptr && like->wgrad_chunk_rows == p->wgrad_chunk_rows &&
                            like->wgrad_chunk_rows_wide == p->wgrad_chunk_rows_wide;

    // host-side sizes (the device rebuilds the same numbers; multi_lora_plan_dump exposes them)
    int64_t s = 0;
    int64_t rb = 0, wc = 0;
    for (int32_t i = 0; i < N; ++i) {
        p->soff[i] = s;
        p->wchunk_start[i] = (int32_t)wc;
        const int64_t Ti = p->off[i + 1] - p->off[i];
        s += Ti * ranks[i];
        if (Ti > 0 && ranks[i] > 0) {
            rb += ceil_div(Ti, kBlockRows);
            const int64_t c = ceil_div(Ti, ranks[i] > kNarrowMaxRank ? p->wgrad_chunk_rows_wide : p->wgrad_chunk_rows);
            wc += c;
            if (c > p->max_chunks_per_adapter) p->max_chunks_per_adapter = (int32_t)c;
        }
        if (ranks[i] > p->max_rank) p->max_rank = ranks[i];
    }
    {
        bool wide = false;
        for (int32_t i = 0; i < N; ++i) {
            if (p->off[i + 1] == p->off[i] || ranks[i] == 0) continue;
            if (ranks[i] % 8) p->ranks_mult8 = false;
            if (ranks[i] > 64) wide = true;
            else if (ranks[i] > p->max_rank_narrow) p->max_rank_narrow = ranks[i];
        }
        p->wgrad_two_classes = wide && p->max_rank_narrow > 0;
    }
    {   // same enumeration as the device-built row-block table: adapters ascending, blocks ascending
        std::vector<int32_t> narrow;
        int32_t idx = 0;
        for (int32_t i = 0; i < N; ++i) {
            const int64_t Ti = p->off[i + 1] - p->off[i];
            if (Ti <= 0 || ranks[i] <= 0) continue;
            const int32_t nb = (int32_t)ceil_div(Ti, kBlockRows);
            for (int32_t b = 0; b < nb; ++b, ++idx) (ranks[i] <= 64 ? narrow : p->block_lists).push_back(idx);
        }
        p->n_blocks_wide = (int32_t)p->block_lists.size();
        p->n_blocks_narrow = (int32_t)narrow.size();
        p->block_lists.insert(p->block_lists.end(), narrow.begin(), narrow.end());
    }
    p->soff[N] = s;
    p->wchunk_start[N] = (int32_t)wc;
    p->R1 = s;
    p->n_row_blocks = (int32_t)rb;
    p->n_wgrad_chunks = (int32_t)wc;
    p->n_gemm_tiles = (int32_t)ceil_div(T, kGemmTileRows);

    const size_t esz = dtype == MLORA_BF16 ? 2 : 4;
    auto up256 = [](size_t v) { return (v + 255) & ~(size_t)255; };
    p->ws_ds_bytes = up256((size_t)p->R1 * esz);
    // fp32 partials of dA_i, dB_i for adapters whose tokens are split over several chunks
    size_t part = 0;   // in floats
    std::vector<int64_t>& part_off = p->part_off;
    part_off.assign(N + 1, 0);
    for (int32_t i = 0; i < N; ++i) {
        const int64_t c = p->wchunk_start[i + 1] - p->wchunk_start[i];
        part_off[i] = (int64_t)part;
        if (c > 1) {
            part += (size_t)c * (size_t)(k + n) * (size_t)ranks[i];
            p->reduce_list.push_back(i);
        }
        if (ranks[i] > 0 && p->off[i + 1] == p->off[i]) p->has_empty_ranked = true;
    }
    p->ws_partial_bytes = up256(part * sizeof(float));

    // carve one device allocation
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t r = o; o += up256(bytes); return r; };
    const bool own_seg = !p->shares_tables, own_wc = !p->shares_wgrad_table;
    const size_t o_off = take(own_seg ? sizeof(int32_t) * (N + 1) : 0);
    const size_t o_rank = take(own_seg ? sizeof(int32_t) * (N + 1) : 0);
    const size_t o_scale = take(own_seg ? sizeof(float) * (N + 1) : 0);
    const size_t o_soff = take(own_seg ? sizeof(int64_t) * (N + 1) : 0);
    const size_t o_rbs = take(own_seg ? sizeof(int32_t) * (N + 1) : 0);
    const size_t o_wcs = take(own_wc ? sizeof(int32_t) * (N + 1) : 0);
    const size_t o_ptrs = take(sizeof(AdapterPtrs) * (N + 1));
    const size_t o_rb = take(own_seg ? sizeof(Entry4) * (size_t)(p->n_row_blocks + 1) : 0);
    const size_t o_gt = take(own_seg ? sizeof(Entry4) * (size_t)(p->n_gemm_tiles + 1) : 0);
    const size_t o_wc = take(own_wc ? sizeof(Entry4) * (size_t)(p->n_wgrad_chunks + 1) : 0);
    const size_t o_wc_tmp = take(own_wc ? sizeof(Entry4) * (size_t)(p->n_wgrad_chunks + 1) : 0);
    const size_t o_probs = take(128 * (size_t)(5 * N + 8));
    const size_t o_part = take(sizeof(int64_t) * (N + 1) + sizeof(int32_t) * (N + 1));   // partial offsets, then the reduce list
    const size_t o_adamw = take(96 * (size_t)(N + 1));
    const size_t o_lists = take(own_seg ? sizeof(int32_t) * (size_t)(p->n_row_blocks + 1) : 0);
    p->d_block_bytes = o;

    p->d_block = std::make_shared<DeviceBlock>();
    if (e == hipSuccess) e = hipMalloc(&p->d_block->ptr, p->d_block_bytes);
    if (e != hipSuccess) {
        delete p;
        return hip_fail(e, "hipMalloc(plan tables)");
    }
    if (like) p->d_shared_block = like->d_block;      // keeps the shared tables alive
    char* base = (char*)p->d_block->ptr;
    const PlanView* lv = like ? &like->view : nullptr;
    int32_t* d_off = own_seg ? (int32_t*)(base + o_off) : const_cast<int32_t*>(lv->off);
    int32_t* d_rank = own_seg ? (int32_t*)(base + o_rank) : const_cast<int32_t*>(lv->rank);
    float* d_scale = own_seg ? (float*)(base + o_scale) : const_cast<float*>(lv->scale);
    int64_t* d_soff = own_seg ? (int64_t*)(base + o_soff) : const_cast<int64_t*>(lv->soff);
    int32_t* d_rbs = own_seg ? (int32_t*)(base + o_rbs) : nullptr;
    int32_t* d_wcs = own_wc ? (int32_t*)(base + o_wcs) : const_cast<int32_t*>(lv->wgrad_chunk_start);
    p->d_ptrs = (AdapterPtrs*)(base + o_ptrs);
    Entry4* d_rb = own_seg ? (Entry4*)(base + o_rb) : const_cast<Entry4*>(lv->row_blocks);
    Entry4* d_gt = own_seg ? (Entry4*)(base + o_gt) : const_cast<Entry4*>(lv->gemm_tiles);
    Entry4* d_wc = own_wc ? (Entry4*)(base + o_wc) : const_cast<Entry4*>(lv->wgrad_chunks);
    p->d_probs = base + o_probs;
    p->d_part_off = (int64_t*)(base + o_part);
    p->d_reduce_list = (int32_t*)(base + o_part + sizeof(int64_t) * (N + 1));
    p->d_adamw = base + o_adamw;
    p->d_block_lists = own_seg ? (int32_t*)(base + o_lists) : like->d_block_lists;

    hipStream_t st = p->build_stream;
    std::vector<int32_t>& off32 = p->off32;
    off32.resize(N + 1);
    for (int32_t i = 0; i <= N; ++i) off32[i] = (int32_t)p->off[i];
    auto fail = [&](hipError_t err, const char* what) {
        delete p;
        return hip_fail(err, what);
    };
    if (own_seg && (e = hipMemcpyAsync(d_off, off32.data(), sizeof(int32_t) * (N + 1), hipMemcpyHostToDevice, st)) != hipSuccess)
        return fail(e, "hipMemcpyAsync(offsets)");
    if (own_seg && N > 0) {
        if ((e = hipMemcpyAsync(d_rank, p->ranks.data(), sizeof(int32_t) * N, hipMemcpyHostToDevice, st)) != hipSuccess)
            return fail(e, "hipMemcpyAsync(ranks)");
        if ((e = hipMemcpyAsync(d_scale, p->scales.data(), sizeof(float) * N, hipMemcpyHostToDevice, st)) != hipSuccess)
            return fail(e, "hipMemcpyAsync(scales)");
    }
    if ((e = hipMemcpyAsync(p->d_part_off, part_off.data(), sizeof(int64_t) * (N + 1), hipMemcpyHostToDevice, st)) != hipSuccess)
        return fail(e, "hipMemcpyAsync(partial offsets)");
    if (!p->reduce_list.empty() &&
        (e = hipMemcpyAsync(p->d_reduce_list, p->reduce_list.data(), sizeof(int32_t) * p->reduce_list.size(),
                            hipMemcpyHostToDevice, st)) != hipSuccess)
        return fail(e, "hipMemcpyAsync(reduce list)");
    if (own_seg && !p->block_lists.empty() &&
        (e = hipMemcpyAsync(p->d_block_lists, p->block_lists.data(), sizeof(int32_t) * p->block_lists.size(),
                            hipMemcpyHostToDevice, st)) != hipSuccess)
        return fail(e, "hipMemcpyAsync(row-block classes)");
    // (a plan that shares the segmentation tables but chunks the tokens differently scans again for its chunk starts)
    if (own_seg)
        hipLaunchKernelGGL(plan_scan_kernel, dim3(1), dim3(64), 0, st, N, d_off, d_rank, d_soff, d_rbs, d_wcs,
                           kBlockRows, p->wgrad_chunk_rows, p->wgrad_chunk_rows_wide);
    else if (own_wc)
        hipLaunchKernelGGL(plan_scan_kernel, dim3(1), dim3(64), 0, st, N, d_off, d_rank, (int64_t*)nullptr,
                           (int32_t*)nullptr, d_wcs, kBlockRows, p->wgrad_chunk_rows, p->wgrad_chunk_rows_wide);
    if (own_seg && p->n_row_blocks > 0)
        hipLaunchKernelGGL(plan_fill_blocks_kernel, dim3((p->n_row_blocks + 255) / 256), dim3(256), 0, st, N,
                           d_off, d_rbs, kBlockRows, d_rb, p->n_row_blocks, (const int32_t*)nullptr, 0);
    if (own_wc && p->n_wgrad_chunks > 0) {
        Entry4* d_wc_tmp = (Entry4*)(base + o_wc_tmp);
        const unsigned blocks = (unsigned)((p->n_wgrad_chunks + 255) / 256);
        if (p->n_wgrad_chunks <= kMaxSortedChunks) {   // canonical table, then reordered by cost
            hipLaunchKernelGGL(plan_fill_blocks_kernel, dim3(blocks), dim3(256), 0, st, N, d_off, d_wcs,
                               p->wgrad_chunk_rows, d_wc_tmp, p->n_wgrad_chunks, (const int32_t*)d_rank,
                               p->wgrad_chunk_rows_wide);
            hipLaunchKernelGGL(plan_sort_chunks_kernel, dim3(blocks), dim3(256), 0, st, d_wc_tmp, d_rank, d_wc,
                               p->n_wgrad_chunks);
        } else {
            hipLaunchKernelGGL(plan_fill_blocks_kernel, dim3(blocks), dim3(256), 0, st, N, d_off, d_wcs,
                               p->wgrad_chunk_rows, d_wc, p->n_wgrad_chunks, (const int32_t*)d_rank,
                               p->wgrad_chunk_rows_wide);
        }
    }
    if (own_seg && p->n_gemm_tiles > 0)
        hipLaunchKernelGGL(plan_fill_gemm_tiles_kernel, dim3((p->n_gemm_tiles + 255) / 256), dim3(256), 0, st, N,
                           d_off, (int32_t)T, kGemmTileRows, d_gt, p->n_gemm_tiles);
    if ((e = hipGetLastError()) != hipSuccess) return fail(e, "plan build kernels");
    prepare_static_workspace();

    PlanView& v = p->view;
    v.N = N; v.T = T; v.k = k; v.n = n;
    v.off = d_off; v.rank = d_rank; v.scale = d_scale; v.soff = d_soff; v.ptrs = p->d_ptrs;
    v.row_blocks = d_rb; v.n_row_blocks = p->n_row_blocks;
    v.gemm_tiles = d_gt; v.n_gemm_tiles = p->n_gemm_tiles;
    v.wgrad_chunks = d_wc; v.n_wgrad_chunks = p->n_wgrad_chunks;
    v.wgrad_chunk_start = d_wcs;
    *out = p;
    return MLORA_OK;
}

extern "C" int multi_lora_plan_create(mlora_plan** out, int dtype, int64_t T, int64_t k, int64_t n,
                                      int32_t N, const int32_t* ranks, const float* scales,
                                      const int64_t* seg_offsets, void* stream) {
    return plan_create_impl(out, dtype, T, k, n, N, ranks, scales, seg_offsets, stream, nullptr);
}

extern "C" int multi_lora_plan_create_like(mlora_plan** out, const mlora_plan* base, int64_t k, int64_t n,
                                           void* stream) {
    if (!out) {
        set_error("out is NULL");
        return MLORA_ERR_NULL;
    }
    *out = nullptr;
    if (!base) {
        set_error("base plan is NULL");
        return MLORA_ERR_NULL;
    }
    // the tables of `base` are built on its own stream: a different stream must see them finished
    if ((hipStream_t)stream != base->build_stream) {
        set_error("multi_lora_plan_create_like: pass the stream the base plan was created on");
        return MLORA_ERR_SHAPE;
    }
    return plan_create_impl(out, base->dtype, base->T, k, n, base->N, base->ranks.data(), base->scales.data(),
                            base->off.data(), stream, base);
}

static void free_events(mlora_plan* plan) {
    for (hipEvent_t ev : plan->prof_start) (void)hipEventDestroy(ev);
    for (hipEvent_t ev : plan->prof_stop) (void)hipEventDestroy(ev);
    plan->prof_start.clear();
    plan->prof_stop.clear();
    plan->prof_kernel.clear();
    plan->prof_used = 0;
    plan->prof_on = false;
}

extern "C" int multi_lora_profile_begin(mlora_plan* plan, int32_t max_records) {
    if (!plan) {
        set_error("plan is NULL");
        return MLORA_ERR_NULL;
    }
    if (max_records < 1 || max_records > (1 << 20)) {
        set_error("max_records must be in [1, 2^20]");
        return MLORA_ERR_SHAPE;
    }
    free_events(plan);
    plan->prof_start.resize(max_records);
    plan->prof_stop.resize(max_records);
    plan->prof_kernel.assign(max_records, MLORA_K_OTHER);
    for (int32_t i = 0; i < max_records; ++i) {
        hipError_t e = hipEventCreate(&plan->prof_start[i]);
        if (e == hipSuccess) e = hipEventCreate(&plan->prof_stop[i]);
        if (e != hipSuccess) {
            plan->prof_start.resize(i);
            plan->prof_stop.resize(i);
            free_events(plan);
            return hip_fail(e, "hipEventCreate");
        }
    }
    plan->prof_on = true;
    return MLORA_OK;
}

extern "C" int multi_lora_profile_end(mlora_plan* plan, int32_t* kernel_ids, float* ms, int32_t cap,
                                      int32_t* count) {
    if (!plan || !count) {
        set_error("plan / count is NULL");
        return MLORA_ERR_NULL;
    }
    plan->prof_on = false;
    const int32_t used = plan->prof_used;
    *count = used;
    int rc = MLORA_OK;
    for (int32_t i = 0; i < used && i < cap; ++i) {
        if (!kernel_ids || !ms) {
            set_error("kernel_ids / ms is NULL");
            rc = MLORA_ERR_NULL;
            break;
        }
        hipError_t e = hipEventSynchronize(plan->prof_stop[i]);
        float t = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&t, plan->prof_start[i], plan->prof_stop[i]);
        if (e != hipSuccess) {
            rc = hip_fail(e, "hipEventElapsedTime");
            break;
        }
        kernel_ids[i] = plan->prof_kernel[i];
        ms[i] = t;
    }
    free_events(plan);
    return rc;
}

extern "C" int multi_lora_plan_destroy(mlora_plan* plan) {
    if (!plan) return MLORA_OK;
    free_events(plan);
    delete plan;      // frees the device block unless another plan still shares it
    return MLORA_OK;
}

extern "C" size_t multi_lora_workspace_bytes(const mlora_plan* plan) {
    if (!plan) return 0;
    return plan->ws_ds_bytes + plan->ws_partial_bytes;
}

extern "C" int multi_lora_plan_geometry(const mlora_plan* plan, int32_t* out) {
    if (!plan || !out) {
        set_error("plan / out is NULL");
        return MLORA_ERR_NULL;
    }
    for (int i = 0; i < MLORA_GEO_COUNT; ++i) out[i] = 0;
    out[MLORA_GEO_BLOCK_ROWS] = kBlockRows;
    out[MLORA_GEO_GEMM_TILE_ROWS] = kGemmTileRows;
    out[MLORA_GEO_GEMM_TILE_COLS] = kGemmTileCols;
    out[MLORA_GEO_WGRAD_CHUNK_ROWS] = plan->wgrad_chunk_rows;
    out[MLORA_GEO_WGRAD_CHUNK_ROWS_WIDE] = plan->wgrad_chunk_rows_wide;
    out[MLORA_GEO_R1_LO] = (int32_t)(plan->R1 & 0x7fffffff);
    out[MLORA_GEO_R1_HI] = (int32_t)(plan->R1 >> 31);
    out[MLORA_GEO_USES_MFMA] = plan->use_mfma ? 1 : 0;
    return MLORA_OK;
}

extern "C" int multi_lora_plan_dump(const mlora_plan* plan, int which, int32_t* entries, int64_t cap,
                                    int64_t* count) {
    if (!plan || !count) {
        set_error("plan / count is NULL");
        return MLORA_ERR_NULL;
    }
    const Entry4* src = nullptr;
    int64_t cnt = 0;
    switch (which) {
        case MLORA_TABLE_ROW_BLOCKS: src = plan->view.row_blocks; cnt = plan->n_row_blocks; break;
        case MLORA_TABLE_GEMM_ROW_TILES: src = plan->view.gemm_tiles; cnt = plan->n_gemm_tiles; break;
        case MLORA_TABLE_WGRAD_CHUNKS: src = plan->view.wgrad_chunks; cnt = plan->n_wgrad_chunks; break;
        default:
            set_error("unknown table id");
            return MLORA_ERR_FLAGS;
    }
    *count = cnt;
    const int64_t ncopy = cnt < cap ? cnt : cap;
    if (ncopy > 0) {
        if (!entries) {
            set_error("entries is NULL");
            return MLORA_ERR_NULL;
        }
        MLORA_HIP_TRY(hipStreamSynchronize(plan->build_stream));
        MLORA_HIP_TRY(hipMemcpy(entries, src, sizeof(Entry4) * (size_t)ncopy, hipMemcpyDeviceToHost));
    }
    return MLORA_OK;
}

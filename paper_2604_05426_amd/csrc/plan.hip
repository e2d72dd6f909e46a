// Plan: argument validation, device-built schedule tables, per-call pointer upload.
//
// The paper builds a table of (adapter_idx, block_idx) pairs on the CPU before each
// forward pass and maps each block to a token range through per-adapter start/end
// offsets, masking the boundary block (App. A.1, "schedule-driven dispatch").  Here the
// host only validates and sizes; the tables themselves are built by device kernels from
// the offsets and ranks, once per segmentation, and shared by every layer of a step.
#include <cmath>
#include <cstring>
#include <mutex>

#include "common.h"

namespace mlora {

static thread_local std::string g_last_error;

void set_error(const std::string& msg) { g_last_error = msg; }

int hip_fail(hipError_t e, const char* what) {
    set_error(std::string("HIP error: ") + hipGetErrorString(e) + " in " + what);
    return MLORA_ERR_HIP;
}

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- device kernels: the segment / tile scheduler ------------------------------------------------

// Scheduler set-up, one workgroup.  From the offsets and ranks alone it
//  (1) chooses the token chunk of the weight-gradient items, per rank class.  Work items are (token chunk, 128-column
//      panel); heterogeneous segment lengths are balanced across the CUs by keeping whole segments when that already
//      yields two items per CU (no partial sums at all) and otherwise halving the chunk until it does or the minimum is
//      reached.  A plan that mixes the two rank classes launches them as two kernels; the rule then holds for each
//      launch by itself (a few long wide-rank segments would otherwise run on after everything else has ended);
//  (2) scans the adapters: ragged S offsets, first row block / class block / chunk of each adapter and where its
//      entries go in the class-ordered tables (wide class first), offsets of the fp32 partial sums, the list of
//      adapters that need the fixed-order sum of partials;
//  (3) leaves the counts in *geo for the host to size the chunk table, the workspace and the launch grids.
// soff, rb_start, cb_start, cb_pos may be NULL (a plan over an existing segmentation only needs the chunk side).
constexpr int kScanThreads = 256;

__global__ __launch_bounds__(kScanThreads) void plan_scan_kernel(
        int32_t N, const int32_t* off, const int32_t* rank, int64_t panels, int64_t kn, int32_t num_cus,
        int block_rows, int block_rows_wide, int min_chunk,
        int64_t* soff, int32_t* rb_start, int32_t* cb_start, int32_t* cb_pos,
        int32_t* wc_start, int32_t* wc_pos, int64_t* part_off, int32_t* reduce_list, DevGeo* geo) {
    __shared__ int64_t red[kScanThreads];
    const int tid = threadIdx.x;
    // items of one launch if the tokens of class `cls` (0: every adapter, 1: narrow ranks, 2: wide ranks) are cut every `chunk`
    auto count_items = [&](int64_t chunk, int cls) -> int64_t {
        int64_t mine = 0;
        for (int32_t i = tid; i < N; i += kScanThreads) {
            const int64_t Ti = off[i + 1] - off[i];
            const int32_t r = rank[i];
            if (Ti <= 0 || r <= 0) continue;
            if ((cls == 1 && r > kNarrowMaxRank) || (cls == 2 && r <= kNarrowMaxRank)) continue;
            mine += (Ti + chunk - 1) / chunk;
        }
        red[tid] = mine;
        __syncthreads();
        for (int s = kScanThreads / 2; s > 0; s >>= 1) {
            if (tid < s) red[tid] += red[tid + s];
            __syncthreads();
        }
        const int64_t total = red[0];
        __syncthreads();
        return total * panels;
    };
    auto choose = [&](int cls) -> int32_t {
        int64_t chunk = (int64_t)1 << 30;
        for (;;) {
            const int64_t items = count_items(chunk, cls);       // uniform over the workgroup
            if (items >= 2 * (int64_t)num_cus || chunk <= min_chunk) break;
            chunk >>= 1;
        }
        return (int32_t)chunk;
    };
    const bool two = count_items((int64_t)1 << 30, 1) > 0 && count_items((int64_t)1 << 30, 2) > 0;
    const int32_t cn = choose(two ? 1 : 0);
    const int32_t cw = two ? choose(2) : cn;
    if (tid != 0) return;

    // class totals first: the wide class comes first in the class-ordered tables
    int32_t wide_blocks = 0, wide_chunks = 0;
    for (int32_t i = 0; i < N; ++i) {
        const int32_t Ti = off[i + 1] - off[i], r = rank[i];
        if (Ti > 0 && r > kNarrowMaxRank) {
            wide_blocks += (Ti + block_rows_wide - 1) / block_rows_wide;
            wide_chunks += (Ti + cw - 1) / cw;
        }
    }
    int64_t s = 0, part = 0;
    int32_t rb = 0, cb = 0, wc = 0, max_c = 0, n_reduce = 0;
    int32_t cb_wide = 0, cb_narrow = wide_blocks, wc_wide = 0, wc_narrow = wide_chunks;
    for (int32_t i = 0; i < N; ++i) {
        const int32_t Ti = off[i + 1] - off[i], r = rank[i];
        const bool wide = r > kNarrowMaxRank;
        if (soff) soff[i] = s;
        if (rb_start) rb_start[i] = rb;
        if (cb_start) { cb_start[i] = cb; cb_pos[i] = wide ? cb_wide : cb_narrow; }
        wc_start[i] = wc;
        wc_pos[i] = wide ? wc_wide : wc_narrow;
        part_off[i] = part;
        s += (int64_t)Ti * r;
        if (Ti > 0 && r > 0) {
            rb += (Ti + block_rows - 1) / block_rows;
            const int br = wide ? block_rows_wide : block_rows;
            const int32_t nb = (Ti + br - 1) / br;
            cb += nb;
            (wide ? cb_wide : cb_narrow) += nb;
            const int cr = wide ? cw : cn;
            const int32_t c = (Ti + cr - 1) / cr;
            wc += c;
            (wide ? wc_wide : wc_narrow) += c;
            if (c > max_c) max_c = c;
            if (c > 1) {
                part += (int64_t)c * kn * r;
                reduce_list[n_reduce++] = i;
            }
        }
    }
    if (soff) soff[N] = s;
    if (rb_start) rb_start[N] = rb;
    if (cb_start) cb_start[N] = cb;
    wc_start[N] = wc;
    DevGeo gg;
    gg.chunk_rows = cn; gg.chunk_rows_wide = cw;
    gg.n_chunks = wc; gg.n_chunks_wide = wide_chunks;
    gg.max_chunks_per_adapter = max_c; gg.n_reduce = n_reduce;
    gg.partial_floats = part;
    gg.R1 = s; gg.n_row_blocks = rb; gg.n_blocks_wide = wide_blocks;
    *geo = gg;
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

// Fills a block table.  Canonical entry e (adapters ascending, blocks ascending; `start` is its prefix over the
// adapters) belongs to adapter i = owner(e) and is block b = e - start[i]: (i, b, off[i] + b*rows_per, min(rows_per,
// rest)), written to out[pos[i] + b].  pos == start gives the canonical table, pos = the class-ordered positions the
// table with the wide rank class first.  Adapters of the wide class take `rows_per_wide` rows per entry.
// (Adapters without entries have start[i] == start[i+1]; the owner is the last i with start[i] <= e.)
__global__ void plan_fill_blocks_kernel(int32_t N, const int32_t* off, const int32_t* rank, const int32_t* start,
                                        const int32_t* pos, int rows_per_narrow, int rows_per_wide, Entry4* out,
                                        int32_t count) {
    const int32_t e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= count) return;
    const int32_t i = find_owner(start, N, e);
    const int32_t b = e - start[i];
    const int rows_per = rank[i] > kNarrowMaxRank ? rows_per_wide : rows_per_narrow;
    const int32_t row0 = off[i] + b * rows_per;
    const int32_t rest = off[i + 1] - row0;
    out[pos[i] + b] = Entry4{i, b, row0, rest < rows_per ? rest : rows_per};
}

// Device-side balancing of the weight-gradient items: inside its rank class (entries [0, n_wide) are the wide class,
// the rest the narrow one) every entry moves to the position given by decreasing cost (tokens x (64 + rank): the
// stream of X / dY dominates, the MFMA work grows with the rank), ties in the order of the input table.  Workgroups
// are dispatched in index order, so the long items start first and the short ones fill the CUs as they drain
// (longest-processing-time-first).  Position = number of entries of the class that sort before this one (counting, no
// atomics: the result is unique).
__global__ void plan_sort_chunks_kernel(const Entry4* in, const int32_t* rank, Entry4* out, int32_t count, int32_t n_wide) {
    const int32_t e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= count) return;
    const Entry4 me = in[e];
    const int64_t key = (int64_t)me.d * (64 + rank[me.a]);
    const int32_t lo = e < n_wide ? 0 : n_wide, hi = e < n_wide ? n_wide : count;
    int32_t pos = lo;
    for (int32_t o = lo; o < hi; ++o) {
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

// Bands of the fused GEMM (kGemmBandTiles consecutive row tiles x all column tiles are worked on by the whole chip at a
// time).  Cost of a band = rank-extension passes its row tiles run per column tile: for every row tile, one pass per
// 64 ranks of every adapter that owns rows of it.  Entry: (band, first row tile, row tiles, cost).
__global__ void plan_band_cost_kernel(int32_t N, const int32_t* off, const int32_t* rank, const Entry4* tiles,
                                      int32_t n_tiles, int band_tiles, Entry4* out, int32_t n_bands) {
    const int32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= n_bands) return;
    const int32_t t0 = b * band_tiles;
    const int32_t nt = (n_tiles - t0) < band_tiles ? (n_tiles - t0) : band_tiles;
    int32_t cost = 0;
    for (int32_t t = t0; t < t0 + nt; ++t) {
        const Entry4 tile = tiles[t];
        for (int32_t i = tile.c; i < tile.d; ++i) {
            const int32_t lo = off[i] > tile.a ? off[i] : tile.a;
            const int32_t hi = off[i + 1] < tile.a + tile.b ? off[i + 1] : tile.a + tile.b;
            if (lo < hi && rank[i] > 0) cost += (rank[i] + 63) / 64;
        }
    }
    out[b] = Entry4{b, t0, nt, cost};
}

// Launch order of the bands: full bands by decreasing cost (the tiles with the most rank-extension work start first, the
// cheap ones fill the tail of the launch), ties by band index; a last band with fewer row tiles stays last (the
// kernel's tile numbering needs every band before it to be full).  Counting sort as above.
__global__ void plan_sort_bands_kernel(const Entry4* in, Entry4* out, int32_t n_bands, int band_tiles) {
    const int32_t e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n_bands) return;
    const Entry4 me = in[e];
    const bool me_partial = me.c < band_tiles;
    int32_t pos = 0;
    for (int32_t o = 0; o < n_bands; ++o) {
        const Entry4 other = in[o];
        const bool o_partial = other.c < band_tiles;
        if (me_partial != o_partial) { if (me_partial) ++pos; continue; }
        if (other.d > me.d || (other.d == me.d && o < e)) ++pos;
    }
    out[pos] = me;
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
// case: the same buffers every training step); a stream under graph capture always records the upload, and from then
// on every eager call uploads as well (a replay of the captured graph puts the captured pointers back into the table,
// which the host mirror cannot see).
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
    if (capturing) p->ptr_upload_captured = true;     // replays of that graph rewrite the table: the mirror cannot follow them
    bool same = p->ptr_mirror_valid && p->ptr_mirror_stream == st && !capturing && !p->ptr_upload_captured;
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
    p->ptr_mirror_valid = !capturing && !p->ptr_upload_captured;
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

// The scheduler set-up kernel runs on a stream of the library's own (one per device, default priority, created on
// first use and kept until the process ends), and plan creation waits for that stream only: the counts it reads back
// arrive without draining whatever the caller has queued on the plan's stream.
static std::mutex g_sched_mutex;
constexpr int kMaxSchedDevices = 64;
static hipStream_t g_sched_stream[kMaxSchedDevices] = {};

static int scheduler_stream(hipStream_t* out) {
    int dev = 0;
    MLORA_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxSchedDevices) {
        set_error("device index beyond the scheduler stream table");
        return MLORA_ERR_SHAPE;
    }
    if (!g_sched_stream[dev]) MLORA_HIP_TRY(hipStreamCreateWithFlags(&g_sched_stream[dev], hipStreamNonBlocking));
    *out = g_sched_stream[dev];
    return MLORA_OK;
}

static inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

// `like`: a plan over the same segmentation (same T, N, ranks, scales, offsets) whose segmentation tables the new plan
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

    std::unique_ptr<mlora_plan> holder(new mlora_plan());
    mlora_plan* p = holder.get();
    p->dtype = dtype;
    p->T = T; p->k = k; p->n = n; p->N = N;
    if (N > 0) {
        p->ranks.assign(ranks, ranks + N);
        p->scales.assign(scales, scales + N);
        p->off.assign(seg_offsets, seg_offsets + N + 1);
    } else {
        p->off.assign(1, 0);
    }
    p->build_stream = (hipStream_t)stream;
    // bf16 with 16-byte row granularity goes to the MFMA kernels, everything else to the FMA kernels
    p->use_mfma = (dtype == MLORA_BF16) && (k % 8 == 0) && (n % 8 == 0);

    int dev = 0;
    MLORA_HIP_TRY(hipGetDevice(&dev));
    {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            p->num_cus = cus;
    }

    // Host side: sizes that follow from the adapters alone (one pass over the adapters, none over blocks or chunks).
    // The tables themselves, the token chunks and everything that depends on them come from the device.
    int64_t R1 = 0, rb = 0, rb_wide = 0, rb_narrow = 0;
    for (int32_t i = 0; i < N; ++i) {
        const int64_t Ti = p->off[i + 1] - p->off[i];
        R1 += Ti * ranks[i];
        if (ranks[i] > p->max_rank) p->max_rank = ranks[i];
        if (ranks[i] > 0 && Ti == 0) p->has_empty_ranked = true;
        if (Ti <= 0 || ranks[i] <= 0) continue;
        rb += ceil_div(Ti, kBlockRows);
        if (ranks[i] % 8) p->ranks_mult8 = false;
        if (ranks[i] > kNarrowMaxRank) {
            rb_wide += ceil_div(Ti, kBlockRowsWide);
        } else {
            rb_narrow += ceil_div(Ti, kBlockRows);
            if (ranks[i] > p->max_rank_narrow) p->max_rank_narrow = ranks[i];
        }
    }
    p->R1 = R1;
    p->n_row_blocks = (int32_t)rb;
    p->n_blocks_wide = (int32_t)rb_wide;
    p->n_blocks_narrow = (int32_t)rb_narrow;
    p->n_gemm_tiles = (int32_t)ceil_div(T, kGemmTileRows);
    p->n_bands = (int32_t)ceil_div(p->n_gemm_tiles, kGemmBandTiles);
    p->shares_tables = like != nullptr;

    // first device allocation: everything whose size the adapters alone fix
    const bool own_seg = !p->shares_tables;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t r = o; o += up256(bytes); return r; };
    const size_t nI = sizeof(int32_t) * (size_t)(N + 1), nL = sizeof(int64_t) * (size_t)(N + 1);
    const size_t o_off = take(own_seg ? nI : 0), o_rank = take(own_seg ? nI : 0), o_scale = take(own_seg ? nI : 0);
    const size_t o_soff = take(own_seg ? nL : 0), o_rbs = take(own_seg ? nI : 0), o_cbs = take(own_seg ? nI : 0);
    const size_t o_cbp = take(own_seg ? nI : 0);
    const size_t o_wcs = take(nI), o_wcp = take(nI), o_part = take(nL), o_red = take(nI), o_geo = take(sizeof(DevGeo));
    const size_t o_ptrs = take(sizeof(AdapterPtrs) * (size_t)(N + 1));
    const size_t o_rb = take(own_seg ? sizeof(Entry4) * (size_t)(p->n_row_blocks + 1) : 0);
    const size_t o_cb = take(own_seg ? sizeof(Entry4) * (size_t)(p->n_row_blocks + 1) : 0);
    const size_t o_gt = take(own_seg ? sizeof(Entry4) * (size_t)(p->n_gemm_tiles + 1) : 0);
    const size_t o_bo = take(own_seg ? sizeof(Entry4) * (size_t)(p->n_bands + 1) : 0);
    const size_t o_bo_tmp = take(own_seg ? sizeof(Entry4) * (size_t)(p->n_bands + 1) : 0);
    const size_t o_probs = take(128 * (size_t)(5 * N + 8));
    const size_t o_adamw = take(96 * (size_t)(N + 1));
    auto block1 = std::make_shared<DeviceBlock>();
    MLORA_HIP_TRY(hipMalloc(&block1->ptr, o));
    p->blocks.push_back(block1);
    if (like) {      // every block the shared tables live in, whoever allocated it
        p->shared_blocks = like->shared_blocks;
        p->shared_blocks.insert(p->shared_blocks.end(), like->blocks.begin(), like->blocks.end());
    }
    char* base = (char*)block1->ptr;
    const PlanView* lv = like ? &like->view : nullptr;
    int32_t* d_off = own_seg ? (int32_t*)(base + o_off) : const_cast<int32_t*>(lv->off);
    int32_t* d_rank = own_seg ? (int32_t*)(base + o_rank) : const_cast<int32_t*>(lv->rank);
    float* d_scale = own_seg ? (float*)(base + o_scale) : const_cast<float*>(lv->scale);
    int64_t* d_soff = own_seg ? (int64_t*)(base + o_soff) : const_cast<int64_t*>(lv->soff);
    int32_t* d_rbs = own_seg ? (int32_t*)(base + o_rbs) : nullptr;
    int32_t* d_cbs = own_seg ? (int32_t*)(base + o_cbs) : nullptr;
    int32_t* d_cbp = own_seg ? (int32_t*)(base + o_cbp) : nullptr;
    int32_t* d_wcs = (int32_t*)(base + o_wcs);
    int32_t* d_wcp = (int32_t*)(base + o_wcp);
    int64_t* d_part = (int64_t*)(base + o_part);
    p->d_reduce_list = (int32_t*)(base + o_red);
    DevGeo* d_geo = (DevGeo*)(base + o_geo);
    p->d_ptrs = (AdapterPtrs*)(base + o_ptrs);
    Entry4* d_rb = own_seg ? (Entry4*)(base + o_rb) : const_cast<Entry4*>(lv->row_blocks);
    Entry4* d_cb = own_seg ? (Entry4*)(base + o_cb) : const_cast<Entry4*>(lv->class_blocks);
    Entry4* d_gt = own_seg ? (Entry4*)(base + o_gt) : const_cast<Entry4*>(lv->gemm_tiles);
    Entry4* d_bo = own_seg ? (Entry4*)(base + o_bo) : const_cast<Entry4*>(lv->band_order);
    p->d_probs = base + o_probs;
    p->d_adamw = base + o_adamw;

    // scheduler set-up on the library's own stream; the host waits for that stream alone
    {
        std::lock_guard<std::mutex> lock(g_sched_mutex);
        hipStream_t ss = nullptr;
        const int src = scheduler_stream(&ss);
        if (src != MLORA_OK) return src;
        if (own_seg) {
            p->off32.resize(N + 1);
            for (int32_t i = 0; i <= N; ++i) p->off32[i] = (int32_t)p->off[i];
            MLORA_HIP_TRY(hipMemcpyAsync(d_off, p->off32.data(), nI, hipMemcpyHostToDevice, ss));
            if (N > 0) {
                MLORA_HIP_TRY(hipMemcpyAsync(d_rank, p->ranks.data(), sizeof(int32_t) * N, hipMemcpyHostToDevice, ss));
                MLORA_HIP_TRY(hipMemcpyAsync(d_scale, p->scales.data(), sizeof(float) * N, hipMemcpyHostToDevice, ss));
            }
        }
        const int64_t panels = ceil_div(k, kWgradPanelCols) + ceil_div(n, kWgradPanelCols);
        hipLaunchKernelGGL(plan_scan_kernel, dim3(1), dim3(kScanThreads), 0, ss, N, d_off, d_rank, panels, k + n,
                           (int32_t)p->num_cus, kBlockRows, kBlockRowsWide, kWgradMinChunkRows, own_seg ? d_soff : nullptr,
                           d_rbs, d_cbs, d_cbp, d_wcs, d_wcp, d_part, p->d_reduce_list, d_geo);
        MLORA_HIP_TRY(hipGetLastError());
        MLORA_HIP_TRY(hipMemcpyAsync(&p->geo, d_geo, sizeof(DevGeo), hipMemcpyDeviceToHost, ss));
        MLORA_HIP_TRY(hipStreamSynchronize(ss));
    }
    const DevGeo& geo = p->geo;
    if (geo.R1 != p->R1 || geo.n_row_blocks != p->n_row_blocks || geo.n_blocks_wide != p->n_blocks_wide) {
        set_error("device-side scheduler disagrees with the host about the segmentation");
        return MLORA_ERR_HIP;
    }
    const size_t esz = dtype == MLORA_BF16 ? 2 : 4;
    p->ws_ds_bytes = up256((size_t)p->R1 * esz);
    p->ws_partial_bytes = up256((size_t)geo.partial_floats * sizeof(float));

    // second allocation: the chunk table, sized by what the device chose
    Entry4 *d_wc = nullptr, *d_wc_tmp = nullptr;
    {
        const size_t tab = up256(sizeof(Entry4) * (size_t)(geo.n_chunks + 1));
        auto block2 = std::make_shared<DeviceBlock>();
        MLORA_HIP_TRY(hipMalloc(&block2->ptr, 2 * tab));
        p->blocks.push_back(block2);
        d_wc = (Entry4*)block2->ptr;
        d_wc_tmp = (Entry4*)((char*)block2->ptr + tab);
    }

    const int32_t n_class_blocks = p->n_blocks_wide + p->n_blocks_narrow;
    // table builds on the plan's stream (their inputs were complete when the wait above returned)
    hipStream_t st = p->build_stream;
    auto grid_for = [](int32_t cnt) { return dim3((unsigned)((cnt + 255) / 256)); };
    if (own_seg && p->n_row_blocks > 0) {
        hipLaunchKernelGGL(plan_fill_blocks_kernel, grid_for(p->n_row_blocks), dim3(256), 0, st, N, d_off, d_rank, d_rbs, d_rbs,
                           kBlockRows, kBlockRows, d_rb, p->n_row_blocks);
        hipLaunchKernelGGL(plan_fill_blocks_kernel, grid_for(n_class_blocks), dim3(256), 0, st, N, d_off, d_rank, d_cbs, d_cbp,
                           kBlockRows, kBlockRowsWide, d_cb, n_class_blocks);
    }
    if (geo.n_chunks > 0) {
        // class-ordered canonical table, then reordered by cost inside each class (very large tables keep the first)
        const bool sorted = geo.n_chunks <= kMaxSortedChunks;
        hipLaunchKernelGGL(plan_fill_blocks_kernel, grid_for(geo.n_chunks), dim3(256), 0, st, N, d_off, d_rank, d_wcs, d_wcp,
                           geo.chunk_rows, geo.chunk_rows_wide, sorted ? d_wc_tmp : d_wc, geo.n_chunks);
        if (sorted)
            hipLaunchKernelGGL(plan_sort_chunks_kernel, grid_for(geo.n_chunks), dim3(256), 0, st, d_wc_tmp, d_rank, d_wc,
                               geo.n_chunks, geo.n_chunks_wide);
    }
    if (own_seg && p->n_gemm_tiles > 0) {
        hipLaunchKernelGGL(plan_fill_gemm_tiles_kernel, grid_for(p->n_gemm_tiles), dim3(256), 0, st, N, d_off, (int32_t)T,
                           kGemmTileRows, d_gt, p->n_gemm_tiles);
        Entry4* d_bo_tmp = (Entry4*)(base + o_bo_tmp);
        const bool sorted = p->n_bands <= kMaxSortedChunks;
        hipLaunchKernelGGL(plan_band_cost_kernel, grid_for(p->n_bands), dim3(256), 0, st, N, d_off, d_rank, d_gt,
                           p->n_gemm_tiles, kGemmBandTiles, sorted ? d_bo_tmp : d_bo, p->n_bands);
        if (sorted)
            hipLaunchKernelGGL(plan_sort_bands_kernel, grid_for(p->n_bands), dim3(256), 0, st, d_bo_tmp, d_bo, p->n_bands,
                               kGemmBandTiles);
    }
    MLORA_HIP_TRY(hipGetLastError());
    prepare_static_workspace();

    PlanView& v = p->view;
    v.N = N; v.T = T; v.k = k; v.n = n;
    v.off = d_off; v.rank = d_rank; v.scale = d_scale; v.soff = d_soff; v.ptrs = p->d_ptrs;
    v.row_blocks = d_rb; v.n_row_blocks = p->n_row_blocks;
    v.class_blocks = d_cb; v.n_class_blocks = n_class_blocks;
    v.gemm_tiles = d_gt; v.n_gemm_tiles = p->n_gemm_tiles;
    v.band_order = d_bo; v.n_bands = p->n_bands;
    v.wgrad_chunks = d_wc; v.n_wgrad_chunks = geo.n_chunks;
    v.wgrad_chunk_start = d_wcs;
    v.part_off = d_part;
    *out = holder.release();
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
    out[MLORA_GEO_WGRAD_CHUNK_ROWS] = plan->geo.chunk_rows;
    out[MLORA_GEO_WGRAD_CHUNK_ROWS_WIDE] = plan->geo.chunk_rows_wide;
    out[MLORA_GEO_BLOCK_ROWS_WIDE] = kBlockRowsWide;
    out[MLORA_GEO_GEMM_BAND_TILES] = kGemmBandTiles;
    out[MLORA_GEO_NUM_CUS] = plan->num_cus;
    out[MLORA_GEO_WGRAD_PANEL_COLS] = kWgradPanelCols;
    out[MLORA_GEO_WGRAD_MIN_CHUNK_ROWS] = kWgradMinChunkRows;
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
        case MLORA_TABLE_WGRAD_CHUNKS: src = plan->view.wgrad_chunks; cnt = plan->geo.n_chunks; break;
        case MLORA_TABLE_CLASS_BLOCKS: src = plan->view.class_blocks; cnt = plan->view.n_class_blocks; break;
        case MLORA_TABLE_GEMM_BAND_ORDER: src = plan->view.band_order; cnt = plan->n_bands; break;
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

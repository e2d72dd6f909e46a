/*
 * multi_lora.h -- C ABI of the fused multi-LoRA linear layer for AMD MI355X (gfx950).
 *
 * Many LoRA jobs share one frozen weight W.  All jobs' tokens sit in one flat
 * activation buffer X[T,k]; adapter i owns the contiguous row segment
 * [seg_offsets[i], seg_offsets[i+1]) and has its own rank r_i, scale s_i and
 * matrices A_i[k,r_i], B_i[r_i,n]  (paper Sec. 2.1 for the LoRA branch Y = XW + XAB,
 * Sec. 5.1 for the grouped forward/backward, App. A.1 for the flat token buffer with
 * per-adapter offsets, the (adapter, block) schedule table and rank masking).
 *
 *   forward    S_i  = X_i A_i                       [T_i, r_i]   (cached for backward)
 *              Y_i  = X_i W + s_i S_i B_i           [T_i, n]
 *   backward   dS_i = s_i dY_i B_i^T                [T_i, r_i]
 *              dX_i = dY_i W^T + dS_i A_i^T         [T_i, k]
 *              dA_i = X_i^T dS_i                    [k, r_i]
 *              dB_i = s_i S_i^T dY_i                [r_i, n]     (W is frozen: no dW)
 *
 * Layout: every matrix is dense row-major.  W is [k,n] (the paper's orientation, not
 * torch's [out,in]).  S and dS are ragged: S_i starts at element sum_{j<i} T_j r_j and
 * is [T_i, r_i] dense.  dtype is one of MLORA_F32 / MLORA_BF16 for all tensors;
 * accumulation is always fp32 and each output is rounded once from the accumulator.
 *
 * Pointers: "device" = device memory the caller owns (for example torch tensors),
 * "host" = ordinary host memory read during the call and free to reuse once the call
 * returns.  `stream` is a hipStream_t passed as void* (NULL = the null stream).
 * Every call only enqueues work on `stream`; none of them synchronises the device.
 * A plan and its workspace may be in use on one stream at a time.
 *
 * Errors: every entry point returns MLORA_OK (0) or a negative mlora_status; argument
 * checks happen before any GPU call, nothing is thrown or aborted, and
 * multi_lora_last_error() returns a thread-local description of the last failure.
 */
#ifndef MULTI_LORA_H_
#define MULTI_LORA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mlora_plan mlora_plan; /* opaque, library-owned */

typedef enum { MLORA_F32 = 0, MLORA_BF16 = 1 } mlora_dtype;

typedef enum {
    MLORA_OK = 0,
    MLORA_ERR_NULL = -1,      /* a required pointer is NULL */
    MLORA_ERR_SHAPE = -2,     /* T, k, n or N out of range */
    MLORA_ERR_SEGMENTS = -3,  /* offsets do not start at 0, decrease, or do not end at T */
    MLORA_ERR_RANK = -4,      /* a rank is outside [0, MLORA_MAX_RANK] */
    MLORA_ERR_DTYPE = -5,
    MLORA_ERR_ALIGN = -6,     /* a device pointer is not 16-byte aligned */
    MLORA_ERR_WORKSPACE = -7, /* workspace NULL although multi_lora_workspace_bytes() > 0 */
    MLORA_ERR_HIP = -8,       /* a HIP runtime call failed; see multi_lora_last_error() */
    MLORA_ERR_FLAGS = -9,     /* unknown or contradictory flag bits */
    MLORA_ERR_SCALE = -10     /* a scale is NaN or infinite */
} mlora_status;

#define MLORA_MAX_RANK 128      /* App. A.1: ranks are small, typically r <= 128 */
#define MLORA_MAX_ADAPTERS 4096

/* flags of multi_lora_fwd / multi_lora_bwd */
#define MLORA_FLAG_BASE_ONLY 1u /* skip every LoRA term: Y = X W, dX = dY W^T; S, dA, dB untouched */
#define MLORA_FLAG_LORA_ONLY 2u /* skip W: fwd Y += s S B in place (Y holds Y_base on entry, the
                                   paper's decoupled "fused GEMM-add", Sec. 5.1 / App. A.1);
                                   bwd dX += dS A^T in place; S, dA, dB as usual */
#define MLORA_FLAG_ACCUM_GRADS 4u /* multi_lora_bwd only: dA_i, dB_i += this call's gradients instead of being
                                   overwritten (gradient accumulation over micro-batches; the paper's runs use 1
                                   accumulation step).  The sum is formed in fp32 from the stored value and the
                                   fp32 result and rounded once to the plan dtype.  dX is not affected. */
#define MLORA_FLAG_GROUP_BANDS 8u /* bf16 tile order only, results unchanged bit for bit: sweep the frozen weight once
                                   per group of four 2048-row bands instead of once per band.  The library does this by
                                   itself when W is larger than half the Infinity Cache and the bands' rows fit the other
                                   half; the flag forces it for any shape (tuning, tests).  Ignored by the fp32 path. */

/* which table multi_lora_plan_dump copies out */
typedef enum {
    MLORA_TABLE_ROW_BLOCKS = 0, /* LoRA block table, 4 x int32 per entry:
                                   adapter, block index within the adapter, first global row, rows.
                                   App. A.1 schedule table; order: adapter ascending, block ascending;
                                   adapters with T_i = 0 or r_i = 0 have no entries. */
    MLORA_TABLE_GEMM_ROW_TILES = 1, /* row tiles of the flat buffer used by the fused GEMMs,
                                   4 x int32 per entry: first row, rows, first adapter touched,
                                   last adapter touched + 1. */
    MLORA_TABLE_WGRAD_CHUNKS = 2, /* token chunks reduced by the weight-gradient kernels, 4 x int32:
                                   adapter, chunk index within the adapter, first global row, rows.
                                   Same entries as a block table with MLORA_GEO_WGRAD_CHUNK_ROWS rows per
                                   block (MLORA_GEO_WGRAD_CHUNK_ROWS_WIDE for adapters with a rank above 64; the
                                   two differ only in plans that hold ranks on both sides of 64, whose two rank
                                   classes are balanced separately), in launch order: adapters with a rank above 64
                                   first, then the others; inside a class by decreasing cost rows x (64 + rank), ties in
                                   canonical order (the device-side balancing of heterogeneous segments);
                                   tables above 16384 entries keep the canonical order inside each class. */
    MLORA_TABLE_CLASS_BLOCKS = 3, /* the LoRA blocks in the order the grouped kernels walk them, same entry format as
                                   MLORA_TABLE_ROW_BLOCKS: adapters with a rank above 64 first (their blocks run longest
                                   and take a kernel build of their own), cut every MLORA_GEO_BLOCK_ROWS_WIDE rows, then
                                   the others, cut every MLORA_GEO_BLOCK_ROWS rows; canonical order inside a class. */
    MLORA_TABLE_GEMM_BAND_ORDER = 4 /* launch order of the fused GEMMs' row bands (MLORA_GEO_GEMM_BAND_TILES consecutive
                                   row tiles x all column tiles are in flight together), 4 x int32: band, first row tile,
                                   row tiles, cost = rank-extension passes of its row tiles (per row tile, one per 64 ranks
                                   of every adapter that owns rows of it).  Full bands by decreasing cost, ties by band
                                   index; a last band with fewer row tiles stays last.  Above 16384 bands: band order. */
} mlora_table;

/* geometry words returned by multi_lora_plan_geometry */
enum {
    MLORA_GEO_BLOCK_ROWS = 0,     /* rows per LoRA block (MLORA_TABLE_ROW_BLOCKS) */
    MLORA_GEO_GEMM_TILE_ROWS = 1, /* rows per fused-GEMM row tile */
    MLORA_GEO_GEMM_TILE_COLS = 2,
    MLORA_GEO_WGRAD_CHUNK_ROWS = 3,
    MLORA_GEO_R1_LO = 4,          /* sum_i T_i r_i, low and high 31 bits */
    MLORA_GEO_R1_HI = 5,
    MLORA_GEO_USES_MFMA = 6,      /* 1 if the bf16 MFMA kernels serve this plan, 0 for the fp32-FMA kernels */
    MLORA_GEO_WGRAD_CHUNK_ROWS_WIDE = 7, /* token chunk of adapters with a rank above 64 */
    MLORA_GEO_BLOCK_ROWS_WIDE = 8,    /* rows per LoRA block of adapters with a rank above 64 */
    MLORA_GEO_GEMM_BAND_TILES = 9,    /* row tiles per band of the fused GEMMs' tile order */
    MLORA_GEO_NUM_CUS = 10,           /* compute units the token chunks were balanced for */
    MLORA_GEO_WGRAD_PANEL_COLS = 11,  /* columns of X / dY one weight-gradient work item covers */
    MLORA_GEO_WGRAD_MIN_CHUNK_ROWS = 12, /* the token chunk is never cut below this */
    MLORA_GEO_COUNT = 13
};

/*
 * Build the per-segmentation plan (App. A.1: the schedule table is built once per step
 * from the per-adapter offsets and shared by every layer).  Validates the arguments,
 * allocates the small device tables and builds them with a device kernel on `stream`.
 *   out          host, receives the plan
 *   T, k, n      token count (>= 0), input width (>= 1), output width (>= 1)
 *   N            number of adapters, 0..MLORA_MAX_ADAPTERS.  With N = 0 all T rows are plain X W rows
 *                (Y = X W, dX = dY W^T); ranks, scales and seg_offsets are then not read and may be NULL,
 *                and the A / B / dA / dB pointer arrays of multi_lora_fwd / multi_lora_bwd may be NULL.
 *   ranks        host [N], each in [0, MLORA_MAX_RANK]; rank 0 = rows pass through as X W
 *   scales       host [N], finite
 *   seg_offsets  host [N+1], seg_offsets[0] = 0, non-decreasing, seg_offsets[N] = T (N >= 1)
 * The token chunks of the weight-gradient items are chosen, and all tables are built and ordered, by device kernels from
 * the offsets and ranks (the device-side scheduler); the call waits for the first of them, which runs on a stream of the
 * library's own, to read back the sizes it chose - it does not wait for work queued on `stream`.
 * With multi_lora_plan_create_like the only entry point that allocates device memory; freed by multi_lora_plan_destroy.
 */
int multi_lora_plan_create(mlora_plan** out, int dtype, int64_t T, int64_t k, int64_t n,
                           int32_t N, const int32_t* ranks, const float* scales,
                           const int64_t* seg_offsets, void* stream);

/*
 * A plan for another layer shape (k, n) over the segmentation of `base` (same T, adapters, ranks, scales and
 * offsets): App. A.1 builds the schedule table once per step and every layer of the step uses it.  The new plan
 * uses the device tables of `base` in place (row blocks, row tiles, offsets, ranks, scales; the weight-gradient
 * item table too when both shapes chunk the tokens alike) and builds only what depends on the layer: its pointer
 * table and workspace layout.  `stream` must be the stream `base` was created on.  The two plans are independent
 * afterwards: either may be destroyed first - also along a chain of plans each made from the one before -, and each is
 * used by one stream at a time as usual.
 */
int multi_lora_plan_create_like(mlora_plan** out, const mlora_plan* base, int64_t k, int64_t n, void* stream);

/* Frees the plan's device tables (synchronises with nothing: destroy a plan only after
 * the work that uses it has finished).  NULL is accepted. */
int multi_lora_plan_destroy(mlora_plan* plan);

/* Argument validation alone, with the same status codes as multi_lora_plan_create and
 * without touching the GPU. */
int multi_lora_validate(int dtype, int64_t T, int64_t k, int64_t n, int32_t N,
                        const int32_t* ranks, const float* scales, const int64_t* seg_offsets);

/* Bytes of caller-allocated device workspace multi_lora_fwd / multi_lora_bwd need
 * (fp32 partial sums of the weight gradients and the dS buffer).  0 is possible. */
size_t multi_lora_workspace_bytes(const mlora_plan* plan);

/* Copies MLORA_GEO_COUNT int32 words describing the plan's tiling into `out` (host). */
int multi_lora_plan_geometry(const mlora_plan* plan, int32_t* out);

/* Copies a device-built table back to the host for bit-exact bookkeeping checks.
 * `entries` (host) receives up to `cap` entries of 4 int32 each; `count` (host) the
 * number of entries the table holds.  Synchronises the plan's build stream. */
int multi_lora_plan_dump(const mlora_plan* plan, int which, int32_t* entries, int64_t cap,
                         int64_t* count);

/*
 * Forward (Sec. 5.1: base GEMM, grouped shrink, fused expand-add; here the expand is
 * folded into the base GEMM's accumulator so Y is written exactly once).
 *   X  device [T,k]        W  device [k,n]
 *   A  host array of N device pointers, A_i [k,r_i]   (entries with r_i = 0 are ignored)
 *   B  host array of N device pointers, B_i [r_i,n]
 *   Y  device [T,n] out (in/out with MLORA_FLAG_LORA_ONLY)
 *   S  device ragged [sum T_i r_i] out, unscaled X_i A_i
 *   workspace  device, multi_lora_workspace_bytes(plan) bytes
 * The pointer arrays are copied into a device table owned by the plan; a call that passes the same
 * pointers on the same stream as the previous call reuses the table without another launch.  One plan
 * must not be used from two streams at once.
 */
int multi_lora_fwd(mlora_plan* plan, const void* X, const void* W, const void* const* A,
                   const void* const* B, void* Y, void* S, void* workspace, uint32_t flags,
                   void* stream);

/*
 * Backward (Sec. 5.1: grouped input gradients dS, dX; grouped weight gradients dA, dB
 * reduced over each adapter's tokens; W frozen).  All outputs are overwritten.
 *   dY device [T,n]   X device [T,k]   W device [k,n]   S device ragged, from forward
 *   A, B   host arrays of N device pointers as in forward
 *   dX device [T,k] out (in/out with MLORA_FLAG_LORA_ONLY)
 *   dA host array of N device pointers, dA_i [k,r_i] out
 *   dB host array of N device pointers, dB_i [r_i,n] out
 * dS is kept in the workspace (first sum T_i r_i elements of the plan dtype).
 */
int multi_lora_bwd(mlora_plan* plan, const void* dY, const void* X, const void* W,
                   const void* const* A, const void* const* B, const void* S, void* dX,
                   void* const* dA, void* const* dB, void* workspace, uint32_t flags,
                   void* stream);

/*
 * multi_lora_bwd for callers that cannot allocate device memory or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results (bit for bit) and errors as
 * multi_lora_bwd, but the workspace (dS and the fp32 partial weight gradients) is a static device array of
 * MLORA_STATIC_WORKSPACE_BYTES that belongs to the loaded library; every GPU the library runs on holds one copy until
 * the process ends.  The call allocates and frees nothing on host or device through HIP.  A plan whose
 * multi_lora_workspace_bytes() exceeds MLORA_STATIC_WORKSPACE_BYTES is rejected with MLORA_ERR_WORKSPACE before any
 * GPU work.  All calls on one GPU share the one array and it keeps the last call's contents (nothing in it has to start
 * at zero: each call writes dS and every partial sum it reads): two multi_lora_bwd_static calls that may overlap on
 * one GPU - different streams, different plans or different threads - race on it and must be serialised by the caller.
 * dS of the last call is not exposed.
 */
#define MLORA_STATIC_WORKSPACE_BYTES (64u << 20)
int multi_lora_bwd_static(mlora_plan* plan, const void* dY, const void* X, const void* W,
                          const void* const* A, const void* const* B, const void* S, void* dX,
                          void* const* dA, void* const* dB, uint32_t flags, void* stream);

/* kernel ids reported by multi_lora_profile_end */
enum {
    MLORA_K_SHRINK = 0,      /* S_i = X_i A_i (grouped) */
    MLORA_K_GEMM_FWD = 1,    /* Y = X W + s_i S_i B_i (fused) */
    MLORA_K_DSHRINK = 2,     /* dS_i = s_i dY_i B_i^T (grouped) */
    MLORA_K_GEMM_BWD = 3,    /* dX = dY W^T + dS_i A_i^T (fused) */
    MLORA_K_WGRAD = 4,       /* dA_i, dB_i token reductions (grouped) */
    MLORA_K_WGRAD_REDUCE = 5,/* fixed-order sum of chunk partials */
    MLORA_K_OTHER = 6,       /* pointer upload, descriptor set-up, FMA-path launches */
    MLORA_K_ADAMW = 7        /* grouped per-adapter AdamW update */
};

/*
 * Per-kernel timing for benchmarks (not from the paper; a measurement aid).  Between
 * multi_lora_profile_begin and multi_lora_profile_end every kernel the plan launches is
 * bracketed by HIP events recorded on the launch stream.  `max_records` bounds the number of
 * launches recorded (later ones are ignored).  multi_lora_profile_end waits for the recorded
 * work, writes up to `cap` (kernel id, milliseconds) pairs to `kernel_ids` / `ms` (host arrays),
 * the number of records to `count`, and switches recording off.
 */
int multi_lora_profile_begin(mlora_plan* plan, int32_t max_records);
int multi_lora_profile_end(mlora_plan* plan, int32_t* kernel_ids, float* ms, int32_t cap,
                           int32_t* count);

/*
 * Per-adapter AdamW on the LoRA matrices, one grouped launch for all adapters.  The paper gives every
 * LoRA job its own optimizer instance (Sec. 5.2) and trains with AdamW, weight decay 0.01, constant
 * learning rate (App., training details); its 8-bit paged state is not reproduced: the state here is
 * fp32.  Update, per element, with t = hp[i].step (1-based, per adapter):
 *     m <- beta1 m + (1-beta1) g ;  v <- beta2 v + (1-beta2) g^2
 *     master <- master - lr ( (m / (1-beta1^t)) / (sqrt(v / (1-beta2^t)) + eps) + weight_decay master )
 *     A_i / B_i <- master rounded to the plan dtype
 * stateA[i] / stateB[i]: device, 3 * numel floats laid out [master | m | v] (numel = k r_i or r_i n).
 * A, B, dA, dB, stateA, stateB: host arrays of N device pointers (entries of rank-0 adapters ignored);
 * hp: host [N].  multi_lora_adamw_init copies A_i, B_i into the masters and zeroes m, v.
 */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    int32_t step;
} mlora_adamw_hparams;

int multi_lora_adamw_init(mlora_plan* plan, const void* const* A, const void* const* B,
                          float* const* stateA, float* const* stateB, void* stream);
int multi_lora_adamw_step(mlora_plan* plan, void* const* A, void* const* B, const void* const* dA,
                          const void* const* dB, float* const* stateA, float* const* stateB,
                          const mlora_adamw_hparams* hp, void* stream);

/*
 * Measurement aids for benchmarks (no part of the layer; both synchronise the stream and take a few tens of ms).
 * multi_lora_calib_mfma: TFLOP/s of a register-only loop of the 16x16x32 bf16 MFMAs the fused GEMM is built from,
 *   8 wavefronts per CU; random_data != 0 uses random operands (the power draw of a real GEMM, under which the
 *   board reaches its power limit and lowers the clock), 0 uses zeros (no throttling).
 * multi_lora_calib_read: GB/s of a coalesced streaming read of `buffer` (device, 16-byte aligned, >= 1 MiB).
 * scratch: device, at least 4096 bytes, never written in practice.  tflops / gbs: host, out.
 */
int multi_lora_calib_mfma(int32_t random_data, void* scratch, float* tflops, void* stream);
int multi_lora_calib_read(const void* buffer, size_t bytes, void* scratch, float* gbs, void* stream);

/* Thread-local text of the last error returned on this thread ("" if none). */
const char* multi_lora_last_error(void);

/* Library version, "major.minor". */
const char* multi_lora_version(void);

/* ---------------------------------------------------------------------------------------------
 * Loss-aware early exit (Sec. 4.1, Algorithm "Loss-Aware Pattern Detection"; Sec. 4.2).  Host only, no GPU work.
 * One monitor tracks n adapters.  Report every training loss with multi_lora_monitor_train_loss (it feeds the
 * exponential moving average lhat <- alpha l + (1 - alpha) lhat, seeded with the first loss) and every validation
 * loss with multi_lora_monitor_val_loss, which appends (lhat, val) to the adapter's histories and applies
 *   divergence:  once `window` evaluations exist, the least-squares slopes of the last `window` values of both
 *                histories; both >= tau_slope for patience_div evaluations in a row -> MLORA_EXIT_DIVERGING;
 *   overfitting: (val - lhat) / lhat > tau_gap for patience_ovf evaluations in a row -> MLORA_EXIT_OVERFITTING
 *                (multi_lora_monitor_state names the evaluation step with the best validation loss to restore);
 * divergence is tested first.  A training or validation loss that is NaN or infinite is divergence decided at once
 * (MLORA_EXIT_DIVERGING from that report on; it enters neither the moving average nor the histories).
 * A decision is final: later reports for that adapter return it again.
 * multi_lora_monitor_warmup_select is the warmup boundary: the surviving adapters are ranked by their latest
 * validation loss (ascending, ties in adapter order, never-evaluated last) and all but the best
 * ceil(ratio x survivors) become MLORA_EXIT_UNDERPERFORMING; `status` (host, [n]) receives every adapter's status.
 * Errors: MLORA_ERR_NULL, MLORA_ERR_SHAPE (index or parameter out of range, validation before any training loss).
 * A monitor is not thread safe.
 */
typedef struct mlora_monitor mlora_monitor;
typedef struct {
    double ema_alpha;       /* weight of the newest training loss, (0, 1] */
    int32_t window;         /* w >= 2, in evaluation steps */
    int32_t patience_div;   /* p_div >= 1 */
    int32_t patience_ovf;   /* p_ovf >= 1 */
    double tau_slope;
    double tau_gap;
} mlora_monitor_params;
typedef struct {
    double ema_train_loss;  /* NaN before the first training loss */
    double best_val_loss;   /* +inf before the first evaluation */
    int32_t best_eval_step; /* 0-based index of that evaluation, -1 before the first */
    int32_t evaluations;
    int32_t count_diverging, count_overfitting;
    int32_t status;         /* MLORA_EXIT_* */
} mlora_monitor_state;
enum { MLORA_EXIT_CONTINUE = 0, MLORA_EXIT_DIVERGING = 1, MLORA_EXIT_OVERFITTING = 2, MLORA_EXIT_UNDERPERFORMING = 3 };

int multi_lora_monitor_create(mlora_monitor** out, int32_t n_adapters, const mlora_monitor_params* params);
int multi_lora_monitor_destroy(mlora_monitor* monitor);
int multi_lora_monitor_train_loss(mlora_monitor* monitor, int32_t adapter, double loss);
int multi_lora_monitor_val_loss(mlora_monitor* monitor, int32_t adapter, double val_loss, int32_t* decision);
int multi_lora_monitor_warmup_select(mlora_monitor* monitor, double ratio, int32_t* status);
int multi_lora_monitor_state(const mlora_monitor* monitor, int32_t adapter, mlora_monitor_state* out);

/* ---------------------------------------------------------------------------------------------
 * Online greedy intra-task scheduling (Sec. 6.1; App. "Intra-Task Scheduling Details").  Host only, no GPU work.
 * multi_lora_memory_model_fit fits the profiled points (total batch x sequence length, peak bytes) to
 * Mhat(B) = k0 + k1 B L by least squares.  A scheduler keeps pending jobs (submission order) and running jobs (admission
 * order); a job fits while  k0 + k1 (B_running + b) L <= safety_margin x capacity_bytes.
 *   _submit   adds a pending job with its per-adapter batch size (ids are the caller's, unique among live jobs);
 *   _fill     greedy pass: pending jobs in decreasing batch size (submission order within a size), every job that fits
 *             is admitted, one that does not is skipped; `admitted` (host, cap entries) receives the ids in order;
 *   _exit     a running job leaves (early exit or completion): the oldest pending job of the same batch size takes the
 *             slot if it fits, then the greedy pass runs over what is still pending; `admitted` as above;
 *   _running  the co-located set in admission order = the adapter order of the next step's batch.
 * If an output array is too small the call returns MLORA_ERR_SHAPE with *count set; the scheduler state has changed.
 * Errors: MLORA_ERR_NULL, MLORA_ERR_SHAPE (bad parameter, duplicate id, job not running).  Not thread safe.
 */
typedef struct mlora_admission mlora_admission;
typedef struct {
    double k0, k1;           /* bytes, bytes per (sample x token) */
    double capacity_bytes;   /* HBM capacity the executor may use */
    double safety_margin;    /* usable fraction of the capacity, (0, 1] */
    int64_t seq_len;         /* L */
} mlora_admission_params;

int multi_lora_memory_model_fit(int32_t n_points, const double* batch_times_seq, const double* peak_bytes,
                                double* k0, double* k1);
int multi_lora_admission_create(mlora_admission** out, const mlora_admission_params* params);
int multi_lora_admission_destroy(mlora_admission* scheduler);
int multi_lora_admission_submit(mlora_admission* scheduler, int32_t job_id, int32_t batch_size);
int multi_lora_admission_fill(mlora_admission* scheduler, int32_t* admitted, int32_t cap, int32_t* count);
int multi_lora_admission_exit(mlora_admission* scheduler, int32_t job_id, int32_t* admitted, int32_t cap, int32_t* count);
int multi_lora_admission_running(const mlora_admission* scheduler, int32_t* job_ids, int32_t* batch_sizes, int32_t cap,
                                 int32_t* count);

/* ---------------------------------------------------------------------------------------------
 * Dynamic inter-task scheduling (Sec. 6.2).  Host only, no GPU work.  n tasks with profiled durations d_i > 0 and GPU
 * requirements g_i in [1, G] on G interchangeable GPUs; a task holds its g_i GPUs from its start for d_i; the makespan
 * is minimised exactly (the problem the paper states as a constraint program over start times, GPU assignments and
 * pair orders with no-overlap constraints per shared GPU).
 *
 * multi_lora_schedule_tasks: one solve.
 *   durations, gpus_needed  host [n], n in [0, MLORA_MAX_TASKS]
 *   release                 host [G] or NULL: time from which GPU q may be used (GPUs still held by running work);
 *                           values before `now`, and NULL, mean `now`
 *   starts                  host [n] out, start times >= now
 *   gpu_masks               host [n] out, bit q set = the task runs on GPU q; handed out in order of start time
 *                           (ties: more GPUs first, then longer, then lower index), lowest idle GPU first
 *   makespan                host out, max(now, max_i starts[i] + d_i)
 *   proved_optimal          host out or NULL: 1 if the search ran to its end (the schedule is the optimum described
 *                           below), 0 if it ran out of its budget of about a second of search and the schedule is the
 *                           best one found until then (valid, not proved optimal; only seen above some 12 tasks)
 * Among the schedules that reach the optimum the result is a fixed one: tasks are ordered by (g descending, d
 * descending, index ascending), orders of the tasks are walked depth first in that order (tasks with equal d and g only
 * in index order), every order is turned into a schedule by placing its tasks one after the other at their earliest
 * feasible start, and the first order that reaches the minimum wins.  Times closer than 1e-9 count as equal.
 * Exact search, exponential in the worst case: meant for the handful of tasks of a cluster queue (the paper's case, 11
 * tasks on 8 GPUs, takes milliseconds).
 *
 * mlora_cluster: the event loop around it.  Task arrival (_submit) and task completion (_complete, usually earlier than
 * the estimate because adapters exit early) re-plan all waiting tasks around the running ones, whose GPUs count as
 * released at their estimated end (or `now` once that has passed).  _poll(now) starts every waiting task whose planned
 * start has come and for which enough GPUs are idle - in order of planned start, lowest idle GPUs first - and reports
 * them; if a task had to start late or could not start because a running task has overrun its estimate it re-plans.
 * _plan reports the waiting tasks in submission order with their planned starts, and the planned makespan.
 * Task ids are handed out by _submit (0, 1, 2, ...).  If an output array is too small the call returns MLORA_ERR_SHAPE
 * with *count set; for _poll the tasks have been started all the same.
 * Errors: MLORA_ERR_NULL, MLORA_ERR_SHAPE (bad parameter, too many waiting tasks, task not running).  Not thread safe.
 */
#define MLORA_MAX_TASKS 24
#define MLORA_MAX_CLUSTER_GPUS 64
typedef struct mlora_cluster mlora_cluster;

int multi_lora_schedule_tasks(int32_t n, const double* durations, const int32_t* gpus_needed, int32_t G,
                              const double* release, double now, double* starts, uint64_t* gpu_masks,
                              double* makespan, int32_t* proved_optimal);
int multi_lora_cluster_create(mlora_cluster** out, int32_t G);
int multi_lora_cluster_destroy(mlora_cluster* cluster);
int multi_lora_cluster_submit(mlora_cluster* cluster, double now, double duration, int32_t gpus, int32_t* task_id);
int multi_lora_cluster_complete(mlora_cluster* cluster, double now, int32_t task_id);
int multi_lora_cluster_poll(mlora_cluster* cluster, double now, int32_t* task_ids, uint64_t* gpu_masks, int32_t cap,
                            int32_t* count);
int multi_lora_cluster_plan(const mlora_cluster* cluster, int32_t* task_ids, double* planned_starts, int32_t cap,
                            int32_t* count, double* planned_makespan);

#ifdef __cplusplus
}
#endif
#endif /* MULTI_LORA_H_ */

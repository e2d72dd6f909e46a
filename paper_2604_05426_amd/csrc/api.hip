// multi_lora_fwd / multi_lora_bwd: argument checks, per-call pointer upload, kernel dispatch.
#include <mutex>

#include "common.h"

using namespace mlora;

// Backward workspace of multi_lora_bwd_static: device memory that belongs to the loaded library, so that callers which may
// not allocate (under graph capture, in a serving loop) have a backward that needs no workspace argument.  Every GPU the
// library runs on holds its own copy of this array at its own address until the process ends.  In host code the array's
// name is only a handle for hipGetSymbolAddress: the device address is looked up once per device and kept in
// g_scratch_ptr, and only that pointer is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[MLORA_STATIC_WORKSPACE_BYTES];

static std::mutex g_scratch_mutex;
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call per device).
static int static_workspace(void** out) {
    int dev = 0;
    MLORA_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) {
        set_error("device index beyond the static workspace table");
        return MLORA_ERR_SHAPE;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        MLORA_HIP_TRY(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) {
            set_error("hipGetSymbolAddress returned a null address for the static workspace");
            return MLORA_ERR_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return MLORA_OK;
}

namespace mlora {
// Called by plan creation (the library's set-up call, with the plan's device current): the lookup then never happens
// inside a caller's capture or timed loop.  A failure here is not fatal; multi_lora_bwd_static looks again and reports.
void prepare_static_workspace() {
    void* p = nullptr;
    if (static_workspace(&p) != MLORA_OK) (void)hipGetLastError();
}
}  // namespace mlora

static inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

static int check_flags(uint32_t flags, bool backward) {
    if (flags & ~(MLORA_FLAG_BASE_ONLY | MLORA_FLAG_LORA_ONLY | MLORA_FLAG_GROUP_BANDS | (backward ? MLORA_FLAG_ACCUM_GRADS : 0u))) {
        set_error("unknown flag bits");
        return MLORA_ERR_FLAGS;
    }
    if ((flags & MLORA_FLAG_BASE_ONLY) && (flags & MLORA_FLAG_LORA_ONLY)) {
        set_error("MLORA_FLAG_BASE_ONLY and MLORA_FLAG_LORA_ONLY exclude each other");
        return MLORA_ERR_FLAGS;
    }
    return MLORA_OK;
}

// every adapter with a rank needs its pointers; all of them 16-byte aligned
static int check_ptr_array(const mlora_plan* p, const void* const* arr, const char* name) {
    if (!arr) {
        set_error(std::string(name) + " is NULL");
        return MLORA_ERR_NULL;
    }
    for (int32_t i = 0; i < p->N; ++i) {
        if (p->ranks[i] == 0) continue;
        if (!arr[i]) {
            set_error(std::string(name) + "[i] is NULL for an adapter with rank > 0");
            return MLORA_ERR_NULL;
        }
        if (misaligned(arr[i])) {
            set_error(std::string(name) + "[i] is not 16-byte aligned");
            return MLORA_ERR_ALIGN;
        }
    }
    return MLORA_OK;
}

extern "C" int multi_lora_fwd(mlora_plan* plan, const void* X, const void* W, const void* const* A,
                              const void* const* B, void* Y, void* S, void* workspace, uint32_t flags,
                              void* stream) {
    (void)workspace;
    if (!plan) {
        set_error("plan is NULL");
        return MLORA_ERR_NULL;
    }
    int rc = check_flags(flags, false);
    if (rc != MLORA_OK) return rc;
    const bool lora = !(flags & MLORA_FLAG_BASE_ONLY) && plan->N > 0;
    const bool base = !(flags & MLORA_FLAG_LORA_ONLY);
    if (plan->T > 0 && (!X || !Y || (base && !W))) {
        set_error("X / W / Y is NULL");
        return MLORA_ERR_NULL;
    }
    if (lora && plan->R1 > 0 && !S) {
        set_error("S is NULL");
        return MLORA_ERR_NULL;
    }
    if (misaligned(X) || misaligned(W) || misaligned(Y) || misaligned(S)) {
        set_error("X / W / Y / S must be 16-byte aligned");
        return MLORA_ERR_ALIGN;
    }
    if (lora) {
        if ((rc = check_ptr_array(plan, A, "A")) != MLORA_OK) return rc;
        if ((rc = check_ptr_array(plan, B, "B")) != MLORA_OK) return rc;
    }
    hipStream_t st = (hipStream_t)stream;
    if (lora && (rc = upload_ptrs(plan, A, B, nullptr, nullptr, st)) != MLORA_OK) return rc;
    if (plan->use_mfma) return mfma_forward(plan, X, W, Y, S, flags, st);
    return fma_forward(plan, X, W, Y, S, flags, st);
}

static int bwd_impl(mlora_plan* plan, const void* dY, const void* X, const void* W,
                    const void* const* A, const void* const* B, const void* S, void* dX,
                    void* const* dA, void* const* dB, void* workspace, uint32_t flags,
                    void* stream) {
    if (!plan) {
        set_error("plan is NULL");
        return MLORA_ERR_NULL;
    }
    int rc = check_flags(flags, true);
    if (rc != MLORA_OK) return rc;
    const bool lora = !(flags & MLORA_FLAG_BASE_ONLY) && plan->N > 0;
    const bool base = !(flags & MLORA_FLAG_LORA_ONLY);
    if (plan->T > 0 && (!dY || !dX || (base && !W) || (lora && !X))) {
        set_error("dY / X / W / dX is NULL");
        return MLORA_ERR_NULL;
    }
    if (lora && plan->R1 > 0 && !S) {
        set_error("S is NULL");
        return MLORA_ERR_NULL;
    }
    if (misaligned(dY) || misaligned(X) || misaligned(W) || misaligned(S) || misaligned(dX) ||
        misaligned(workspace)) {
        set_error("dY / X / W / S / dX / workspace must be 16-byte aligned");
        return MLORA_ERR_ALIGN;
    }
    if (lora) {
        if (multi_lora_workspace_bytes(plan) > 0 && !workspace) {
            set_error("workspace is NULL but multi_lora_workspace_bytes(plan) > 0");
            return MLORA_ERR_WORKSPACE;
        }
        if ((rc = check_ptr_array(plan, A, "A")) != MLORA_OK) return rc;
        if ((rc = check_ptr_array(plan, B, "B")) != MLORA_OK) return rc;
        if ((rc = check_ptr_array(plan, (const void* const*)dA, "dA")) != MLORA_OK) return rc;
        if ((rc = check_ptr_array(plan, (const void* const*)dB, "dB")) != MLORA_OK) return rc;
    }
    hipStream_t st = (hipStream_t)stream;
    if (lora && (rc = upload_ptrs(plan, A, B, dA, dB, st)) != MLORA_OK) return rc;
    void* dS = workspace;
    float* partials = workspace ? (float*)((char*)workspace + plan->ws_ds_bytes) : nullptr;
    if (plan->use_mfma) return mfma_backward(plan, dY, X, W, S, dX, dS, partials, flags, st);
    return fma_backward(plan, dY, X, W, S, dX, dS, flags, st);
}

extern "C" int multi_lora_bwd(mlora_plan* plan, const void* dY, const void* X, const void* W,
                              const void* const* A, const void* const* B, const void* S, void* dX,
                              void* const* dA, void* const* dB, void* workspace, uint32_t flags,
                              void* stream) {
    return bwd_impl(plan, dY, X, W, A, B, S, dX, dA, dB, workspace, flags, stream);
}

extern "C" int multi_lora_bwd_static(mlora_plan* plan, const void* dY, const void* X, const void* W,
                                     const void* const* A, const void* const* B, const void* S, void* dX,
                                     void* const* dA, void* const* dB, uint32_t flags, void* stream) {
    if (!plan) {
        set_error("plan is NULL");
        return MLORA_ERR_NULL;
    }
    const size_t need = multi_lora_workspace_bytes(plan);
    if (need > (size_t)MLORA_STATIC_WORKSPACE_BYTES) {
        set_error("multi_lora_bwd_static: the plan needs " + std::to_string(need) + " bytes of workspace, the static workspace holds " +
                  std::to_string((size_t)MLORA_STATIC_WORKSPACE_BYTES) + "; use multi_lora_bwd with a caller-allocated workspace");
        return MLORA_ERR_WORKSPACE;
    }
    void* ws = nullptr;
    const int rc = static_workspace(&ws);
    if (rc != MLORA_OK) return rc;
    // nothing in the workspace has to start at zero: dS is written in full by the gradient shrink before anybody reads it,
    // and every partial weight-gradient block is written by its chunk's work item before the fixed-order sum reads it
    return bwd_impl(plan, dY, X, W, A, B, S, dX, dA, dB, ws, flags, stream);
}

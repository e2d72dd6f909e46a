// Grouped per-adapter AdamW on the LoRA matrices (fp32 state, decoupled weight decay).
//
// The paper keeps one optimizer instance per LoRA job (Sec. 5.2) and trains with AdamW, weight decay
// 0.01, constant learning rate (App., training details).  Here all adapters are updated by one launch:
// the per-adapter pointers and hyper-parameters travel to a device table through kernel arguments,
// then grid.y enumerates (adapter, matrix) pairs and grid.x strides over the elements.  The update is
// a pure stream (28 bytes per bf16 parameter), so it is bound by HBM bandwidth.
#include <cmath>
#include <cstring>

#include "common.h"

namespace mlora {

struct AdamwEntry {
    void* A; void* B;
    const void* dA; const void* dB;
    float* sA; float* sB;
    float lr, beta1, beta2, eps, wd;
    float c1, c2;   // 1 / (1 - beta1^t), 1 / (1 - beta2^t)
    float pad;
};
static_assert(sizeof(AdamwEntry) <= 96, "plan reserves 96 bytes per optimizer entry");

struct AdamwBatch {
    AdamwEntry e[16];
};

__global__ void adamw_upload_kernel(AdamwEntry* dst, AdamwBatch batch, int32_t base, int32_t count) {
    const int32_t i = threadIdx.x;
    if (i < count) dst[base + i] = batch.e[i];
}

template <typename T> __device__ inline float ldp(const T* p);
template <> __device__ inline float ldp<float>(const float* p) { return *p; }
template <> __device__ inline float ldp<uint16_t>(const uint16_t* p) { return __uint_as_float(((uint32_t)*p) << 16); }
template <typename T> __device__ inline void stp(T* p, float v);
template <> __device__ inline void stp<float>(float* p, float v) { *p = v; }
template <> __device__ inline void stp<uint16_t>(uint16_t* p, float v) {
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) { *p = (uint16_t)((u >> 16) | 0x40); return; }
    u += 0x7fffu + ((u >> 16) & 1u);
    *p = (uint16_t)(u >> 16);
}

// INIT: master <- parameter, m = v = 0.  Otherwise one AdamW step.
template <typename T, bool INIT>
__global__ __launch_bounds__(256) void adamw_kernel(const AdamwEntry* __restrict__ table, const int32_t* __restrict__ rank,
                                                    int64_t k, int64_t n) {
    const int32_t i = blockIdx.y >> 1;
    const bool isB = blockIdx.y & 1;
    const int64_t r = rank[i];
    const int64_t numel = isB ? r * n : k * r;
    if (numel == 0) return;
    const AdamwEntry e = table[i];
    T* param = (T*)(isB ? e.B : e.A);
    const T* grad = (const T*)(isB ? e.dB : e.dA);
    float* master = isB ? e.sB : e.sA;
    float* m = master + numel;
    float* v = m + numel;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < numel; idx += stride) {
        if (INIT) {
            master[idx] = ldp<T>(param + idx);
            m[idx] = 0.f;
            v[idx] = 0.f;
        } else {
            const float g = ldp<T>(grad + idx);
            const float mn = e.beta1 * m[idx] + (1.0f - e.beta1) * g;
            const float vn = e.beta2 * v[idx] + (1.0f - e.beta2) * g * g;
            float th = master[idx];
            th = th - e.lr * ((mn * e.c1) / (sqrtf(vn * e.c2) + e.eps) + e.wd * th);
            m[idx] = mn;
            v[idx] = vn;
            master[idx] = th;
            stp<T>(param + idx, th);
        }
    }
}

static bool misaligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) != 0; }

static int run(mlora_plan* p, void* const* A, void* const* B, const void* const* dA, const void* const* dB,
               float* const* sA, float* const* sB, const mlora_adamw_hparams* hp, bool init, hipStream_t st) {
    if (!p) { set_error("plan is NULL"); return MLORA_ERR_NULL; }
    if (p->N == 0) return MLORA_OK;
    if (!A || !B || !sA || !sB || (!init && (!dA || !dB || !hp))) {
        set_error("A / B / dA / dB / stateA / stateB / hp is NULL");
        return MLORA_ERR_NULL;
    }
    for (int32_t i = 0; i < p->N; ++i) {
        if (p->ranks[i] == 0) continue;
        if (!A[i] || !B[i] || !sA[i] || !sB[i] || (!init && (!dA[i] || !dB[i]))) {
            set_error("a pointer of an adapter with rank > 0 is NULL");
            return MLORA_ERR_NULL;
        }
        if (misaligned4(sA[i]) || misaligned4(sB[i])) {
            set_error("optimizer state must be 4-byte aligned");
            return MLORA_ERR_ALIGN;
        }
        if (!init) {
            const mlora_adamw_hparams& h = hp[i];
            if (h.step < 1 || !(h.beta1 >= 0.f && h.beta1 < 1.f) || !(h.beta2 >= 0.f && h.beta2 < 1.f) ||
                !std::isfinite(h.lr) || !std::isfinite(h.eps) || !std::isfinite(h.weight_decay)) {
                set_error("AdamW hyper-parameters out of range (step >= 1, 0 <= beta < 1, finite lr / eps / weight_decay)");
                return MLORA_ERR_SCALE;
            }
        }
    }
    AdamwEntry* table = (AdamwEntry*)p->d_adamw;
    for (int32_t base = 0; base < p->N; base += 16) {
        AdamwBatch batch;
        std::memset(&batch, 0, sizeof(batch));
        const int32_t cnt = (p->N - base) < 16 ? (p->N - base) : 16;
        for (int32_t j = 0; j < cnt; ++j) {
            const int32_t i = base + j;
            AdamwEntry& e = batch.e[j];
            e.A = A[i]; e.B = B[i]; e.sA = sA[i]; e.sB = sB[i];
            if (!init) {
                e.dA = dA[i]; e.dB = dB[i];
                const mlora_adamw_hparams& h = hp[i];
                e.lr = h.lr; e.beta1 = h.beta1; e.beta2 = h.beta2; e.eps = h.eps; e.wd = h.weight_decay;
                e.c1 = (float)(1.0 / (1.0 - std::pow((double)h.beta1, (double)h.step)));
                e.c2 = (float)(1.0 / (1.0 - std::pow((double)h.beta2, (double)h.step)));
            }
        }
        ProfScope prof(p, MLORA_K_OTHER, st);
        hipLaunchKernelGGL(adamw_upload_kernel, dim3(1), dim3(16), 0, st, table, batch, base, cnt);
    }
    const int64_t big = (p->k > p->n ? p->k : p->n) * (int64_t)(p->max_rank > 0 ? p->max_rank : 1);
    int64_t gx = (big + 256 * 4 - 1) / (256 * 4);
    if (gx < 1) gx = 1;
    if (gx > 256) gx = 256;
    const dim3 grid((unsigned)gx, (unsigned)(2 * p->N));
    {
        ProfScope prof(p, MLORA_K_ADAMW, st);
        const bool f32 = p->dtype == MLORA_F32;
        if (init && f32)       hipLaunchKernelGGL((adamw_kernel<float, true>), grid, dim3(256), 0, st, table, p->view.rank, p->k, p->n);
        else if (init)         hipLaunchKernelGGL((adamw_kernel<uint16_t, true>), grid, dim3(256), 0, st, table, p->view.rank, p->k, p->n);
        else if (f32)          hipLaunchKernelGGL((adamw_kernel<float, false>), grid, dim3(256), 0, st, table, p->view.rank, p->k, p->n);
        else                   hipLaunchKernelGGL((adamw_kernel<uint16_t, false>), grid, dim3(256), 0, st, table, p->view.rank, p->k, p->n);
    }
    MLORA_HIP_TRY(hipGetLastError());
    return MLORA_OK;
}

}  // namespace mlora

extern "C" int multi_lora_adamw_init(mlora_plan* plan, const void* const* A, const void* const* B,
                                     float* const* stateA, float* const* stateB, void* stream) {
    return mlora::run(plan, (void* const*)A, (void* const*)B, nullptr, nullptr, stateA, stateB, nullptr, true,
                      (hipStream_t)stream);
}

extern "C" int multi_lora_adamw_step(mlora_plan* plan, void* const* A, void* const* B, const void* const* dA,
                                     const void* const* dB, float* const* stateA, float* const* stateB,
                                     const mlora_adamw_hparams* hp, void* stream) {
    return mlora::run(plan, A, B, dA, dB, stateA, stateB, hp, false, (hipStream_t)stream);
}

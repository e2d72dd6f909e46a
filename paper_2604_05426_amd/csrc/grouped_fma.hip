// Descriptor-driven grouped GEMM on the vector ALUs (fp32 FMA, fp32 accumulate).
//
// Serves fp32 plans and bf16 plans whose k or n is not a multiple of 8.  Every step of
// the layer (paper Sec. 5.1) is one grouped launch whose problems are the adapters'
// diagonal blocks only: S_i = X_i A_i, Y_i += s_i S_i B_i, dS_i = s_i dY_i B_i^T,
// dX_i += dS_i A_i^T, dA_i = X_i^T dS_i, dB_i = s_i S_i^T dY_i; the two frozen-weight
// GEMMs are single-problem launches of the same kernel.  Descriptors are built on the
// device from the plan tables, so a layer call is O(1) launches whatever N is.
#include "common.h"

namespace mlora {

struct GProb {
    const void* A;
    const void* B;
    void* C;
    int64_t lda, ldb, ldc;
    int32_t M, N, K;
    int32_t transA, transB, accumulate;
    float alpha;
    int32_t tile_start;
};
static_assert(sizeof(GProb) <= 128, "descriptor scratch is sized for 128-byte descriptors");

enum FmaOp { OP_SHRINK = 0, OP_EXPAND, OP_DSHRINK, OP_DXLORA, OP_WGRAD_A, OP_WGRAD_B };

constexpr int FT = 64;   // tile edge
constexpr int FK = 16;   // contraction step

struct FmaOperands {
    const void* X;
    const void* dY;
    void* Y;
    void* dX;
    void* S;   // S (fwd out / bwd in)
    void* dS;
    int accum_grads;   // dA_i, dB_i += result
};

template <typename T> __device__ inline float ld(const T* p);
template <> __device__ inline float ld<float>(const float* p) { return *p; }
template <> __device__ inline float ld<uint16_t>(const uint16_t* p) {
    return __uint_as_float(((uint32_t)*p) << 16);
}
template <typename T> __device__ inline void st(T* p, float v);
template <> __device__ inline void st<float>(float* p, float v) { *p = v; }
template <> __device__ inline void st<uint16_t>(uint16_t* p, float v) {
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) { *p = (uint16_t)((u >> 16) | 0x40); return; }  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);   // round to nearest even
    *p = (uint16_t)(u >> 16);
}

// One thread per adapter writes its descriptor; thread 0 then scans the tile counts.
template <typename T>
__global__ void fma_make_probs_kernel(PlanView pv, FmaOperands ops, int op, GProb* probs) {
    const int32_t N = pv.N;
    for (int32_t i = threadIdx.x; i < N; i += blockDim.x) {
        const int64_t row0 = pv.off[i];
        const int32_t Ti = pv.off[i + 1] - pv.off[i];
        const int32_t r = pv.rank[i];
        const float s = pv.scale[i];
        const int64_t so = pv.soff[i];
        const AdapterPtrs ap = pv.ptrs[i];
        GProb g{};
        g.alpha = 1.0f;
        switch (op) {
            case OP_SHRINK:
                g.A = (const T*)ops.X + row0 * pv.k; g.lda = pv.k;
                g.B = ap.A; g.ldb = r;
                g.C = (T*)ops.S + so; g.ldc = r;
                g.M = Ti; g.N = r; g.K = (int32_t)pv.k;
                break;
            case OP_EXPAND:
                g.A = (const T*)ops.S + so; g.lda = r;
                g.B = ap.B; g.ldb = pv.n;
                g.C = (T*)ops.Y + row0 * pv.n; g.ldc = pv.n;
                g.M = Ti; g.N = (int32_t)pv.n; g.K = r; g.alpha = s; g.accumulate = 1;
                break;
            case OP_DSHRINK:
                g.A = (const T*)ops.dY + row0 * pv.n; g.lda = pv.n;
                g.B = ap.B; g.ldb = pv.n; g.transB = 1;
                g.C = (T*)ops.dS + so; g.ldc = r;
                g.M = Ti; g.N = r; g.K = (int32_t)pv.n; g.alpha = s;
                break;
            case OP_DXLORA:
                g.A = (const T*)ops.dS + so; g.lda = r;
                g.B = ap.A; g.ldb = r; g.transB = 1;
                g.C = (T*)ops.dX + row0 * pv.k; g.ldc = pv.k;
                g.M = Ti; g.N = (int32_t)pv.k; g.K = r; g.accumulate = 1;
                break;
            case OP_WGRAD_A:
                g.A = (const T*)ops.X + row0 * pv.k; g.lda = pv.k; g.transA = 1;
                g.B = (const T*)ops.dS + so; g.ldb = r;
                g.C = ap.dA; g.ldc = r;
                g.M = (int32_t)pv.k; g.N = r; g.K = Ti; g.accumulate = ops.accum_grads;
                break;
            case OP_WGRAD_B:
                g.A = (const T*)ops.S + so; g.lda = r; g.transA = 1;
                g.B = (const T*)ops.dY + row0 * pv.n; g.ldb = pv.n;
                g.C = ap.dB; g.ldc = pv.n;
                g.M = r; g.N = (int32_t)pv.n; g.K = Ti; g.alpha = s; g.accumulate = ops.accum_grads;
                break;
        }
        if (r == 0) g.M = 0;   // rank-0 adapters have no LoRA work in any op
        probs[i] = g;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t t = 0;
        for (int32_t i = 0; i < N; ++i) {
            probs[i].tile_start = t;
            t += ((probs[i].M + FT - 1) / FT) * ((probs[i].N + FT - 1) / FT);
        }
        probs[N].tile_start = t;
    }
}

__global__ void fma_single_prob_kernel(GProb g, GProb* probs) {
    if (threadIdx.x == 0) {
        g.tile_start = 0;
        probs[0] = g;
        GProb end{};
        end.tile_start = ((g.M + FT - 1) / FT) * ((g.N + FT - 1) / FT);
        probs[1] = end;
    }
}

template <typename T>
__global__ __launch_bounds__(256) void fma_grouped_gemm_kernel(const GProb* __restrict__ probs, int32_t nprobs) {
    __shared__ float As[FK][FT + 4];
    __shared__ float Bs[FK][FT + 4];
    const int32_t tile = blockIdx.x;
    if (tile >= probs[nprobs].tile_start) return;
    int32_t lo = 0, hi = nprobs;
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if (probs[mid].tile_start <= tile) lo = mid; else hi = mid;
    }
    const GProb g = probs[lo];
    const int32_t local = tile - g.tile_start;
    const int32_t tiles_n = (g.N + FT - 1) / FT;
    const int32_t m0 = (local / tiles_n) * FT;
    const int32_t n0 = (local % tiles_n) * FT;
    const T* A = (const T*)g.A;
    const T* B = (const T*)g.B;
    T* C = (T*)g.C;
    const int tid = threadIdx.x;
    const int ty = tid / 16, tx = tid % 16;
    float acc[4][4] = {};
    for (int32_t k0 = 0; k0 < g.K; k0 += FK) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int idx = tid + 256 * j;
            int m, kk;
            if (g.transA) { m = idx % FT; kk = idx / FT; } else { m = idx / FK; kk = idx % FK; }
            float v = 0.f;
            if (m0 + m < g.M && k0 + kk < g.K)
                v = g.transA ? ld<T>(A + (int64_t)(k0 + kk) * g.lda + (m0 + m))
                             : ld<T>(A + (int64_t)(m0 + m) * g.lda + (k0 + kk));
            As[kk][m] = v;
            int nn, kb;
            if (g.transB) { kb = idx % FK; nn = idx / FK; } else { nn = idx % FT; kb = idx / FT; }
            float w = 0.f;
            if (n0 + nn < g.N && k0 + kb < g.K)
                w = g.transB ? ld<T>(B + (int64_t)(n0 + nn) * g.ldb + (k0 + kb))
                             : ld<T>(B + (int64_t)(k0 + kb) * g.ldb + (n0 + nn));
            Bs[kb][nn] = w;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < FK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int32_t m = m0 + ty * 4 + i;
        if (m >= g.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int32_t nn = n0 + tx * 4 + j;
            if (nn >= g.N) continue;
            T* c = C + (int64_t)m * g.ldc + nn;
            float v = g.alpha * acc[i][j];
            if (g.accumulate) v += ld<T>(c);
            st<T>(c, v);
        }
    }
}

static inline int64_t tiles2(int64_t M, int64_t N) { return ((M + FT - 1) / FT) * ((N + FT - 1) / FT); }

// host-side tile count of one grouped op (same formula as the device scan)
static int64_t grouped_tiles(const mlora_plan* p, int op) {
    int64_t t = 0;
    for (int32_t i = 0; i < p->N; ++i) {
        const int64_t Ti = p->off[i + 1] - p->off[i];
        const int64_t r = p->ranks[i];
        switch (op) {
            case OP_SHRINK: case OP_DSHRINK: t += tiles2(Ti, r); break;
            case OP_EXPAND: t += tiles2(Ti, r > 0 ? p->n : 0); break;
            case OP_DXLORA: t += tiles2(Ti, r > 0 ? p->k : 0); break;
            case OP_WGRAD_A: t += tiles2(p->k, r); break;
            case OP_WGRAD_B: t += tiles2(r, p->n); break;
        }
    }
    return t;
}

template <typename T>
static int run_grouped(mlora_plan* p, const FmaOperands& ops, int op, int slot, hipStream_t st) {
    if (p->N == 0) return MLORA_OK;
    GProb* probs = (GProb*)((char*)p->d_probs + (size_t)128 * ((size_t)slot * (p->N + 1)));
    ProfScope prof(p, MLORA_K_OTHER, st);
    hipLaunchKernelGGL(fma_make_probs_kernel<T>, dim3(1), dim3(256), 0, st, p->view, ops, op, probs);
    const int64_t tiles = grouped_tiles(p, op);
    if (tiles > 0)
        hipLaunchKernelGGL(fma_grouped_gemm_kernel<T>, dim3((unsigned)tiles), dim3(256), 0, st, probs, p->N);
    MLORA_HIP_TRY(hipGetLastError());
    return MLORA_OK;
}

template <typename T>
static int run_single(mlora_plan* p, const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K,
                      int64_t lda, int64_t ldb, int64_t ldc, int transB, hipStream_t st) {
    if (M == 0 || N == 0) return MLORA_OK;
    GProb g{};
    g.A = A; g.B = B; g.C = C; g.lda = lda; g.ldb = ldb; g.ldc = ldc;
    g.M = (int32_t)M; g.N = (int32_t)N; g.K = (int32_t)K; g.transB = transB; g.alpha = 1.0f;
    GProb* probs = (GProb*)((char*)p->d_probs + (size_t)128 * ((size_t)4 * (p->N + 1)));
    ProfScope prof(p, MLORA_K_OTHER, st);
    hipLaunchKernelGGL(fma_single_prob_kernel, dim3(1), dim3(64), 0, st, g, probs);
    hipLaunchKernelGGL(fma_grouped_gemm_kernel<T>, dim3((unsigned)tiles2(M, N)), dim3(256), 0, st, probs, 1);
    MLORA_HIP_TRY(hipGetLastError());
    return MLORA_OK;
}

template <typename T>
static int fwd_t(mlora_plan* p, const void* X, const void* W, void* Y, void* S, uint32_t flags, hipStream_t st) {
    FmaOperands ops{};
    ops.X = X; ops.Y = Y; ops.S = S;
    int rc;
    if (!(flags & MLORA_FLAG_BASE_ONLY))
        if ((rc = run_grouped<T>(p, ops, OP_SHRINK, 0, st)) != MLORA_OK) return rc;
    if (!(flags & MLORA_FLAG_LORA_ONLY))
        if ((rc = run_single<T>(p, X, W, Y, p->T, p->n, p->k, p->k, p->n, p->n, 0, st)) != MLORA_OK) return rc;
    if (!(flags & MLORA_FLAG_BASE_ONLY))
        if ((rc = run_grouped<T>(p, ops, OP_EXPAND, 1, st)) != MLORA_OK) return rc;
    return MLORA_OK;
}

template <typename T>
static int bwd_t(mlora_plan* p, const void* dY, const void* X, const void* W, const void* S, void* dX, void* dS,
                 uint32_t flags, hipStream_t st) {
    FmaOperands ops{};
    ops.X = X; ops.dY = dY; ops.dX = dX; ops.S = const_cast<void*>(S); ops.dS = dS;
    ops.accum_grads = (flags & MLORA_FLAG_ACCUM_GRADS) ? 1 : 0;
    int rc;
    if (!(flags & MLORA_FLAG_BASE_ONLY))
        if ((rc = run_grouped<T>(p, ops, OP_DSHRINK, 0, st)) != MLORA_OK) return rc;
    if (!(flags & MLORA_FLAG_LORA_ONLY))
        if ((rc = run_single<T>(p, dY, W, dX, p->T, p->k, p->n, p->n, p->n, p->k, 1, st)) != MLORA_OK) return rc;
    if (!(flags & MLORA_FLAG_BASE_ONLY)) {
        if ((rc = run_grouped<T>(p, ops, OP_DXLORA, 1, st)) != MLORA_OK) return rc;
        if ((rc = run_grouped<T>(p, ops, OP_WGRAD_A, 2, st)) != MLORA_OK) return rc;
        if ((rc = run_grouped<T>(p, ops, OP_WGRAD_B, 3, st)) != MLORA_OK) return rc;
    }
    return MLORA_OK;
}

int fma_forward(mlora_plan* p, const void* X, const void* W, void* Y, void* S, uint32_t flags, hipStream_t st) {
    return p->dtype == MLORA_F32 ? fwd_t<float>(p, X, W, Y, S, flags, st) : fwd_t<uint16_t>(p, X, W, Y, S, flags, st);
}

int fma_backward(mlora_plan* p, const void* dY, const void* X, const void* W, const void* S, void* dX, void* dS,
                 uint32_t flags, hipStream_t st) {
    return p->dtype == MLORA_F32 ? bwd_t<float>(p, dY, X, W, S, dX, dS, flags, st)
                                 : bwd_t<uint16_t>(p, dY, X, W, S, dX, dS, flags, st);
}

}  // namespace mlora

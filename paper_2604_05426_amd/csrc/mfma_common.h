// Device helpers shared by the bf16 MFMA kernels (gfx950 / CDNA4, 64-wide wavefronts).
#pragma once

#include "common.h"

namespace mlora {

typedef uint16_t u16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf2f(u16 v) { return __uint_as_float(((uint32_t)v) << 16); }

// fp32 -> bf16, round to nearest even, NaN preserved
__device__ __forceinline__ u16 f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u16)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (u16)(u >> 16);
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    return (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16);
}

// v_mfma_f32_32x32x16_bf16:  C[32x32] += A[32x16] * B[16x32].
// Lane l supplies A[row l%32][8*(l/32) .. +7] and B[8*(l/32) .. +7][col l%32];
// it receives C[(i/4)*8 + (l/32)*4 + i%4][l%32] in c[i], i = 0..15.
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// v_mfma_f32_16x16x32_bf16:  C[16x16] += A[16x32] * B[32x16].
// Lane l supplies A[row l%16][8*(l/16) .. +7] and B[8*(l/16) .. +7][col l%16];
// it receives C[4*(l/16) + i][l%16] in c[i], i = 0..3.
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// two fp32 -> packed bf16 with the hardware conversion (round to nearest even)
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
typedef float f32x2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack2hw(float lo, float hi) {
    const f32x2v f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2v));
}

// A pointer the compiler may keep in vector registers although it is the same in every lane, moved to scalar registers.
__device__ __forceinline__ const char* uniform_ptr(const void* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const char*>(((uint64_t)hi << 32) | lo);
}

// Direct global -> LDS load of 16 bytes per lane: lane i's data lands at LDS byte address lds_base + 16 i
// (lds_base is wavefront-uniform).  Issued through inline assembly so that the compiler's wait-count
// insertion does not serialise later LDS reads behind it; the caller waits with an explicit vmcnt and a
// barrier before anybody reads the data.
// The global address is a wavefront-uniform base pointer plus a 32-bit per-lane byte offset.
__device__ __forceinline__ void dma16(unsigned voff, const void* sbase, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_base) : "memory", "m0");
}

// Swizzle key of contraction row k of a [contraction][column] LDS tile that is read with the transposing load
// for 16x16x32 MFMA operands: the eight rows one such read touches per half-wavefront (k, k+1, k+2, k+3 and the
// same plus 8) get eight different keys; rows k and k+4 share one (they belong to different read instructions).
__device__ __forceinline__ int nn_swz(int k) { return (k & 3) | (((k >> 3) & 1) << 2); }

__device__ __forceinline__ bf16x8 lds_read_frag(const u16* p) {
    return *reinterpret_cast<const bf16x8*>(p);
}

// ds_read_b64_tr_b16: within each group of 16 lanes, lane j supplies the address of 4
// consecutive 16-bit elements; lanes 4q..4q+3 together name 16 elements of "row" q
// (q = 0..3), and lane i of the group receives element i of rows 0..3.  Reading a
// row-major [contraction][column] tile this way hands every lane 4 consecutive
// contraction values of one column, which is what the MFMA operands want.
__device__ __forceinline__ s16x4 lds_read_tr(const u16* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4*)(uintptr_t)(uint32_t)(uintptr_t)p);
}

// Two transposing reads (contraction rows r0..r0+3 and r0+4..r0+7) -> one MFMA operand.
__device__ __forceinline__ bf16x8 lds_read_frag_tr(const u16* p_lo, const u16* p_hi) {
    const s16x4 lo = lds_read_tr(p_lo);
    const s16x4 hi = lds_read_tr(p_hi);
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ uint4 zero4() { return make_uint4(0u, 0u, 0u, 0u); }

// 16-byte store / load with the non-temporal hint (data that is written once, or read once, by the kernel)
typedef unsigned int u32x4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_streaming(void* dst, uint4 v) {
    const u32x4v vv = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(vv, reinterpret_cast<u32x4v*>(dst));
}
__device__ __forceinline__ uint4 load_streaming(const void* src) {
    const u32x4v v = __builtin_nontemporal_load(reinterpret_cast<const u32x4v*>(src));
    return make_uint4(v[0], v[1], v[2], v[3]);
}

// 8 consecutive bf16 starting at p; the first `valid` (0..8) are read, the rest are zero.
// `vec_ok` says p is 16-byte aligned (then a full chunk is one 128-bit load).
__device__ __forceinline__ uint4 load_chunk(const u16* p, int valid, bool vec_ok) {
    if (valid >= 8 && vec_ok) return *reinterpret_cast<const uint4*>(p);
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (e < valid) w[e >> 1] |= ((uint32_t)p[e]) << ((e & 1) * 16);
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// Same, with 64-bit pieces when p is 8-byte aligned (ranks that are multiples of 4 but not of 8).  For kernels that load a
// chunk once per work item; the extra paths cost registers in a kernel that loads chunks in its inner loop.
__device__ __forceinline__ uint4 load_chunk_a8(const u16* p, int valid, bool vec_ok) {
    if (valid >= 8 && vec_ok) return *reinterpret_cast<const uint4*>(p);
    if ((reinterpret_cast<uintptr_t>(p) & 7) != 0) return load_chunk(p, valid, false);
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        if (valid >= 4 * h + 4) {
            const uint2 v = *reinterpret_cast<const uint2*>(p + 4 * h);
            w[2 * h] = v.x; w[2 * h + 1] = v.y;
        } else {
#pragma unroll
            for (int e = 4 * h; e < 4 * h + 4; ++e)
                if (e < valid) w[e >> 1] |= ((uint32_t)p[e]) << ((e & 1) * 16);
        }
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}

__device__ __forceinline__ uint4 scale_chunk(uint4 v, float s) {
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float lo = __uint_as_float(w[e] << 16) * s;
        const float hi = __uint_as_float(w[e] & 0xffff0000u) * s;
        w[e] = pack2(lo, hi);
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}

}  // namespace mlora

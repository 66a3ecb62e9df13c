// Device-side helpers shared by the HIP kernels of libems (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ems {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

struct F16 {};   // element-type tags
struct BF16 {};

// D(16x16) += A(16x32) * B(32x16), 16-bit inputs, fp32 accumulate.
// Lane l supplies A[row l%16][k = 8*(l/16)+e] and B[k = 8*(l/16)+e][col l%16],
// e = 0..7, and holds D[row 4*(l/16)+i][col l%16], i = 0..3.
__device__ __forceinline__ f32x4 mfma16x16x32(F16, u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma16x16x32(BF16, u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Two fp32 -> one packed pair of 16-bit floats (round to nearest even), lo in bits 0..15.
__device__ __forceinline__ uint32_t pack2(F16, float lo, float hi) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 v = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ uint32_t pack2(BF16, float lo, float hi) {
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    b2 v = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, v);
}

// Exact widening of one 16-bit pattern.
__device__ __forceinline__ float widen(F16, uint16_t bits) {
    return (float)__builtin_bit_cast(_Float16, bits);
}
__device__ __forceinline__ float widen(BF16, uint16_t bits) {
    return __uint_as_float((uint32_t)bits << 16);
}
// Value of the rounded 16-bit number as fp32 (for hi/lo splitting).
__device__ __forceinline__ float round16(F16, float x) { return (float)(_Float16)x; }
__device__ __forceinline__ float round16(BF16, float x) { return (float)(__bf16)x; }

// (lo16(x), lo16(y)) and (hi16(x), hi16(y)) as packed pairs, x in the low half.
__device__ __forceinline__ uint32_t pair_lo(uint32_t x, uint32_t y) {
    return __builtin_amdgcn_perm(y, x, 0x05040100u);
}
__device__ __forceinline__ uint32_t pair_hi(uint32_t x, uint32_t y) {
    return __builtin_amdgcn_perm(y, x, 0x07060302u);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Load from global memory at (wave-uniform 64-bit base) + (per-lane 32-bit byte offset);
// the explicit global address space lets the compiler emit global_load with a scalar base.
template <typename V>
__device__ __forceinline__ V gload(uint64_t base, uint32_t off) {
    return *reinterpret_cast<const __attribute__((address_space(1))) V*>(base + off);
}

// The same for data that is read exactly once (K/V cache rows, logits): a non-temporal load
// does not displace reusable lines from the caches and streams measurably faster from HBM
// on MI355X (a plain read kernel: ~7.0 TB/s with it, ~6.1 TB/s without).
template <typename V>
__device__ __forceinline__ V gload_stream(uint64_t base, uint32_t off) {
    return __builtin_nontemporal_load(
        reinterpret_cast<const __attribute__((address_space(1))) V*>(base + off));
}

// Reductions over the four lanes {n, n+16, n+32, n+48} that share one MFMA column,
// with the gfx950 row-swap instructions (no LDS round trip): after the 16-lane swap
// the two results hold rows (0,0,2,2) and (1,1,3,3), after the 32-lane swap the lower
// and the upper half of the wave.
__device__ __forceinline__ float quad_max(float x) {
    u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float quad_sum(float x) {
    u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <typename T>
__device__ __forceinline__ T uniform(T v) {   // wave-uniform value -> scalar register
    static_assert(sizeof(T) == 4, "32-bit only");
    return __builtin_bit_cast(T, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, v)));
}
__device__ __forceinline__ uint64_t uniform_addr(const void* p) {
    uint64_t u = (uint64_t)p;
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u);
    uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
    return ((uint64_t)hi << 32) | lo;
}

}  // namespace ems

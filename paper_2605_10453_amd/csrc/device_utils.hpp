// Small device helpers shared by the gfx950 kernels: bf16 unpacking, the
// (logit desc, id asc) order, and wavefront-wide (64-lane) reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace slimspec {

constexpr int kWave = 64;
constexpr float kNegInf = -__builtin_huge_valf();
constexpr int kNoId = 0x7fffffff;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Two bf16 values packed in one 32-bit word (low half = even element).
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint16_t float_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// exp(x) and ln(x) through the hardware base-2 units.
__device__ __forceinline__ float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * kLog2e); }
__device__ __forceinline__ float fast_log(float x) { return __builtin_amdgcn_logf(x) * kLn2; }

// Order of the outputs: larger logit first, equal logits: smaller id first.
__device__ __forceinline__ bool ranks_before(float va, int ia, float vb, int ib) {
    return (va > vb) || (va == vb && ia < ib);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

// Butterfly sum: the same pairing for every lane, so all lanes end with the
// same bits and the result does not depend on timing.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// All lanes receive the (value, id) pair that ranks first among the 64 lanes.
__device__ __forceinline__ void wave_first(float &v, int &i) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        float ov = __shfl_xor(v, off, kWave);
        int oi = __shfl_xor(i, off, kWave);
        if (ranks_before(ov, oi, v, i)) { v = ov; i = oi; }
    }
}

}  // namespace slimspec

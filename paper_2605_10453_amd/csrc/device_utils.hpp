// Small device helpers shared by the gfx950 kernels: bf16 unpacking, the
// (logit desc, id asc) order as a 64-bit key, and wavefront-wide (64-lane)
// reductions built on DPP lane permutes (no LDS traffic, no bpermute latency).
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

// exp(x) and ln(x) through the hardware base-2 units.
__device__ __forceinline__ float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * kLog2e); }
__device__ __forceinline__ float fast_log(float x) { return __builtin_amdgcn_logf(x) * kLn2; }

// The 16-bit row operand of the matrix-core head kernel: t log2(e) rounded to bf16 (nearest even) or to f16.  One
// definition for the kernel that writes the operand and for the merge, which recomputes from it the logit the head
// kernel saw for a column without a recorded value.
__device__ __forceinline__ uint32_t operand_bf16_bits(float t) {
    const uint32_t u = __float_as_uint(t * kLog2e);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ _Float16 operand_f16(float t) { return (_Float16)(t * kLog2e); }
// ... and the value of t it stands for
__device__ __forceinline__ float operand_value(float t, bool as_f16) {
    return (as_f16 ? (float)operand_f16(t) : __uint_as_float(operand_bf16_bits(t) << 16)) * kLn2;
}

// Order of the outputs: larger logit first, equal logits: smaller id first.
__device__ __forceinline__ bool ranks_before(float va, int ia, float vb, int ib) {
    return (va > vb) || (va == vb && ia < ib);
}

// ---------------------------------------------------------------------------
// 64-bit sort key: high word = logit mapped to an unsigned integer with the same
// order (-0 is first turned into +0 so that equal logits give equal words), low
// word = ~tiebreak, so that a larger key ranks first and, among equal logits,
// the smaller tiebreak (vocabulary id or list position) ranks first.
__device__ __forceinline__ uint32_t float_order_bits(float v) {
    uint32_t u = __float_as_uint(v + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float float_from_order_bits(uint32_t o) {
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7fffffffu) : ~o);
}
__device__ __forceinline__ uint64_t make_key(float v, uint32_t tiebreak) {
    return ((uint64_t)float_order_bits(v) << 32) | (uint32_t)~tiebreak;
}
__device__ __forceinline__ float key_value(uint64_t k) { return float_from_order_bits((uint32_t)(k >> 32)); }
__device__ __forceinline__ uint32_t key_tiebreak(uint64_t k) { return ~(uint32_t)k; }
constexpr uint64_t kNoKey = 0;      // ranks after every real key (a real key has a non-zero high word)

// ---------------------------------------------------------------------------
// Lane permutes.  DPP controls: quad_perm [1,0,3,2] = 0xB1 (lane ^ 1), quad_perm
// [2,3,0,1] = 0x4E (lane ^ 2), row_half_mirror = 0x141 (7 - lane within 8),
// row_mirror = 0x140 (15 - lane within 16).  After the first two steps all lanes
// of a quad agree, after the mirrors all lanes of a row of 16 agree; the two
// gfx950 permlane swaps then exchange rows of 16 and halves of 32.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) { return __uint_as_float(dpp_u32<CTRL>(__float_as_uint(x))); }

// value held by the lane 16 (STEP == 16) or 32 (STEP == 32) positions away, xor-wise
template <int STEP>
__device__ __forceinline__ void swap_pair(uint32_t x, uint32_t &a, uint32_t &b) {
    if constexpr (STEP == 16) {
        auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
        a = r[0]; b = r[1];
    } else {
        auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
        a = r[0]; b = r[1];
    }
}

#define SLIMSPEC_WAVE_REDUCE_F32(NAME, OP)                                            \
    __device__ __forceinline__ float NAME(float v) {                                  \
        v = OP(v, dpp_f32<0xB1>(v));                                                  \
        v = OP(v, dpp_f32<0x4E>(v));                                                  \
        v = OP(v, dpp_f32<0x141>(v));                                                 \
        v = OP(v, dpp_f32<0x140>(v));                                                 \
        uint32_t a, b;                                                                \
        swap_pair<16>(__float_as_uint(v), a, b);                                      \
        v = OP(__uint_as_float(a), __uint_as_float(b));                               \
        swap_pair<32>(__float_as_uint(v), a, b);                                      \
        v = OP(__uint_as_float(a), __uint_as_float(b));                               \
        return v;                                                                     \
    }
__device__ __forceinline__ float op_max(float a, float b) { return fmaxf(a, b); }
__device__ __forceinline__ float op_add(float a, float b) { return a + b; }
// Every lane ends with the same bits: each step combines two values that all
// lanes of the group already share, and max / + are commutative bit for bit.
SLIMSPEC_WAVE_REDUCE_F32(wave_max, op_max)
SLIMSPEC_WAVE_REDUCE_F32(wave_sum, op_add)
#undef SLIMSPEC_WAVE_REDUCE_F32

__device__ __forceinline__ uint64_t u64_from(uint32_t hi, uint32_t lo) { return ((uint64_t)hi << 32) | lo; }
__device__ __forceinline__ uint64_t u64_max(uint64_t a, uint64_t b) { return a > b ? a : b; }

// Largest 64-bit key of the wavefront, in every lane.
__device__ __forceinline__ uint64_t wave_max_key(uint64_t k) {
    uint32_t hi = (uint32_t)(k >> 32), lo = (uint32_t)k;
#define SLIMSPEC_STEP(CTRL)                                                           \
    {                                                                                 \
        uint64_t o = u64_from(dpp_u32<CTRL>(hi), dpp_u32<CTRL>(lo));                  \
        k = u64_max(k, o); hi = (uint32_t)(k >> 32); lo = (uint32_t)k;                \
    }
    SLIMSPEC_STEP(0xB1) SLIMSPEC_STEP(0x4E) SLIMSPEC_STEP(0x141) SLIMSPEC_STEP(0x140)
#undef SLIMSPEC_STEP
    uint32_t ha, hb, la, lb;
    swap_pair<16>(hi, ha, hb); swap_pair<16>(lo, la, lb);
    k = u64_max(u64_from(ha, la), u64_from(hb, lb)); hi = (uint32_t)(k >> 32); lo = (uint32_t)k;
    swap_pair<32>(hi, ha, hb); swap_pair<32>(lo, la, lb);
    return u64_max(u64_from(ha, la), u64_from(hb, lb));
}

// ---------------------------------------------------------------------------
// Standard Gumbel noise as a pure function of (seed, row, vocabulary id), for one draw per row from softmax(z) by
// the Gumbel-max rule argmax_v (z_v + g_v) (sampling at temperature 1, section 5.3):
//     x = id * 0x9E3779B1 + row * 0x85EBCA77 + seed_lo;  x = mix(x);  x += seed_hi * 0xC2B2AE3D;  x = mix(x)
//     mix(x): x ^= x >> 16; x *= 0x21F0AAAD; x ^= x >> 15; x *= 0x735A2D97; x ^= x >> 15
//     n = x >> 9,  u = (2 n + 1) / 2^24,  E = -ln(1 - u) ~ Exp(1),  g = -ln E
// The draws that decide a sample are the large ones, i.e. small E = small u: there E comes from the series of
// -ln(1 - u) (the hardware logarithm of a number next to 1 would lose them); elsewhere 1 - u is exact in fp32.
struct GumbelKey { uint32_t row_term, hi_term; };      // row * 0x85EBCA77 + seed_lo,  seed_hi * 0xC2B2AE3D
__device__ __forceinline__ GumbelKey gumbel_key(uint32_t seed_lo, uint32_t seed_hi, uint32_t row) {
    return {row * 0x85EBCA77u + seed_lo, seed_hi * 0xC2B2AE3Du};
}
__device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= 0x21F0AAADu; x ^= x >> 15; x *= 0x735A2D97u; x ^= x >> 15;
    return x;
}
// g / ln 2 (the noise in base-2 units: add it to a logit times log2 e)
__device__ __forceinline__ float gumbel_base2(const GumbelKey &key, uint32_t id) {
    uint32_t x = id * 0x9E3779B1u + key.row_term;
    x = mix32(x);
    x += key.hi_term;
    x = mix32(x);
    const uint32_t m = 2u * (x >> 9) + 1u;                          // u = m / 2^24, m odd, < 2^24
    const float u = (float)m * 5.9604644775390625e-8f;              // exact
    const float series = u * (1.f + u * (0.5f + u * (0.33333334f + u * (0.25f + u * 0.2f))));
    const float direct = -__builtin_amdgcn_logf((float)(16777216u - m) * 5.9604644775390625e-8f) * kLn2;   // 1 - u is exact
    const float E = (m < (1u << 18)) ? series : direct;
    return -__builtin_amdgcn_logf(E);
}

// Orders the shared-memory accesses of one wavefront: writes before it are visible to
// the reads of the other lanes after it (the LDS serves a wavefront's requests in
// order; this keeps the compiler from reordering across the point).
__device__ __forceinline__ void lds_wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace slimspec

// Register-staged MFMA tile loop of the down-projection t = h A for calls with many rows (paper section 4.1).
//
// Orientation.  The weight matrix M is [K, N] row-major (here A: K = d, N = r) and the activations X are
// [rows, K].  The kernel computes the transposed product  Z^T[n, row] = sum_k M[k, n] X[row, k]  with
// v_mfma_f32_32x32x16_bf16: the MFMA "A" operand is a 32 (n) x 16 (k) piece of M^T, the "B" operand a
// 16 (k) x 32 (row) piece of X^T.  In the 32x32 result a lane then owns ONE row (lane % 32) and 16 values of n.
//
// Both operands want, per lane, 8 consecutive k for a fixed n (or row).  M has n contiguous, so its tiles are
// transposed on the way into LDS: a lane loads 8 rows k of 8 adjacent n (eight 128-bit loads), regroups them
// in registers into 8 vectors "8 consecutive k of one n" and writes each vector with one ds_write_b128.
//
// LDS tile layout, in units of 16 bytes (= 8 k-values of one n or one row):
//   M tile  [KB/8 kgroups][8 j][32 g]     vector (kg, j, g) holds n = n0 + 8 g + j
//   X tile  [KB/8 kgroups][XS]            vector (kg, row)
// so MFMA tile j of the 256-wide n tile reads 32 consecutive vectors (lanes 0..31: kgroup 2s,
// lanes 32..63: kgroup 2s + 1, for k-step s), and its result element i of lane l is
//   n = n0 + 8 m + j,  m = 8 (i / 4) + 4 (l / 32) + (i % 4),   row = l % 32.
#pragma once
#include "device_utils.hpp"

namespace slimspec {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kKB = 64;          // k per LDS stage
constexpr int kKG = kKB / 8;     // k-groups of 8 per stage
constexpr int kNT = 256;         // n (vocabulary / rank columns) per tile

// WR x WV wavefronts; a wavefront owns TR row tiles x TV n-tiles of 32 x 32.
template <int WR_, int WV_, int TR_, int TV_>
struct TileCfg {
    static constexpr int WR = WR_, WV = WV_, TR = TR_, TV = TV_;
    static_assert(WV * TV == 8, "the n tile is 8 MFMA tiles wide");
    static constexpr int THREADS = WR * WV * 64;
    static constexpr int RT = WR * TR * 32;                 // rows per tile
    static constexpr int XS = RT + 1;                       // X k-group stride (vectors); odd: spreads banks
    static constexpr int M_VECS = kKG * kNT;                // 2048 vectors = 32 KB
    static constexpr int X_VECS = kKG * XS;
    static constexpr int STAGE_VECS = M_VECS + X_VECS;
    static constexpr int LDS_BYTES = 2 * STAGE_VECS * 16;
    static constexpr int M_TASKS = (kKG * 32) / THREADS;    // (kgroup, g) load tasks per thread
    static_assert(M_TASKS >= 1 && M_TASKS * THREADS == kKG * 32, "thread count must divide 256");
    static constexpr int X_PIECES = (kKG * RT + THREADS - 1) / THREADS;
};

// ---------------------------------------------------------------------------
// M tile: global -> registers (raw bf16 rows) -> LDS (k-contiguous, f16 or bf16).
template <class C>
struct MRegs { uint4 w[C::M_TASKS][8]; };

// Branch-free: addresses past the end of the k range [.., K) or of the columns [.., N) are clamped
// to the last valid group of 8, so every load is in bounds and returns real (finite) weights.
// Clamped k rows meet zero activations (the X tile is zero there); clamped columns are ignored
// by the epilogues.  Straight-line loads let the compiler count outstanding loads exactly, which
// the two-stage-deep prefetch relies on.
// Addresses are formed as (uniform row pointer M + i N) + one 32-bit per-lane offset, so that the
// 8 loads of a task share a single offset register (scalar base + vector offset addressing).
template <class C>
__device__ __forceinline__ void load_m_regs(MRegs<C> &r, const uint16_t *__restrict__ M,
                                            int K, int N, int k0, int n0, int tid)
{
#pragma unroll
    for (int t = 0; t < C::M_TASKS; ++t) {
        const int q = tid + t * C::THREADS;
        const int kg = q >> 5, g = q & 31;
        const int n = min(n0 + g * 8, N - 8);
        const int k = min(k0 + kg * 8, K - 8);
        const uint32_t off = (uint32_t)k * (uint32_t)N + (uint32_t)n;      // < 2^31 elements (K N = d r: checked on the host)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint16_t *row_i = M + (size_t)i * N;                       // uniform
            r.w[t][i] = *reinterpret_cast<const uint4 *>(row_i + off);
        }
    }
}

// 8 rows k (a[0..7]) of one 32-bit column pair -> the two k-contiguous vectors of that pair.
__device__ __forceinline__ void regroup_pair(const uint32_t (&a)[8], uint4 &even, uint4 &odd)
{
    constexpr uint32_t LO = 0x05040100u, HI = 0x07060302u;   // v_perm_b32 byte selectors
    even = make_uint4(__builtin_amdgcn_perm(a[1], a[0], LO), __builtin_amdgcn_perm(a[3], a[2], LO),
                      __builtin_amdgcn_perm(a[5], a[4], LO), __builtin_amdgcn_perm(a[7], a[6], LO));
    odd = make_uint4(__builtin_amdgcn_perm(a[1], a[0], HI), __builtin_amdgcn_perm(a[3], a[2], HI),
                     __builtin_amdgcn_perm(a[5], a[4], HI), __builtin_amdgcn_perm(a[7], a[6], HI));
}

// Quarter PR (0..3) of the regroup-and-store of a loaded M tile: column pair PR of every task.
template <class C, int PR>
__device__ __forceinline__ void store_m_quarter(const MRegs<C> &r, uint4 *__restrict__ m_tile, int tid)
{
#pragma unroll
    for (int t = 0; t < C::M_TASKS; ++t) {
        const int q = tid + t * C::THREADS;
        const int kg = q >> 5, g = q & 31;
        uint4 *dst = m_tile + (kg * 8) * 32 + g;            // + j * 32
        uint32_t a[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint4 &w = r.w[t][i];
            a[i] = PR == 0 ? w.x : PR == 1 ? w.y : PR == 2 ? w.z : w.w;
        }
        uint4 even, odd;
        regroup_pair(a, even, odd);
        dst[(2 * PR) * 32] = even;
        dst[(2 * PR + 1) * 32] = odd;
    }
}

template <class C>
__device__ __forceinline__ void store_m_lds(const MRegs<C> &r, uint4 *__restrict__ m_tile, int tid)
{
    store_m_quarter<C, 0>(r, m_tile, tid);
    store_m_quarter<C, 1>(r, m_tile, tid);
    store_m_quarter<C, 2>(r, m_tile, tid);
    store_m_quarter<C, 3>(r, m_tile, tid);
}

// ---------------------------------------------------------------------------
// X tile: row-major bf16 activations [rows, ldx] (h itself).
template <class C>
struct XRegs { u32x4 w[C::X_PIECES]; };      // native vectors: plain register copies, global -> LDS

// Branch-free: rows past the end are clamped (their results are never used), k >= K reads as zero
// (select after an in-bounds load).
template <class C>
__device__ __forceinline__ void load_x_regs(XRegs<C> &r, const uint16_t *__restrict__ X,
                                            int K, int ldx, int rows, int k0, int row0, int tid)
{
#pragma unroll
    for (int i = 0; i < C::X_PIECES; ++i) {
        const int p = min(tid + i * C::THREADS, kKG * C::RT - 1);
        const int row = min(row0 + (p >> 3), rows - 1), k = k0 + (p & 7) * 8;
        const uint32_t off = (uint32_t)row * (uint32_t)ldx + (uint32_t)min(k, K - 8);
        u32x4 v = *reinterpret_cast<const u32x4 *>(X + off);
        if (k >= K) v = u32x4{0u, 0u, 0u, 0u};
        r.w[i] = v;
    }
}

template <class C>
__device__ __forceinline__ void store_x_lds(const XRegs<C> &r, uint4 *__restrict__ x_tile, int tid)
{
    u32x4 *xt = reinterpret_cast<u32x4 *>(x_tile);
#pragma unroll
    for (int i = 0; i < C::X_PIECES; ++i) {
        const int p = tid + i * C::THREADS;
        if (C::X_PIECES * C::THREADS == kKG * C::RT || p < kKG * C::RT) xt[(p & 7) * C::XS + (p >> 3)] = r.w[i];
    }
}

// ---------------------------------------------------------------------------
// One LDS stage (kKB of k) into the accumulators of this wavefront.
__device__ __forceinline__ void mfma_32x32x16(const uint4 &a, const uint4 &b, f32x16 &c)
{
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

template <class C>
struct Frags { uint4 x[C::TR], m[C::TV]; };

template <class C>
__device__ __forceinline__ void load_frags(Frags<C> &f, const uint4 *__restrict__ m_tile,
                                           const uint4 *__restrict__ x_tile, int s, int wr, int wv, int lane)
{
    const int kg = 2 * s + (lane >> 5), l32 = lane & 31;
#pragma unroll
    for (int rt = 0; rt < C::TR; ++rt) f.x[rt] = x_tile[kg * C::XS + (wr * C::TR + rt) * 32 + l32];
#pragma unroll
    for (int j = 0; j < C::TV; ++j) f.m[j] = m_tile[(kg * 8 + wv * C::TV + j) * 32 + l32];
}

// Operands of k-step s + 1 are read from LDS while the MFMAs of k-step s run; the scheduling
// barriers keep the compiler from hoisting all reads of the stage to the top (which would hold
// four k-steps of operands in registers at once).
//
// `fresh` starts a new accumulation: the first k-step then takes a zero C operand instead of the
// old accumulators.  The accumulators are never written by anything but an MFMA and are read (in
// the epilogues) only through read_acc(), so that the register allocator can keep them in AGPRs
// for the whole kernel instead of copying them in and out of VGPRs around every stage.
template <class C>
__device__ __forceinline__ void mma_stage(f32x16 (&acc)[C::TR][C::TV], const uint4 *__restrict__ m_tile,
                                          const uint4 *__restrict__ x_tile, int wr, int wv, int lane, bool fresh)
{
    constexpr int S = kKB / 16;
    Frags<C> f[2];
    load_frags<C>(f[0], m_tile, x_tile, 0, wr, wv, lane);
    load_frags<C>(f[1], m_tile, x_tile, 1, wr, wv, lane);
    if (fresh) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int rt = 0; rt < C::TR; ++rt)
#pragma unroll
            for (int j = 0; j < C::TV; ++j) { acc[rt][j] = zero; mfma_32x32x16(f[0].m[j], f[0].x[rt], acc[rt][j]); }
    } else {
#pragma unroll
        for (int rt = 0; rt < C::TR; ++rt)
#pragma unroll
            for (int j = 0; j < C::TV; ++j) mfma_32x32x16(f[0].m[j], f[0].x[rt], acc[rt][j]);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 1; s < S; ++s) {
        if (s + 1 < S) load_frags<C>(f[(s + 1) & 1], m_tile, x_tile, s + 1, wr, wv, lane);
#pragma unroll
        for (int rt = 0; rt < C::TR; ++rt)
#pragma unroll
            for (int j = 0; j < C::TV; ++j) mfma_32x32x16(f[s & 1].m[j], f[s & 1].x[rt], acc[rt][j]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// one accumulator element, read straight from its AGPR
__device__ __forceinline__ float read_acc(const float &a) {
    float v;
    asm("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
    return v;
}

// n offset (inside the 256-wide tile) of result element i of MFMA tile j, for a lane in half `half`
__device__ __forceinline__ int tile_n_offset(int j, int i, int half) {
    return 8 * (8 * (i >> 2) + 4 * half + (i & 3)) + j;
}

}  // namespace slimspec

// Matrix-core building blocks for calls with many rows (paper section 4.1: the two dense
// products of the low-rank head, t = h A and z = t B, and the full head z = h W).
//
// Orientation.  The weight matrix M is [K, N] row-major (A: K = d, N = r;  B: K = r, N = V;
// W: K = d, N = V) and the activations X are [rows, K].  The kernels compute the transposed
// product  Z^T[n, row] = sum_k M[k, n] X[row, k]  with v_mfma_f32_32x32x16_{f16,bf16}:
// the MFMA "A" operand is a 32 (n) x 16 (k) piece of M^T, the "B" operand a 16 (k) x 32 (row)
// piece of X^T.  In the 32x32 result a lane then owns ONE row (lane % 32) and 16 values of n,
// so everything that is reduced per row (running max, sum of exp, top-k) stays inside a lane.
//
// Both operands want, per lane, 8 consecutive k for a fixed n (or row).  M has n contiguous, so
// its tiles are transposed on the way into LDS: a lane loads 8 rows k of 8 adjacent n (eight
// 128-bit loads), regroups them in registers into 8 vectors "8 consecutive k of one n" (the
// bf16 -> f16 conversion of the low-rank head happens in the same step) and writes each vector
// with one ds_write_b128.
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
        const uint32_t off = (uint32_t)k * (uint32_t)N + (uint32_t)n;      // < 2^31 elements (checked on the host)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint16_t *row_i = M + (size_t)i * N;                       // uniform
            r.w[t][i] = *reinterpret_cast<const uint4 *>(row_i + off);
        }
    }
}

__device__ __forceinline__ uint32_t pack_f16_from_bf16_lo(uint32_t a, uint32_t b) {
    auto h = __builtin_amdgcn_cvt_pkrtz(__uint_as_float(a << 16), __uint_as_float(b << 16));
    return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ uint32_t pack_f16_from_bf16_hi(uint32_t a, uint32_t b) {
    auto h = __builtin_amdgcn_cvt_pkrtz(__uint_as_float(a & 0xffff0000u), __uint_as_float(b & 0xffff0000u));
    return __builtin_bit_cast(uint32_t, h);
}

// 8 rows k (a[0..7]) of one 32-bit column pair -> the two k-contiguous vectors of that pair.
template <bool F16>
__device__ __forceinline__ void regroup_pair(const uint32_t (&a)[8], uint4 &even, uint4 &odd)
{
    if constexpr (F16) {
        // every finite bf16 in the f16 range converts exactly (8 significand bits fit in 11)
        even = make_uint4(pack_f16_from_bf16_lo(a[0], a[1]), pack_f16_from_bf16_lo(a[2], a[3]),
                          pack_f16_from_bf16_lo(a[4], a[5]), pack_f16_from_bf16_lo(a[6], a[7]));
        odd = make_uint4(pack_f16_from_bf16_hi(a[0], a[1]), pack_f16_from_bf16_hi(a[2], a[3]),
                         pack_f16_from_bf16_hi(a[4], a[5]), pack_f16_from_bf16_hi(a[6], a[7]));
    } else {
        constexpr uint32_t LO = 0x05040100u, HI = 0x07060302u;   // v_perm_b32 byte selectors
        even = make_uint4(__builtin_amdgcn_perm(a[1], a[0], LO), __builtin_amdgcn_perm(a[3], a[2], LO),
                          __builtin_amdgcn_perm(a[5], a[4], LO), __builtin_amdgcn_perm(a[7], a[6], LO));
        odd = make_uint4(__builtin_amdgcn_perm(a[1], a[0], HI), __builtin_amdgcn_perm(a[3], a[2], HI),
                         __builtin_amdgcn_perm(a[5], a[4], HI), __builtin_amdgcn_perm(a[7], a[6], HI));
    }
}

// Quarter PR (0..3) of the regroup-and-store of a loaded M tile: column pair PR of every task.
template <class C, bool F16, int PR>
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
        regroup_pair<F16>(a, even, odd);
        dst[(2 * PR) * 32] = even;
        dst[(2 * PR + 1) * 32] = odd;
    }
}

template <class C, bool F16>
__device__ __forceinline__ void store_m_lds(const MRegs<C> &r, uint4 *__restrict__ m_tile, int tid)
{
    store_m_quarter<C, F16, 0>(r, m_tile, tid);
    store_m_quarter<C, F16, 1>(r, m_tile, tid);
    store_m_quarter<C, F16, 2>(r, m_tile, tid);
    store_m_quarter<C, F16, 3>(r, m_tile, tid);
}

// ---------------------------------------------------------------------------
// X tile.  Two sources: the k-grouped scratch layout [K/8][rows_pad] of 16-byte vectors written
// by the down-projection (straight copy), or row-major bf16 activations [rows, K] (h itself).
template <class C>
struct XRegs { u32x4 w[C::X_PIECES]; };      // native vectors: plain register copies, global -> LDS

// Branch-free.  Row-major X [rows, ldx] (bf16 activations): rows past the end are clamped (their
// results are never used), k >= K reads as zero (select after an in-bounds load).  k-grouped X
// (the f16 scratch [Kpad / 8][rows_pad] written by the down-projection) is zero-padded to a
// multiple of kKB in k and to rows_pad rows, so it needs no guard at all.
template <class C, bool ROW_MAJOR>
__device__ __forceinline__ void load_x_regs(XRegs<C> &r, const uint16_t *__restrict__ X,
                                            int K, int ldx, int rows, int rows_pad, int k0, int row0, int tid)
{
    if constexpr (ROW_MAJOR) {
#pragma unroll
        for (int i = 0; i < C::X_PIECES; ++i) {
            const int p = min(tid + i * C::THREADS, kKG * C::RT - 1);
            const int row = min(row0 + (p >> 3), rows - 1), k = k0 + (p & 7) * 8;
            const uint32_t off = (uint32_t)row * (uint32_t)ldx + (uint32_t)min(k, K - 8);
            u32x4 v = *reinterpret_cast<const u32x4 *>(X + off);
            if (k >= K) v = u32x4{0u, 0u, 0u, 0u};
            r.w[i] = v;
        }
    } else {
        // piece p = tid + i THREADS -> (k-group p / RT, row p % RT); THREADS is a multiple or a divisor of RT,
        // so consecutive pieces of a thread differ by a uniform stride: one per-lane offset register
        static_assert(C::THREADS % C::RT == 0 || C::RT % C::THREADS == 0, "piece stride must be uniform");
        const int p0 = min(tid, kKG * C::RT - 1);
        const uint32_t off = ((uint32_t)((k0 >> 3) + p0 / C::RT) * (uint32_t)rows_pad + (uint32_t)(row0 + p0 % C::RT)) * 8u;
#pragma unroll
        for (int i = 0; i < C::X_PIECES; ++i) {
            const size_t step = (C::THREADS >= C::RT)
                ? (size_t)i * (C::THREADS / C::RT) * rows_pad * 8                  // whole k-groups further
                : (size_t)((i * C::THREADS) / C::RT) * rows_pad * 8 + (size_t)((i * C::THREADS) % C::RT) * 8;
            r.w[i] = *reinterpret_cast<const u32x4 *>(X + step + off);
        }
    }
}

// piece I of the X tile into LDS
template <class C, bool ROW_MAJOR, int I>
__device__ __forceinline__ void store_x_piece(const XRegs<C> &r, uint4 *__restrict__ x_tile, int tid)
{
    if constexpr (I < C::X_PIECES) {
        const int p = tid + I * C::THREADS;
        if (C::X_PIECES * C::THREADS == kKG * C::RT || p < kKG * C::RT) {
            u32x4 *xt = reinterpret_cast<u32x4 *>(x_tile);
            if constexpr (ROW_MAJOR) xt[(p & 7) * C::XS + (p >> 3)] = r.w[I];
            else xt[(p / C::RT) * C::XS + p % C::RT] = r.w[I];
        }
    }
}

template <class C, bool ROW_MAJOR>
__device__ __forceinline__ void store_x_lds(const XRegs<C> &r, uint4 *__restrict__ x_tile, int tid)
{
    static_assert(C::X_PIECES <= 8, "piece count");
    store_x_piece<C, ROW_MAJOR, 0>(r, x_tile, tid); store_x_piece<C, ROW_MAJOR, 1>(r, x_tile, tid);
    store_x_piece<C, ROW_MAJOR, 2>(r, x_tile, tid); store_x_piece<C, ROW_MAJOR, 3>(r, x_tile, tid);
    store_x_piece<C, ROW_MAJOR, 4>(r, x_tile, tid); store_x_piece<C, ROW_MAJOR, 5>(r, x_tile, tid);
    store_x_piece<C, ROW_MAJOR, 6>(r, x_tile, tid); store_x_piece<C, ROW_MAJOR, 7>(r, x_tile, tid);
}

// ---------------------------------------------------------------------------
// One LDS stage (kKB of k) into the accumulators of this wavefront.
template <bool F16>
__device__ __forceinline__ void mfma_32x32x16(const uint4 &a, const uint4 &b, f32x16 &c)
{
    if constexpr (F16)
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
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
template <class C, bool F16>
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
            for (int j = 0; j < C::TV; ++j) { acc[rt][j] = zero; mfma_32x32x16<F16>(f[0].m[j], f[0].x[rt], acc[rt][j]); }
    } else {
#pragma unroll
        for (int rt = 0; rt < C::TR; ++rt)
#pragma unroll
            for (int j = 0; j < C::TV; ++j) mfma_32x32x16<F16>(f[0].m[j], f[0].x[rt], acc[rt][j]);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 1; s < S; ++s) {
        if (s + 1 < S) load_frags<C>(f[(s + 1) & 1], m_tile, x_tile, s + 1, wr, wv, lane);
#pragma unroll
        for (int rt = 0; rt < C::TR; ++rt)
#pragma unroll
            for (int j = 0; j < C::TV; ++j) mfma_32x32x16<F16>(f[s & 1].m[j], f[s & 1].x[rt], acc[rt][j]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Scheduling request for one k-step: after every MFMA, one LDS read (operands of the next k-step)
// and a few VALU instructions (the conversion), then the LDS writes.  A wavefront issues in order,
// so the conversion only overlaps the matrix cores if it sits between the MFMAs in program order.
template <int NMFMA>
__device__ __forceinline__ void interleave_hint() {
#pragma unroll
    for (int i = 0; i < NMFMA; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);      // DS read
        __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);      // VALU
    }
    __builtin_amdgcn_sched_group_barrier(0x200, 8, 0);          // DS write
}

// The same stage, with the regroup-and-store of the NEXT stage's tiles (already in registers)
// spread over its four k-steps: the matrix cores work through the MFMAs of a k-step while the
// wavefront issues one quarter of the M conversion, its LDS writes and a share of the X writes.
template <class C, bool F16, bool XROW>
__device__ __forceinline__ void mma_stage_and_store(f32x16 (&acc)[C::TR][C::TV], const uint4 *__restrict__ m_tile,
                                                    const uint4 *__restrict__ x_tile, int wr, int wv, int lane,
                                                    const MRegs<C> &next_m, const XRegs<C> &next_x,
                                                    uint4 *__restrict__ next_m_tile, uint4 *__restrict__ next_x_tile, int tid)
{
    static_assert(kKB / 16 == 4, "four k-steps, four quarters");
    Frags<C> f[2];
    load_frags<C>(f[0], m_tile, x_tile, 0, wr, wv, lane);
#define SLIMSPEC_KSTEP(S)                                                                               \
    if (S + 1 < 4) load_frags<C>(f[(S + 1) & 1], m_tile, x_tile, S + 1, wr, wv, lane);                  \
    _Pragma("unroll") for (int rt = 0; rt < C::TR; ++rt)                                                \
        _Pragma("unroll") for (int j = 0; j < C::TV; ++j)                                               \
            mfma_32x32x16<F16>(f[S & 1].m[j], f[S & 1].x[rt], acc[rt][j]);                              \
    store_m_quarter<C, F16, S>(next_m, next_m_tile, tid);                                               \
    store_x_piece<C, XROW, S>(next_x, next_x_tile, tid);                                                \
    store_x_piece<C, XROW, S + 4>(next_x, next_x_tile, tid);                                            \
    interleave_hint<C::TR * C::TV>();                                                                   \
    __builtin_amdgcn_sched_barrier(0);
    SLIMSPEC_KSTEP(0) SLIMSPEC_KSTEP(1) SLIMSPEC_KSTEP(2) SLIMSPEC_KSTEP(3)
#undef SLIMSPEC_KSTEP
}

// Accumulators are zeroed in place in their AGPRs (an inline-asm write keeps them in the AGPR class,
// like read_acc below).
template <int TR, int TV>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[TR][TV]) {
#pragma unroll
    for (int rt = 0; rt < TR; ++rt)
#pragma unroll
        for (int j = 0; j < TV; ++j)
#pragma unroll
            for (int i = 0; i < 16; ++i) asm volatile("v_accvgpr_write_b32 %0, 0" : "=a"(acc[rt][j][i]));
}

// one accumulator element, read straight from its AGPR
__device__ __forceinline__ float read_acc(const float &a) {
    float v;
    asm("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
    return v;
}

// Block-wide barrier that orders LDS traffic only: global loads in flight (the register prefetch
// of later stages) are not waited for.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// n offset (inside the 256-wide tile) of result element i of MFMA tile j, for a lane in half `half`
__device__ __forceinline__ int tile_n_offset(int j, int i, int half) {
    return 8 * (8 * (i >> 2) + 4 * half + (i & 3)) + j;
}

}  // namespace slimspec

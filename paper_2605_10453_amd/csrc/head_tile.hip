// Vocabulary-tiled up-projection on the matrix cores with the fused log-sum-exp / top-k epilogue
// (paper section 4.1: logits = t B, or h W for the full head, never written to memory), for calls with many rows.
//
// Shape of the kernel
//   * A wavefront owns 64 rows x 128 columns of logits = 2 x 4 MFMA tiles of 32 x 32
//     (v_mfma_f32_32x32x16_bf16, accumulators in VGPRs), two wavefronts per SIMD.
//     WR = 4: one block of 8 wavefronts = 256 rows x 256 columns per CU (least traffic per MFMA);
//     WR = 2: blocks of 4 wavefronts = 128 rows x 256 columns, two per CU (calls with few rows).
//   * The transposed product z^T = M^T x^T is computed, so that the 16 values an MFMA tile gives a
//     lane belong to ONE row: running max, sum of exp and candidate bookkeeping stay inside the lane.
//   * Stages of 32 contraction elements travel global memory -> LDS without passing registers
//     (global_load_lds_dwordx4): the M tile row-major as it lies in memory, the X tile as 16-byte
//     vectors of 8 consecutive contraction elements.  NBUF stage buffers; loads are issued
//     NBUF - 1 stages ahead.  MFMA operands come from LDS with ds_read_b64_tr_b16 (M: transposes
//     the row-major tile into 4 consecutive contraction elements per lane) and ds_read_b128 (X).
//   * 16-byte pieces of an M row are stored XOR-swizzled by (k mod 4) so that the four rows a
//     transposing read touches fall into different banks.
//   * X arrives multiplied by log2(e) and the accumulators of a tile start at minus the row's
//     running maximum, so that the epilogue's 2^v needs no multiply or subtract.  The full head (z = h W)
//     runs the same kernel on h itself (NAT): natural-log units, one multiply per exponential.
//
// Waits: the compiler does not see the direct-to-LDS loads (inline asm), so the kernel counts them
// itself: every wavefront issues exactly LPS per stage, vector memory returns in order, hence
// s_waitcnt vmcnt((NBUF - 2) LPS) = "the stage needed next has landed".  No other vector memory
// instruction may sit inside the main loop: the kernel must not spill.
#include "head_stream.hpp"
#include "launch.hpp"
#include <type_traits>

namespace slimspec {

namespace {

constexpr int kTKB = 32;                                   // contraction elements per stage
constexpr int kTNT = 256;                                  // vocabulary columns per tile
constexpr int kTMBytes = kTKB * kTNT * 2;                  // 16 KB of M per stage

template <int WR>
struct TileShape {
    static constexpr int NW = 2 * WR;                      // wavefronts per block
    static constexpr int RT = 64 * WR;                     // rows per block
    static constexpr int XBYTES = (kTKB / 8) * RT * 16;
    static constexpr int STAGE = kTMBytes + XBYTES;
    static constexpr int NBUF = WR == 4 ? 4 : 3;
    static constexpr int LDS = NBUF * STAGE;               // WR 4: 128 KB (one block per CU); WR 2: 72 KB (two)
    static constexpr int MPW = 16 / NW;                    // M loads per wavefront and stage (2 rows each)
    static constexpr int LPS = MPW + 2;                    // loads per wavefront and stage
    static constexpr int WAIT = (NBUF - 2) * LPS;
};

typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define LDS_PTR(T, byte_addr) ((__attribute__((address_space(3))) T *)(uintptr_t)(byte_addr))

// 16 bytes per lane, global memory -> LDS at buf + OFF + 16 * lane (buf uniform)
template <int OFF>
__device__ __forceinline__ void dma16(uint32_t buf, uint32_t voff, const void *base) {
    asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(buf), "v"(voff), "s"(base), "n"(OFF) : "memory", "scc");
}
// the lane number, recomputed wherever it is used (volatile: not hoisted into a long-lived register)
__device__ __forceinline__ uint32_t lane_id_now() {
    uint32_t l;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
    return l;
}
// Two bf16 values -> the same two values in f16 (exact for magnitudes in [2^-14, 65504]; smaller ones become
// f16 subnormals with an absolute error below 2^-25, larger ones infinities, which the merge answers with its
// exhaustive exact pass).  Plain 32-bit VALU instructions: packed 16-bit arithmetic does not overlap with MFMAs.
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t b) {
    typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
    const f16x2_t h = __builtin_bit_cast(f16x2_t, __builtin_amdgcn_cvt_pkrtz(__uint_as_float(b << 16), __uint_as_float(b & 0xffff0000u)));
    return __builtin_bit_cast(uint32_t, h);
}
template <int N>
__device__ __forceinline__ void wait_loads() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }

}  // namespace

// X: [8 ceil(K / 64)][rows_pad] 16-byte vectors: 8 consecutive contraction elements of one row, zero beyond K and
//    beyond the last row; rows_pad a multiple of 64 WR.  NAT = false: the contraction input times log2(e), bf16
//    (F16: f16): logits come out in base-2 units.  NAT = true: the bf16 input itself (full head): natural units.
// M: [K][V] bf16 row-major, V and K multiples of 8
// part: [rows][gw * hg.spb][3 + 3 L] stream records (values in base-2 units): hg.spb = 4, 2 or 1 per row and block
// DBG != 0 (experiment builds only, -DSLIMSPEC_DIAG_DBG=n): timing experiments (1 no epilogue, 2 loads only, 3 no loads);
// their results are meaningless
// SAMPLE: every lane also keeps, per row, the largest logit + Gumbel noise it has seen (Gumbel-max sampling with the
//         seed in `sd`; the noise's row index is sd.row_base + the row of this launch); records then have 20 floats:
//         [12] the largest sum (in the record's units), [13] its id, [14] the second largest, [15] its id,
//         [16] the third largest, [17..19] unused.
struct SampleSeed { uint32_t seed_lo, seed_hi; int row_base; };

template <int L, int WR, bool F16, bool NAT, int DBG, bool SAMPLE>
__global__ __launch_bounds__(128 * WR, 2) void head_tile_kernel(
    const uint4 *__restrict__ X, const uint16_t *__restrict__ M, float *__restrict__ part,
    int rows, int rows_pad, int K, int V, HeadGrid hg, SampleSeed sd)
{
    using S = TileShape<WR>;
    extern __shared__ __align__(1024) unsigned char lds_raw[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) unsigned char *)lds_raw);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, wv = wave & 1;
    const int half = lane >> 5, l32 = lane & 31, g1 = (lane >> 4) & 1, j16 = lane & 15;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int rb = slot % hg.n_rb, col = (slot / hg.n_rb) * 8 + xcd;
    const int row0 = rb * S::RT;
    const int nkb = (K + kTKB - 1) / kTKB;
    const int njobs = (col < hg.n_vt) ? (hg.n_vt - col + hg.gw - 1) / hg.gw : 0;
    const int total = njobs * nkb;
    const bool ktail = (K & (kTKB - 1)) != 0;

    // ---- direct-to-LDS loads of one stage.
    // M load uu of this wavefront covers stage rows 2 MPW wave + 2 uu + (lane >> 5); lane -> stored piece
    // lane & 31, which holds source piece (lane & 31) ^ ((row & 3) << 2).
    const uint32_t rowb = (uint32_t)V * 2u;                    // bytes per row of M
    uint32_t mv[2];                                            // lane offsets from the row pair's first row (even / odd pair)
    const auto set_tile = [&](int vt) {
        // once per tile: recomputed from the lane number rather than kept in registers through the main loop
        const uint32_t ln = lane_id_now();
        const uint32_t kp = ln >> 5, pp = ln & 31;
        const uint32_t mcol_e = (pp ^ (kp << 2)) * 16u;        // source byte column when (row & 3) = kp
        const uint32_t mcol_o = (pp ^ ((2u + kp) << 2)) * 16u; // ... when (row & 3) = 2 + kp
        const uint32_t climit = (uint32_t)(V - vt * kTNT - 8) * 2u;      // last 16-byte piece of the row that exists
        mv[0] = kp * rowb + min(mcol_e, climit);
        mv[1] = (kp + 2u) * rowb + min(mcol_o, climit);
    };
    const uint32_t xv0 = (uint32_t)lane * 16u;
    constexpr int RPW = 2 * S::MPW;                            // stage rows of M per wavefront
    const int xi = 2 * wave;                                   // X loads xi, xi + 1: k-group xi / WR, rows 64 (xi % WR) ...
    const unsigned char *const m_wave = reinterpret_cast<const unsigned char *>(M) + (size_t)(RPW * wave) * rowb;
    const unsigned char *const x_wave =
        reinterpret_cast<const unsigned char *>(X + (size_t)(xi / WR) * rows_pad + row0 + 64 * (xi % WR));
    const size_t m_step = (size_t)kTKB * rowb, x_step = (size_t)4 * rows_pad * 16;
    const uint32_t m_lds = (uint32_t)(wave * RPW * 512);
    const uint32_t x_lds = (uint32_t)(kTMBytes + ((xi / WR) * S::RT + 64 * (xi % WR)) * 16);

    // position of the stage whose loads are issued next
    int a_vt = col, a_kb = 0;
    const unsigned char *mptr = m_wave + (size_t)col * kTNT * 2, *xptr = x_wave;
    const auto issue_stage = [&](uint32_t buf) {
        const uint32_t mb = buf + m_lds;
        if (ktail && a_kb == nkb - 1) {
            // last, partial k-block: rows beyond K are read from rows K - 2, K - 1 (they meet zeros of X)
            const uint32_t ce = mv[0], co = mv[1] - 2u * rowb;
            const unsigned char *tile0 = reinterpret_cast<const unsigned char *>(M) + (size_t)a_vt * kTNT * 2;
            const int k0 = a_kb * kTKB + RPW * wave;
            dma16<0>(mb, ce, tile0 + (size_t)min(k0, K - 2) * rowb);
            dma16<1024>(mb, co, tile0 + (size_t)min(k0 + 2, K - 2) * rowb);
            if (S::MPW == 4) {
                dma16<2048>(mb, ce, tile0 + (size_t)min(k0 + 4, K - 2) * rowb);
                dma16<3072>(mb, co, tile0 + (size_t)min(k0 + 6, K - 2) * rowb);
            }
        } else {
            dma16<0>(mb, mv[0], mptr);
            dma16<1024>(mb, mv[1], mptr);
            if (S::MPW == 4) {
                const unsigned char *mptr4 = mptr + 4 * (size_t)rowb;
                dma16<2048>(mb, mv[0], mptr4);
                dma16<3072>(mb, mv[1], mptr4);
            }
        }
        const uint32_t xb = buf + x_lds;
        dma16<0>(xb, xv0, xptr);
        dma16<1024>(xb, xv0, xptr + 1024);
    };
    const auto advance_ahead = [&]() {
        if (++a_kb == nkb) {
            a_kb = 0; a_vt += hg.gw;
            mptr = m_wave + (size_t)a_vt * kTNT * 2; xptr = x_wave;
            set_tile(a_vt);
        } else { mptr += m_step; xptr += x_step; }
    };

    // ---- operand addresses inside a stage
    const uint32_t xa = (uint32_t)(kTMBytes + (half * S::RT + wr * 64 + l32) * 16);
    // M fragment of MFMA tile jj: ma0 ^ (jj << 6) (the swizzle exchanges 64-byte groups; stage buffers are 1 KB aligned)
    const uint32_t ma0 = (uint32_t)((8 * half + (j16 >> 2)) * 512
                                    + (wv * 16 + 4 * (j16 >> 2) + 2 * g1 + ((j16 & 3) >> 1)) * 16 + (j16 & 1) * 8);

    Stream<L> st[2];
    stream_init(st[0]);
    stream_init(st[1]);
    SampleTrack smp[2];
    sample_init(smp[0]);
    sample_init(smp[1]);
    f32x16 acc[2][4];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[rt][jj][i] = 0.f;

    const long long dbg_t0 = DBG ? clock64() : 0, dbg_w0 = DBG ? wall_clock64() : 0;
    if (total > 0) {
        int c_vt = col, c_kb = 0;                                         // stage being multiplied
        uint32_t buf_cur = lds0, buf_ahead = lds0;
        const auto next_buf = [&](uint32_t b) { return (b + S::STAGE == lds0 + S::LDS) ? lds0 : b + S::STAGE; };
        set_tile(col);
        issue_stage(buf_ahead);                                           // stage 0
#pragma unroll
        for (int pre = 1; pre < S::NBUF - 1; ++pre) {                     // stages 1 .. NBUF - 2 (past the end: the last stage once more)
            if (pre < total) advance_ahead();
            buf_ahead = next_buf(buf_ahead);
            issue_stage(buf_ahead);
        }
        wait_loads<S::WAIT>();
        // F16: every wavefront turns the part of the M tile that it loaded itself (so no barrier is needed before)
        // from bf16 into f16, in place; the barrier that publishes the stage comes after.
        const uint32_t own_m = m_lds + (uint32_t)lane * 16u;
        u32x4 raw[S::MPW];
        const auto read_own = [&](uint32_t buf) {
#pragma unroll
            for (int u = 0; u < S::MPW; ++u) raw[u] = *LDS_PTR(u32x4, buf + own_m + u * 1024);
        };
        const auto convert_own = [&](uint32_t buf) {
#pragma unroll
            for (int u = 0; u < S::MPW; ++u) {
                u32x4 c;
#pragma unroll
                for (int e = 0; e < 4; ++e) c[e] = bf16x2_to_f16x2(raw[u][e]);
                *LDS_PTR(u32x4, buf + own_m + u * 1024) = c;
            }
        };
        if (F16) {
            read_own(buf_cur);
            convert_own(buf_cur);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        __builtin_amdgcn_s_barrier();

        // Operand reads run one k-step (8 MFMAs) ahead of their use, also across stages: the barrier that
        // publishes the next stage sits between the two k-steps of the current one.
        u32x4 xf[2][2], mf[2][4];                                         // [k-step][tile], 8 16-bit values each
        const auto read_operands = [&](uint32_t buf, auto ks_tag) {
            constexpr int ks = decltype(ks_tag)::value;
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
                xf[ks][rt] = *LDS_PTR(u32x4, buf + xa + ks * (2 * S::RT * 16) + rt * 512);
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const uint32_t mj = (buf + ma0) ^ (uint32_t)(jj << 6);
                const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4i16, mj + ks * 8192));
                const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4i16, mj + ks * 8192 + 2048));
                mf[ks][jj] = __builtin_bit_cast(u32x4, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            }
        };
        const auto multiply = [&](auto ks_tag) {
            constexpr int ks = decltype(ks_tag)::value;
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    acc[rt][jj] = F16 ? __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, mf[ks][jj]), __builtin_bit_cast(f16x8, xf[ks][rt]), acc[rt][jj], 0, 0, 0)
                                      : __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, mf[ks][jj]), __builtin_bit_cast(bf16x8, xf[ks][rt]), acc[rt][jj], 0, 0, 0);
        };
        const auto multiply_rows = [&](auto ks_tag, auto rt_tag) {        // one row tile of a k-step: 4 MFMAs
            constexpr int ks = decltype(ks_tag)::value, rt = decltype(rt_tag)::value;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                acc[rt][jj] = F16 ? __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, mf[ks][jj]), __builtin_bit_cast(f16x8, xf[ks][rt]), acc[rt][jj], 0, 0, 0)
                                  : __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, mf[ks][jj]), __builtin_bit_cast(bf16x8, xf[ks][rt]), acc[rt][jj], 0, 0, 0);
        };
        using KS0 = std::integral_constant<int, 0>;
        using KS1 = std::integral_constant<int, 1>;
        if (DBG != 2) read_operands(buf_cur, KS0{});

        for (int q = 0; q < total; ++q) {
            const bool last_kb = c_kb == nkb - 1;
            const uint32_t buf_next = next_buf(buf_cur);
            if (F16) {
                // own part of the next stage: landed (before this iteration's loads are issued: one stage fewer may
                // be outstanding) -> registers; converted while the first k-step multiplies; back to LDS
                wait_loads<(S::NBUF - 3) * S::LPS>();
                read_own(buf_next);
            }
            if (DBG != 2) read_operands(buf_cur, KS1{});
            if (q + S::NBUF - 1 < total) advance_ahead();
            buf_ahead = next_buf(buf_ahead);
            if (DBG != 3) issue_stage(buf_ahead);
            if (F16) {
                if (DBG != 2) multiply(KS0{});
                convert_own(buf_next);
                // issue order: an MFMA first (its operands are in registers), then three conversion instructions
                // behind every MFMA, the LDS writes last
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 3 * S::MPW / 2, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x200, S::MPW, 0);
                __builtin_amdgcn_sched_barrier(0);
                // half of the second k-step before the barrier: the LDS writes above land behind its MFMAs
                if (DBG != 2) multiply_rows(KS1{}, KS0{});
                __builtin_amdgcn_sched_barrier(0);
            } else {
                if (DBG != 2) multiply(KS0{});
                __builtin_amdgcn_sched_barrier(0);                        // the waits below stay behind the first k-step's MFMAs
            }
            // every read of this stage has returned (its buffer is reloaded after the barrier); the next stage has landed
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if (!F16) wait_loads<S::WAIT>();
            __builtin_amdgcn_s_barrier();
            if (DBG != 2 && !last_kb && q + 1 < total) read_operands(buf_next, KS0{});
            if (DBG != 2) { if (F16) multiply_rows(KS1{}, KS1{}); else multiply(KS1{}); }
            __builtin_amdgcn_sched_barrier(0);

            if (DBG != 0 && last_kb) {
#pragma unroll
                for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) { st[rt].s += acc[rt][jj][0] + acc[rt][jj][7]; acc[rt][jj][0] = 0.f; }
            }
            if (DBG == 0 && last_kb) {
                // The accumulators hold base-2 logits minus the row's reference (its running maximum when the
                // tile began; the first tile finds its own maximum first).
                const int n0 = c_vt * kTNT;
                const bool tail = n0 + kTNT > V;
                const bool first = c_vt == col;
#pragma unroll
                for (int rt = 0; rt < 2; ++rt) {
                    if (tail) {
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) {
                            const int cbase = n0 + 32 * (4 * wv + jj) + 4 * (int)(lane_id_now() >> 5);
#pragma unroll
                            for (int i = 0; i < 16; ++i)
                                if (cbase + 8 * (i >> 2) + (i & 3) >= V) acc[rt][jj][i] = kNegBig;
                        }
                    }
                    float ref = st[rt].mc;
                    if (first) {
                        float m4[4];
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) {
                            float m = vmax3(acc[rt][jj][0], acc[rt][jj][1], acc[rt][jj][2]);
#pragma unroll
                            for (int i = 3; i < 15; i += 2) m = vmax3(m, acc[rt][jj][i], acc[rt][jj][i + 1]);
                            m4[jj] = vmax(m, acc[rt][jj][15]);
                        }
                        ref = vmax(vmax3(m4[0], m4[1], m4[2]), m4[3]);
                        ref = vmax(ref, -1.0e30f);                        // a tile of nothing but masked columns
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                            for (int i = 0; i < 16; ++i) acc[rt][jj][i] -= ref;
                    }
                    float tile_max = kNegBig;
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        float v[16];
#pragma unroll
                        for (int i = 0; i < 16; ++i) v[i] = acc[rt][jj][i];
                        stream_group_rel<L, NAT>(st[rt], v, ref, tile_max, c_vt * 8 + 4 * wv + jj);
                        if constexpr (SAMPLE) {
                            const uint32_t ln = lane_id_now();
                            const int srow = sd.row_base + row0 + (wr * 2 + rt) * 32 + (int)(ln & 31);
                            sample_group<NAT>(smp[rt], v, ref, gumbel_key(sd.seed_lo, sd.seed_hi, (uint32_t)srow),
                                              n0 + 32 * (4 * wv + jj) + 4 * (int)(ln >> 5));
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    // the first tile's reference is its own maximum (-1e30 and an empty sum if every column was
                    // masked: the vocabulary's last tile); later tiles move the reference up when they exceed it
                    const float mc_new = first ? ref : vmax(ref, tile_max);
                    // (in two halves: one logit 127 binary orders above the old reference leaves s near the top of the
                    // float range and the whole factor below its bottom, where the hardware exponential has no value)
                    if (!first) {
                        const float half_step = __builtin_amdgcn_exp2f(0.5f * (NAT ? (ref - mc_new) * kLog2e : ref - mc_new));
                        st[rt].s = (st[rt].s * half_step) * half_step;
                    }
                    st[rt].mc = mc_new;
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[rt][jj][i] = -mc_new;
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (DBG != 2 && last_kb && q + 1 < total) read_operands(buf_next, KS0{});      // kept out of the epilogue's registers
            buf_cur = buf_next;
            if (q + 1 < total && ++c_kb == nkb) { c_kb = 0; c_vt += hg.gw; }
        }
        wait_loads<0>();                                                  // the surplus loads of the last stages
    }

    if (DBG) {                                         // timing experiments: cycles and 100 MHz ticks of this block
        if (tid == 0 && blockIdx.x < 8 && (size_t)rows * hg.gw * (3 + 3 * L) >= 64) {
            reinterpret_cast<long long *>(part)[2 * blockIdx.x] = clock64() - dbg_t0;
            reinterpret_cast<long long *>(part)[2 * blockIdx.x + 1] = wall_clock64() - dbg_w0;
        }
        const size_t slot = 64 + (size_t)blockIdx.x * blockDim.x + tid, n_part = (size_t)rows * hg.gw * (3 + 3 * L);
        if (slot < n_part) part[slot] = st[0].s + st[1].s;                          // keeps the arithmetic alive
        return;
    }

    // ---- the records of (row, block).  A row has four lane streams in a block (two half-wavefronts x two column
    // halves), 16 groups each.  hg.spb = 4: every lane stream is written as it is; 2: the half-wavefronts are folded,
    // one record per column half; 1: all four folded into one record.  Folding keeps three groups of the folded
    // streams' 32 or 64 per row, and a row whose best groups crowd into one record pays an exact rescan of all the
    // record's columns in the merge: the fewer records a row has in all (large row counts: few column blocks), the
    // less is folded.  From here on a tag also names the half: tag * 2 + half.
    constexpr int REC = 3 + 3 * L + (SAMPLE ? 8 : 0);
    if (hg.spb == kStreamsPerBlock) {
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            const Stream<L> &a = st[rt];
            const int row = row0 + (wr * 2 + rt) * 32 + l32;
            if (row >= rows) continue;
            float *w = part + (((size_t)row * hg.gw + col) * kStreamsPerBlock + (wv * 2 + half)) * REC;
            w[0] = NAT ? a.mc * kLog2e : a.mc;                          // records carry the running maximum in base-2 units
            w[1] = a.s; w[2] = a.U;
#pragma unroll
            for (int l = 0; l < L; ++l) { w[3 + 3 * l] = a.x[l]; w[4 + 3 * l] = a.y[l]; w[5 + 3 * l] = __int_as_float(a.tag[l] * 2 + half); }
            if constexpr (SAMPLE) {
                w[3 + 3 * L] = smp[rt].w1; w[4 + 3 * L] = __int_as_float(smp[rt].id1); w[5 + 3 * L] = smp[rt].w2;
                w[6 + 3 * L] = __int_as_float(smp[rt].id2); w[7 + 3 * L] = smp[rt].w3;
            }
        }
        return;
    }
    // fold the half-wavefronts (fixed order)
    float *xchg = reinterpret_cast<float *>(lds_raw);                      // [RT][REC + 1], free after the last barrier
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
        Stream<L> &a = st[rt];
        if (NAT) a.mc *= kLog2e;                                        // records carry the running maximum in base-2 units
#pragma unroll
        for (int l = 0; l < L; ++l) a.tag[l] = a.tag[l] * 2 + half;
        Stream<L> o;
        o.mc = __shfl_xor(a.mc, 32); o.s = __shfl_xor(a.s, 32); o.U = __shfl_xor(a.U, 32);
#pragma unroll
        for (int l = 0; l < L; ++l) { o.x[l] = __shfl_xor(a.x[l], 32); o.y[l] = __shfl_xor(a.y[l], 32); o.tag[l] = __shfl_xor(a.tag[l], 32); }
        if (half == 0) stream_combine(a, o);                                // lanes 0..31 now hold both halves
        if constexpr (SAMPLE) {
            SampleTrack so;
            so.w1 = __shfl_xor(smp[rt].w1, 32); so.w2 = __shfl_xor(smp[rt].w2, 32); so.w3 = __shfl_xor(smp[rt].w3, 32);
            so.id1 = __shfl_xor(smp[rt].id1, 32); so.id2 = __shfl_xor(smp[rt].id2, 32);
            if (half == 0) sample_combine(smp[rt], so);
        }
    }
    if (hg.spb == 2) {
        if (half == 0) {
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) {
                const int row = row0 + (wr * 2 + rt) * 32 + l32;
                if (row >= rows) continue;
                float *w = part + (((size_t)row * hg.gw + col) * 2 + wv) * REC;
                w[0] = st[rt].mc; w[1] = st[rt].s; w[2] = st[rt].U;
#pragma unroll
                for (int l = 0; l < L; ++l) { w[3 + 3 * l] = st[rt].x[l]; w[4 + 3 * l] = st[rt].y[l]; w[5 + 3 * l] = __int_as_float(st[rt].tag[l]); }
                if constexpr (SAMPLE) {
                    w[3 + 3 * L] = smp[rt].w1; w[4 + 3 * L] = __int_as_float(smp[rt].id1); w[5 + 3 * L] = smp[rt].w2;
                    w[6 + 3 * L] = __int_as_float(smp[rt].id2); w[7 + 3 * L] = smp[rt].w3;
                }
            }
        }
        return;
    }
    // ... and the two column halves, through shared memory
    __syncthreads();                                                        // every wavefront is past its last operand read
    if (wv == 1 && half == 0) {
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            float *o = xchg + ((wr * 2 + rt) * 32 + l32) * (REC + 1);
            o[0] = st[rt].mc; o[1] = st[rt].s; o[2] = st[rt].U;
#pragma unroll
            for (int l = 0; l < L; ++l) { o[3 + 3 * l] = st[rt].x[l]; o[4 + 3 * l] = st[rt].y[l]; o[5 + 3 * l] = __int_as_float(st[rt].tag[l]); }
            if constexpr (SAMPLE) {
                o[3 + 3 * L] = smp[rt].w1; o[4 + 3 * L] = __int_as_float(smp[rt].id1); o[5 + 3 * L] = smp[rt].w2;
                o[6 + 3 * L] = __int_as_float(smp[rt].id2); o[7 + 3 * L] = smp[rt].w3;
            }
        }
    }
    __syncthreads();
    if (wv == 0 && half == 0) {
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            const int row = row0 + (wr * 2 + rt) * 32 + l32;
            const float *i = xchg + ((wr * 2 + rt) * 32 + l32) * (REC + 1);
            Stream<L> o;
            o.mc = i[0]; o.s = i[1]; o.U = i[2];
#pragma unroll
            for (int l = 0; l < L; ++l) { o.x[l] = i[3 + 3 * l]; o.y[l] = i[4 + 3 * l]; o.tag[l] = __float_as_int(i[5 + 3 * l]); }
            stream_combine(st[rt], o);
            if constexpr (SAMPLE) {
                SampleTrack so;
                so.w1 = i[3 + 3 * L]; so.id1 = __float_as_int(i[4 + 3 * L]); so.w2 = i[5 + 3 * L];
                so.id2 = __float_as_int(i[6 + 3 * L]); so.w3 = i[7 + 3 * L];
                sample_combine(smp[rt], so);
            }
            if (row >= rows) continue;
            float *w = part + ((size_t)row * hg.gw + col) * REC;
            w[0] = st[rt].mc; w[1] = st[rt].s; w[2] = st[rt].U;
#pragma unroll
            for (int l = 0; l < L; ++l) { w[3 + 3 * l] = st[rt].x[l]; w[4 + 3 * l] = st[rt].y[l]; w[5 + 3 * l] = __int_as_float(st[rt].tag[l]); }
            if constexpr (SAMPLE) {
                w[3 + 3 * L] = smp[rt].w1; w[4 + 3 * L] = __int_as_float(smp[rt].id1); w[5 + 3 * L] = smp[rt].w2;
                w[6 + 3 * L] = __int_as_float(smp[rt].id2); w[7 + 3 * L] = smp[rt].w3;
            }
        }
    }
}

// Row-major bf16 rows [rows, K] -> the X layout of head_tile_kernel (zero beyond K and beyond the last row).
// grid = (rows_pad / 64, 8 ceil(K / 64)); one thread per 16-byte vector.
__global__ __launch_bounds__(64) void regroup_rows_kernel(const uint16_t *__restrict__ h, uint4 *__restrict__ X,
                                                          int rows, int rows_pad, int K)
{
    const int row = blockIdx.x * 64 + threadIdx.x, kg = blockIdx.y;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (row < rows && kg * 8 < K) v = *reinterpret_cast<const uint4 *>(h + (size_t)row * K + kg * 8);       // K is a multiple of 8
    X[(size_t)kg * rows_pad + row] = v;
}

hipError_t launch_regroup_rows(const uint16_t *h, void *X, int rows, int rows_pad, int K, hipStream_t st)
{
    dim3 grid(rows_pad / 64, 8 * ((K + 63) / 64));
    regroup_rows_kernel<<<grid, 64, 0, st>>>(h, static_cast<uint4 *>(X), rows, rows_pad, K);
    return hipGetLastError();
}

int head_tile_rows_per_block(int rows) {
#ifdef SLIMSPEC_DIAG_TILE128      // experiment builds only: 128-row blocks at any row count
    return 128;
#endif
    return rows > 128 ? 256 : 128;
}

template <int WR, bool F16, bool NAT, int DBG, bool SAMPLE>
static hipError_t launch_tile_cfg(const void *X, const uint16_t *M, float *part, int rows, int rows_pad,
                                  int K, int V, int n_rb, int gw, const SampleSeed &sd, hipStream_t st)
{
    using S = TileShape<WR>;
    auto fn = head_tile_kernel<kStreamList, WR, F16, NAT, DBG, SAMPLE>;
    static LdsLimit lds_limit;
    hipError_t e = lds_limit.raise(reinterpret_cast<const void *>(fn), S::LDS);
    if (e != hipSuccess) return e;
    HeadGrid hg{n_rb, gw, (V + kTNT - 1) / kTNT, streams_per_block(gw)};
    fn<<<n_rb * gw, 64 * S::NW, S::LDS, st>>>(static_cast<const uint4 *>(X), M, part, rows, rows_pad, K, V, hg, sd);
    return hipGetLastError();
}

// Experiment builds only (-DSLIMSPEC_DIAG_DBG=1|2|3): a timing-only variant of the kernel replaces the real one;
// its records are not records, the merge must not read them and the calls report SLIMSPEC_UNSUPPORTED.
#ifndef SLIMSPEC_DIAG_DBG
#define SLIMSPEC_DIAG_DBG 0
#endif
bool head_tile_timing_only() { return SLIMSPEC_DIAG_DBG != 0; }

hipError_t launch_head_tile(const void *X, bool x_is_f16, bool natural_units, const uint16_t *M, float *part, int rows, int rows_pad,
                            int K, int V, int n_rb, int gw, const SampleOut &so, int row_base, hipStream_t st)
{
    const bool big = head_tile_rows_per_block(rows) == 256;
    const SampleSeed sd{so.seed_lo, so.seed_hi, row_base};
#define SLIMSPEC_TILE_S(F16, NAT, DBG, SMP) (big ? launch_tile_cfg<4, F16, NAT, DBG, SMP>(X, M, part, rows, rows_pad, K, V, n_rb, gw, sd, st) \
                                                 : launch_tile_cfg<2, F16, NAT, DBG, SMP>(X, M, part, rows, rows_pad, K, V, n_rb, gw, sd, st))
#define SLIMSPEC_TILE_F(F16, NAT, DBG) (so.on ? SLIMSPEC_TILE_S(F16, NAT, 0, true) : SLIMSPEC_TILE_S(F16, NAT, DBG, false))
#define SLIMSPEC_TILE(DBG) (natural_units ? SLIMSPEC_TILE_F(false, true, DBG) \
                                          : (x_is_f16 ? SLIMSPEC_TILE_F(true, false, DBG) : SLIMSPEC_TILE_F(false, false, DBG)))
    return SLIMSPEC_TILE(SLIMSPEC_DIAG_DBG);
#undef SLIMSPEC_TILE
#undef SLIMSPEC_TILE_F
#undef SLIMSPEC_TILE_S
}

}  // namespace slimspec

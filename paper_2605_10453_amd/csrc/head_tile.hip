// Vocabulary-tiled up-projection on the matrix cores with the fused log-sum-exp / top-k epilogue
// (paper section 4.1: logits = t B, never written to memory), for calls with many rows.
//
// Shape of the kernel
//   * One block = 4 wavefronts = a 128-row x 256-column tile of logits; two blocks share a CU (two
//     wavefronts per SIMD, from different blocks and therefore at different phases: one block's
//     epilogue overlaps the other block's matrix instructions).  A wavefront owns 64 rows x 128
//     columns = 2 x 4 MFMA tiles of 32 x 32 (v_mfma_f32_32x32x16_bf16, accumulators in VGPRs).
//   * The transposed product z^T = M^T x^T is computed, so that the 16 values an MFMA tile gives a
//     lane belong to ONE row: running max, sum of exp and candidate bookkeeping stay inside the lane.
//   * Stages of 32 contraction elements travel global memory -> LDS without passing registers
//     (global_load_lds_dwordx4): the M tile row-major as it lies in memory, the X tile as 16-byte
//     vectors of 8 consecutive contraction elements.  Three stage buffers; loads are issued two
//     stages ahead.  MFMA operands come from LDS with ds_read_b64_tr_b16 (M: transposes the
//     row-major tile into 4 consecutive contraction elements per lane) and ds_read_b128 (X).
//   * 16-byte pieces of an M row are stored XOR-swizzled by (k mod 4) so that the four rows a
//     transposing read touches fall into different banks.
//
// Waits: the compiler does not see the direct-to-LDS loads (inline asm), so the kernel counts them
// itself: every wavefront issues exactly 6 per stage, vector memory returns in order, hence
// s_waitcnt vmcnt(6) = "everything but the stage issued last has landed".  No other vector memory
// instruction may sit inside the main loop (the kernel must not spill).
#include "head_stream.hpp"
#include "launch.hpp"

namespace slimspec {

namespace {

constexpr int kTKB = 32;                                   // contraction elements per stage
constexpr int kTNT = 256;                                  // vocabulary columns per tile
constexpr int kTRT = 128;                                  // rows per block
constexpr int kTStages = 3;
constexpr int kTMBytes = kTKB * kTNT * 2;                  // 16 KB
constexpr int kTXBytes = (kTKB / 8) * kTRT * 16;           //  8 KB
constexpr int kTStageBytes = kTMBytes + kTXBytes;
constexpr int kTLdsBytes = kTStages * kTStageBytes;        // 72 KB: two blocks per CU

typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef short v8i16 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define LDS_PTR(T, byte_addr) ((__attribute__((address_space(3))) T *)(uintptr_t)(byte_addr))

// 16 bytes per lane, global memory -> LDS at buf + OFF + 16 * lane (buf uniform)
template <int OFF>
__device__ __forceinline__ void dma16(uint32_t buf, uint32_t voff, const void *base) {
    asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(buf), "v"(voff), "s"(base), "n"(OFF) : "memory", "scc");
}

}  // namespace

// X: [8 ceil(K / 64)][rows_pad] 16-byte vectors: 8 consecutive contraction elements of one row, bf16, times
//    log2(e), zero beyond K
// M: [K][V] bf16 row-major, V and K multiples of 8
// part: [rows][nsr][3 + 3 L] stream records (values in base-2 units), nsr = 4 gw
template <int L>
__global__ __launch_bounds__(256, 2) void head_tile_kernel(
    const uint4 *__restrict__ X, const uint16_t *__restrict__ M, float *__restrict__ part,
    int rows, int rows_pad, int K, int V, HeadGrid hg)
{
    extern __shared__ __align__(1024) unsigned char lds_raw[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) unsigned char *)lds_raw);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, wv = wave & 1;
    const int half = lane >> 5, l32 = lane & 31, g1 = (lane >> 4) & 1, j16 = lane & 15;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int rb = slot % hg.n_rb, col = (slot / hg.n_rb) * 8 + xcd;
    const int row0 = rb * kTRT;
    const int nkb = (K + kTKB - 1) / kTKB;
    const int njobs = (col < hg.n_vt) ? (hg.n_vt - col + hg.gw - 1) / hg.gw : 0;
    const int total = njobs * nkb;
    const bool ktail = (K & (kTKB - 1)) != 0;

    // ---- direct-to-LDS loads of one stage: 4 of M, 2 of X per wavefront.
    // M load uu of this wavefront covers stage rows 8 wave + 2 uu + (lane >> 5); lane -> stored piece lane & 31,
    // which holds source piece (lane & 31) ^ ((row & 3) << 2).
    const uint32_t kp = lane >> 5, pp = lane & 31;
    const uint32_t mcol_e = (pp ^ (kp << 2)) * 16u;            // source byte column when (row & 3) = kp
    const uint32_t mcol_o = (pp ^ ((2u + kp) << 2)) * 16u;     // ... when (row & 3) = 2 + kp
    const uint32_t rowb = (uint32_t)V * 2u;                    // bytes per row of M
    uint32_t mv[2];                                            // lane offsets from the row pair's first row (even / odd pair)
    const auto set_tile = [&](int vt) {
        const uint32_t climit = (uint32_t)(V - vt * kTNT - 8) * 2u;      // last 16-byte piece of the row that exists
        const uint32_t ce = min(mcol_e, climit), co = min(mcol_o, climit);
        mv[0] = kp * rowb + ce;
        mv[1] = (kp + 2u) * rowb + co;
    };
    const uint32_t xv0 = (uint32_t)lane * 16u;
    const unsigned char *const m_wave = reinterpret_cast<const unsigned char *>(M) + (size_t)(8 * wave) * rowb;
    const unsigned char *const x_wave = reinterpret_cast<const unsigned char *>(X + (size_t)wave * rows_pad + row0);
    const size_t m_step = (size_t)kTKB * rowb, x_step = (size_t)4 * rows_pad * 16;

    // position of the stage whose loads are issued next
    int a_vt = col, a_kb = 0;
    const unsigned char *mptr = m_wave + (size_t)col * kTNT * 2, *xptr = x_wave;
    const auto issue_stage = [&](uint32_t buf) {
        if (ktail && a_kb == nkb - 1) {
            // last, partial k-block: rows beyond K are read from row K - 2 / K - 1 (they meet zeros of X)
            const uint32_t ce = mv[0] - kp * rowb, co = mv[1] - (kp + 2u) * rowb;
            const unsigned char *tile0 = reinterpret_cast<const unsigned char *>(M) + (size_t)a_vt * kTNT * 2;
#define SLIMSPEC_TAIL_LOAD(UU)                                                                            \
            { const int krow = min(a_kb * kTKB + 8 * wave + 2 * UU, K - 2);                                 \
              dma16<(UU) * 1024>(buf + (uint32_t)(wave * 4096), kp * rowb + ((UU & 1) ? co : ce), tile0 + (size_t)krow * rowb); }
            SLIMSPEC_TAIL_LOAD(0) SLIMSPEC_TAIL_LOAD(1) SLIMSPEC_TAIL_LOAD(2) SLIMSPEC_TAIL_LOAD(3)
#undef SLIMSPEC_TAIL_LOAD
        } else {
            const uint32_t mb = buf + (uint32_t)(wave * 4096);
            const unsigned char *mptr4 = mptr + 4 * (size_t)rowb;
            dma16<0>(mb, mv[0], mptr);
            dma16<1024>(mb, mv[1], mptr);
            dma16<2048>(mb, mv[0], mptr4);
            dma16<3072>(mb, mv[1], mptr4);
        }
        const uint32_t xb = buf + (uint32_t)(kTMBytes + wave * kTRT * 16);
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
    const uint32_t xa = (uint32_t)(kTMBytes + (half * kTRT + wr * 64 + l32) * 16);
    // M fragment of MFMA tile jj: ma0 ^ (jj << 6) (the swizzle exchanges 64-byte groups; stage buffers are 1 KB aligned)
    const uint32_t ma0 = (uint32_t)((8 * half + (j16 >> 2)) * 512
                                    + (wv * 16 + 4 * (j16 >> 2) + 2 * g1 + ((j16 & 3) >> 1)) * 16 + (j16 & 1) * 8);

    Stream<L> st[2];
    stream_init(st[0]);
    stream_init(st[1]);
    f32x16 acc[2][4];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[rt][jj][i] = 0.f;

    if (total > 0) {
        int c_vt = col, c_kb = 0;                                         // stage being multiplied
        uint32_t buf_cur = lds0, buf_ahead = lds0;
        const auto next_buf = [&](uint32_t b) { return (b + kTStageBytes == lds0 + kTLdsBytes) ? lds0 : b + kTStageBytes; };
        set_tile(col);
        issue_stage(buf_ahead);                                           // stage 0
        if (total > 1) advance_ahead();
        buf_ahead = next_buf(buf_ahead);
        issue_stage(buf_ahead);                                           // stage 1 (or stage 0 once more)
        asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
        __builtin_amdgcn_s_barrier();

        for (int q = 0; q < total; ++q) {
            if (q + 2 < total) advance_ahead();                           // past the end: the last stage once more
            buf_ahead = next_buf(buf_ahead);
            issue_stage(buf_ahead);

#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                bf16x8 xf[2], mf[4];
#pragma unroll
                for (int rt = 0; rt < 2; ++rt)
                    xf[rt] = __builtin_bit_cast(bf16x8, *LDS_PTR(u32x4, buf_cur + xa + ks * 4096 + rt * 512));
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const uint32_t mj = (buf_cur + ma0) ^ (uint32_t)(jj << 6);
                    const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4i16, mj + ks * 8192));
                    const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4i16, mj + ks * 8192 + 2048));
                    mf[jj] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                }
#pragma unroll
                for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj)
                        acc[rt][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(mf[jj], xf[rt], acc[rt][jj], 0, 0, 0);
            }

            if (c_kb == nkb - 1) {
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
                            const int cbase = n0 + 32 * (4 * wv + jj) + 4 * half;
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
                        stream_group_rel<L>(st[rt], v, ref, tile_max, c_vt * 8 + 4 * wv + jj);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    const float mc_new = first ? tile_max : vmax(ref, tile_max);
                    st[rt].s *= __builtin_amdgcn_exp2f(ref - mc_new);
                    st[rt].mc = mc_new;
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[rt][jj][i] = -mc_new;
                }
            }
            asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            buf_cur = next_buf(buf_cur);
            if (q + 1 < total && ++c_kb == nkb) { c_kb = 0; c_vt += hg.gw; }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                  // the surplus loads of the last stages
    }

    // one partial per (row, stream): stream = (col * 2 + wv) * 2 + half
    const int nsr = hg.gw * 4;
    const int sidx = (col * 2 + wv) * 2 + half;
    constexpr int REC = 3 + 3 * L;
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
        const int row = row0 + (wr * 2 + rt) * 32 + l32;
        if (row >= rows) continue;
        float *o = part + ((size_t)row * nsr + sidx) * REC;
        o[0] = st[rt].mc; o[1] = st[rt].s; o[2] = st[rt].U;
#pragma unroll
        for (int l = 0; l < L; ++l) {
            o[3 + 3 * l] = st[rt].x[l];
            o[4 + 3 * l] = st[rt].y[l];
            o[5 + 3 * l] = __int_as_float(st[rt].tag[l]);
        }
    }
}

hipError_t launch_head_tile(const void *X, const uint16_t *M, float *part, int rows, int rows_pad,
                            int K, int V, int n_rb, int gw, hipStream_t st)
{
    auto fn = head_tile_kernel<kStreamList>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, kTLdsBytes);
    if (e != hipSuccess) return e;
    HeadGrid hg{n_rb, gw, (V + kTNT - 1) / kTNT};
    fn<<<n_rb * gw, 256, kTLdsBytes, st>>>(static_cast<const uint4 *>(X), M, part, rows, rows_pad, K, V, hg);
    return hipGetLastError();
}

}  // namespace slimspec

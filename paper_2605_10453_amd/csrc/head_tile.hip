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

// 16 bytes per lane, global memory -> LDS at lds_addr + 16 * lane (lds_addr uniform)
__device__ __forceinline__ void dma16(uint32_t lds_addr, uint32_t voff, const void *base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(voff), "s"(base) : "memory");
}

}  // namespace

// X: [ceil(K / 8) padded to a multiple of 8 groups][rows_pad] 16-byte vectors (8 bf16, zero beyond K)
// M: [K][V] bf16 row-major, V a multiple of 8, K even
// part: [rows][nsr][3 + 3 L] stream records, nsr = 4 gw
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

    // ---- direct-to-LDS loads of one stage: 4 of M, 2 of X per wavefront
    // M load u of the stage (u = 4 wave + uu) covers stage rows 2u, 2u + 1: lane -> (row 2u + (lane >> 5), stored piece lane & 31)
    const uint32_t kp = lane >> 5, pp = lane & 31;
    const uint32_t mcol_e = (pp ^ (kp << 2)) * 16u;            // source byte column when (row & 3) = kp
    const uint32_t mcol_o = (pp ^ ((2u + kp) << 2)) * 16u;     // ... when (row & 3) = 2 + kp
    const uint32_t mrow = kp * (uint32_t)V * 2u;
    const auto issue_stage = [&](int vt, int kb, uint32_t buf) {
        const int n0 = vt * kTNT;
        const uint32_t climit = (uint32_t)(V - n0 - 8) * 2u;   // last 16-byte piece of the row that exists
        const uint32_t ve = mrow + min(mcol_e, climit), vo = mrow + min(mcol_o, climit);
#pragma unroll
        for (int uu = 0; uu < 4; ++uu) {
            const int krow = min(kb * kTKB + 8 * wave + 2 * uu, K - 2);
            const uint16_t *src = M + (size_t)krow * V + n0;
            dma16(buf + (uint32_t)((4 * wave + uu) * 1024), (uu & 1) ? vo : ve, src);
        }
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const uint4 *src = X + (size_t)(kb * 4 + wave) * rows_pad + row0 + hh * 64;
            dma16(buf + (uint32_t)(kTMBytes + (wave * kTRT + hh * 64) * 16), (uint32_t)lane * 16u, src);
        }
    };

    // ---- operand addresses inside a stage
    const uint32_t xa = (uint32_t)(kTMBytes + (half * kTRT + wr * 64 + l32) * 16);
    uint32_t ma[4];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
        ma[jj] = (uint32_t)((8 * half + (j16 >> 2)) * 512
                            + (wv * 16 + 4 * (jj ^ (j16 >> 2)) + 2 * g1 + ((j16 & 3) >> 1)) * 16 + (j16 & 1) * 8);

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

    struct Pos { int vt, kb; };
    const auto advance = [&](Pos p) { Pos o = p; if (++o.kb == nkb) { o.kb = 0; o.vt += hg.gw; } return o; };
    if (total > 0) {
        Pos cur{col, 0}, ahead{col, 0};
        uint32_t buf_cur = lds0, buf_ahead = lds0;
        const auto next_buf = [&](uint32_t b) { return (b + kTStageBytes == lds0 + kTLdsBytes) ? lds0 : b + kTStageBytes; };
        issue_stage(ahead.vt, ahead.kb, buf_ahead);                       // stage 0
        if (total > 1) ahead = advance(ahead);
        buf_ahead = next_buf(buf_ahead);
        issue_stage(ahead.vt, ahead.kb, buf_ahead);                       // stage 1 (or stage 0 once more)
        asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
        __builtin_amdgcn_s_barrier();

        for (int q = 0; q < total; ++q) {
            if (q + 2 < total) ahead = advance(ahead);                    // past the end: the last stage once more
            buf_ahead = next_buf(buf_ahead);
            issue_stage(ahead.vt, ahead.kb, buf_ahead);

#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                bf16x8 xf[2], mf[4];
#pragma unroll
                for (int rt = 0; rt < 2; ++rt)
                    xf[rt] = __builtin_bit_cast(bf16x8, *LDS_PTR(u32x4, buf_cur + xa + ks * 4096 + rt * 512));
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4i16, buf_cur + ma[jj] + ks * 8192));
                    const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4i16, buf_cur + ma[jj] + ks * 8192 + 2048));
                    mf[jj] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                }
#pragma unroll
                for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj)
                        acc[rt][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(mf[jj], xf[rt], acc[rt][jj], 0, 0, 0);
            }

            if (cur.kb == nkb - 1) {
                const int n0 = cur.vt * kTNT;
                const bool tail = n0 + kTNT > V;
#pragma unroll
                for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        float v[16];
#pragma unroll
                        for (int i = 0; i < 16; ++i) v[i] = acc[rt][jj][i];
                        if (tail) {
                            const int cbase = n0 + 32 * (4 * wv + jj) + 4 * half;
#pragma unroll
                            for (int i = 0; i < 16; ++i)
                                if (cbase + 8 * (i >> 2) + (i & 3) >= V) v[i] = kNegBig;
                        }
                        stream_group<L>(st[rt], v, cur.vt * 8 + 4 * wv + jj);
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[rt][jj][i] = 0.f;
                        __builtin_amdgcn_sched_barrier(0);
                    }
            }
            asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            buf_cur = next_buf(buf_cur);
            if (q + 1 < total) cur = advance(cur);
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

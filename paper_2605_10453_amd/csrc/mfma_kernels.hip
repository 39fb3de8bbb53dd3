// Matrix-core kernels for calls with many rows (paper section 4.1).
//
//   down_gemm_kernel     partial sums of t = h A over a slice of d (bf16 MFMA, fp32 accumulate)
//   down_finish_kernel   fixed-order sum of the slices -> fp32 t, f16 t in the k-grouped layout the
//                        up-projection reads, per-row rounding statistics, an rms estimate of B
//   head_mfma_kernel     persistent vocabulary-tiled up-projection z^T = M^T x^T with the fused
//                        epilogue: every lane keeps, for each row it owns, a running max / sum of exp
//                        and the L largest "group maxima" of its own share of the vocabulary; one
//                        partial per lane stream goes to the merge.  No logit is written to memory.
//
// Epilogue bookkeeping.  One 32x32 MFMA tile gives a lane 16 logits of one row (a "group").  The
// low 4 bits of each logit are replaced by its position in the group, so that plain max / min /
// median instructions carry the argmax along; a 37-instruction network yields the group's largest
// and second largest value.  Per (lane, row) a short list holds the L groups with the largest
// maxima, each with its second largest value and a tag naming the group; U is the largest
// maximum that fell off the list.  The merge knows from these bounds exactly which logits might
// still belong to the top-k and re-evaluates those in fp32.
#include "mfma_core.hpp"
#include "launch.hpp"
#include "head_stream.hpp"
#include <type_traits>

namespace slimspec {

// ---------------------------------------------------------------------------
// t = h A, slice z of the contraction.  grid = (ceil(r / 256), row blocks, slices).
template <class C>
__global__ __launch_bounds__(C::THREADS) void down_gemm_kernel(
    const uint16_t *__restrict__ h, const uint16_t *__restrict__ A, float *__restrict__ part,
    int rows, int ld, int d, int r, int kslice)
{
    extern __shared__ uint4 lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave / C::WV, wv = wave % C::WV;
    const int n0 = blockIdx.x * kNT, row0 = blockIdx.y * C::RT;
    const int kbeg = blockIdx.z * kslice, kend = min(d, kbeg + kslice);
    const int nkb = (kend - kbeg + kKB - 1) / kKB;

    f32x16 acc[C::TR][C::TV];
    MRegs<C> mr;
    XRegs<C> xr;
    load_m_regs<C>(mr, A, kend, r, kbeg, n0, tid);
    load_x_regs<C, true>(xr, h, kend, d, rows, 0, kbeg, row0, tid);
    store_m_lds<C, false>(mr, lds, tid);
    store_x_lds<C, true>(xr, lds + C::M_VECS, tid);
    __syncthreads();
    for (int kb = 0; kb < nkb; ++kb) {
        uint4 *cur = lds + (kb & 1) * C::STAGE_VECS, *nxt = lds + ((kb + 1) & 1) * C::STAGE_VECS;
        const bool more = kb + 1 < nkb;
        if (more) {
            load_m_regs<C>(mr, A, kend, r, kbeg + (kb + 1) * kKB, n0, tid);
            load_x_regs<C, true>(xr, h, kend, d, rows, 0, kbeg + (kb + 1) * kKB, row0, tid);
        }
        mma_stage<C, false>(acc, cur, cur + C::M_VECS, wr, wv, lane, kb == 0);
        if (more) {
            store_m_lds<C, false>(mr, nxt, tid);
            store_x_lds<C, true>(xr, nxt + C::M_VECS, tid);
        }
        __syncthreads();
    }
    // partial sums are stored column-major, part[slice][n][ld]: the 32 lanes of a half-wavefront hold
    // 32 consecutive rows of one n, so every store instruction writes two full 128-byte lines
    const int half = lane >> 5, l32 = lane & 31;
    float *dst = part + (size_t)blockIdx.z * r * ld;
#pragma unroll
    for (int rt = 0; rt < C::TR; ++rt) {
        const int row = row0 + (wr * C::TR + rt) * 32 + l32;      // < ld by construction
#pragma unroll
        for (int j = 0; j < C::TV; ++j)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int n = n0 + tile_n_offset(wv * C::TV + j, i, half);
                if (n < r) dst[(size_t)n * ld + row] = read_acc(acc[rt][j][i]);
            }
    }
}

// ---------------------------------------------------------------------------
// Fixed-order sum of the slices.  grid = (rows_pad / 64 + 1, 2 ceil(r / 64)); block (bx, by) of 256
// threads owns rows [64 bx, 64 bx + 64) and the four 8-wide k-groups 4 by .. 4 by + 3 (thread =
// (row, k-group)); the extra block row bx = rows_pad / 64 estimates rms(B) (by = 0 only).
//   part  [slices, r, ld]     fp32 partial sums, ld = rows_pad
//   t32   [rows_pad, r]       fp32 t (zero for padding rows)
//   t16   [8 ceil(r / 64), rows_pad]   16-byte vectors of 8 f16 (round to nearest even), zero for k >= r
//   stat  [2 ceil(r / 64), rows_pad]   per block column: (sum of (t - f16(t))^2, sum of t^2) of its 32 entries
//   brms  [1]                 sqrt(mean of B^2 over a fixed sample of entries)
constexpr int kBrmsPositions = 4;

__global__ __launch_bounds__(256) void down_finish_kernel(
    const float *__restrict__ part, int slices, int rows, int rows_pad, int r,
    float *__restrict__ t32, uint4 *__restrict__ t16, float2 *__restrict__ stat,
    const uint16_t *__restrict__ B, int V, float *__restrict__ brms, int as_bf16)
{
    __shared__ float red_a[4][64], red_b[4][64];
    const int tid = threadIdx.x, lane = tid & 63, kgl = tid >> 6;
    if ((int)blockIdx.x * 64 >= rows_pad) {
        if (blockIdx.y != 0) return;
        // sample: 8 adjacent entries of every row of B at a few column positions spread over V
        float a = 0.f;
        for (int q = tid; q < r * kBrmsPositions; q += 256) {
            const int j = q / kBrmsPositions, pos = q % kBrmsPositions;
            const int col = (int)(((long long)pos * (V / 8)) / kBrmsPositions) * 8;
            const uint4 w = *reinterpret_cast<const uint4 *>(B + (size_t)j * V + col);
            const float f[8] = {bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y),
                                bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w)};
#pragma unroll
            for (int e = 0; e < 8; ++e) a += f[e] * f[e];
        }
        a = wave_sum(a);
        if (lane == 0) red_a[kgl][0] = a;
        __syncthreads();
        if (tid == 0)
            brms[0] = sqrtf((((red_a[0][0] + red_a[1][0]) + red_a[2][0]) + red_a[3][0]) / (float)(r * kBrmsPositions * 8));
        return;
    }
    const int row = blockIdx.x * 64 + lane;
    const int kg = blockIdx.y * 4 + kgl;
    float a = 0.f, b = 0.f;
    if (kg < r / 8) {
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = 0.f;
        if (row < rows) {
            for (int s = 0; s < slices; ++s) {                // fixed order
                const float *src = part + ((size_t)s * r + kg * 8) * rows_pad + row;
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] += src[(size_t)e * rows_pad];
            }
        }
        float4 *o = reinterpret_cast<float4 *>(t32 + (size_t)row * r + kg * 8);
        o[0] = make_float4(v[0], v[1], v[2], v[3]);
        o[1] = make_float4(v[4], v[5], v[6], v[7]);
        if (as_bf16 == 1) {
            uint32_t hb[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                // bf16 operand of the direct-to-LDS head kernel, in base-2 units: t log2(e)
                const uint32_t u = __float_as_uint(v[e] * kLog2e);
                hb[e] = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;            // round to nearest even
                const float dlt = v[e] - __uint_as_float(hb[e] << 16) * kLn2;
                a += dlt * dlt;
                b += v[e] * v[e];
            }
            t16[(size_t)kg * rows_pad + row] = make_uint4(hb[0] | (hb[1] << 16), hb[2] | (hb[3] << 16),
                                                          hb[4] | (hb[5] << 16), hb[6] | (hb[7] << 16));
        } else {
            // f16 operand: t itself (register-staged kernel) or t log2(e) (direct-to-LDS kernel: base-2 units)
            const float scale = (as_bf16 == 2) ? kLog2e : 1.0f;
            const float back = (as_bf16 == 2) ? kLn2 : 1.0f;
            f16x8 hv;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                hv[e] = (_Float16)(v[e] * scale);
                const float dlt = v[e] - (float)hv[e] * back;
                a += dlt * dlt;
                b += v[e] * v[e];
            }
            t16[(size_t)kg * rows_pad + row] = __builtin_bit_cast(uint4, hv);
        }
    } else {
        t16[(size_t)kg * rows_pad + row] = make_uint4(0, 0, 0, 0);     // zero padding of k up to a multiple of 64
    }
    red_a[kgl][lane] = a;
    red_b[kgl][lane] = b;
    __syncthreads();
    if (kgl == 0)
        stat[(size_t)blockIdx.y * rows_pad + row] =
            make_float2(((red_a[0][lane] + red_a[1][lane]) + red_a[2][lane]) + red_a[3][lane],
                        ((red_b[0][lane] + red_b[1][lane]) + red_b[2][lane]) + red_b[3][lane]);
}

template <class C, bool F16, bool XROW, int L>
__global__ __launch_bounds__(C::THREADS, 1) void head_mfma_kernel(
    const uint16_t *__restrict__ X, const uint16_t *__restrict__ M, float *__restrict__ part,
    int rows, int rows_pad, int K, int V, HeadGrid hg)
{
    extern __shared__ uint4 lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave / C::WV, wv = wave % C::WV;
    const int half = lane >> 5, l32 = lane & 31;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int rb = slot % hg.n_rb, col = (slot / hg.n_rb) * 8 + xcd;
    const int row0 = rb * C::RT;
    const int nkb = (K + kKB - 1) / kKB;
    const int njobs = (col < hg.n_vt) ? (hg.n_vt - col + hg.gw - 1) / hg.gw : 0;
    const int total = njobs * nkb;

    Stream<L> st[C::TR];
#pragma unroll
    for (int rt = 0; rt < C::TR; ++rt) stream_init(st[rt]);
    f32x16 acc[C::TR][C::TV];
    // Software pipeline over the flattened (tile, k-block) stages q = 0 .. total - 1:
    //   stage q + 2: rows of M and the X tile -> registers (global loads issued at the start of stage q)
    //   stage q + 1: registers -> k-contiguous f16/bf16 vectors -> LDS, interleaved with the MFMAs of stage q
    //   stage q    : MFMAs from LDS
    // The steady state has no branch around a load, so that the compiler's count of loads in flight
    // stays exact and a stage never waits for the loads it has just issued.
    struct Pos { int vt, kb; };
    const auto advance = [&](Pos p) { Pos o = p; if (++o.kb == nkb) { o.kb = 0; o.vt += hg.gw; } return o; };
    MRegs<C> mreg[2];
    XRegs<C> xreg[2];
    const auto load_stage = [&](MRegs<C> &m, XRegs<C> &x, Pos p) {
        load_x_regs<C, XROW>(x, X, K, K, rows, rows_pad, p.kb * kKB, row0, tid);
        load_m_regs<C>(m, M, K, V, p.kb * kKB, p.vt * kNT, tid);
    };
    Pos cur{col, 0}, loaded{col, 0};
    zero_acc(acc);
    if (total > 0) {
        load_stage(mreg[0], xreg[0], cur);
        store_m_lds<C, F16>(mreg[0], lds, tid);
        store_x_lds<C, XROW>(xreg[0], lds + C::M_VECS, tid);
        if (total > 1) loaded = advance(cur);
        load_stage(mreg[1], xreg[1], loaded);             // stage 1 (a harmless reload of stage 0 if there is none)
    }
    __syncthreads();

    // one stage; PAR = q & 1 selects the LDS stage and the register sets at compile time
    auto run_stage = [&](auto par_tag, int q) {
        constexpr int PAR = decltype(par_tag)::value;
        uint4 *st_cur = lds + PAR * C::STAGE_VECS, *st_nxt = lds + (PAR ^ 1) * C::STAGE_VECS;
        const Pos ahead = (q + 2 < total) ? advance(loaded) : loaded;      // past the end: reload the last stage
        load_stage(mreg[PAR], xreg[PAR], ahead);
        __builtin_amdgcn_sched_barrier(0);
        mma_stage_and_store<C, F16, XROW>(acc, st_cur, st_cur + C::M_VECS, wr, wv, lane,
                                          mreg[PAR ^ 1], xreg[PAR ^ 1], st_nxt, st_nxt + C::M_VECS, tid);
        if (cur.kb == nkb - 1) {
            const int n0 = cur.vt * kNT;
            const bool tail = n0 + kNT > V;
            const int mlim = (V - n0) >> 3;               // groups of 8 columns that exist in this tile
#pragma unroll
            for (int rt = 0; rt < C::TR; ++rt)
#pragma unroll
                for (int j = 0; j < C::TV; ++j) {
                    float v[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i) v[i] = read_acc(acc[rt][j][i]);
                    if (tail) {
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            if (8 * (i >> 2) + 4 * half + (i & 3) >= mlim) v[i] = kNegBig;
                    }
                    stream_group<L>(st[rt], v, cur.vt * 8 + wv * C::TV + j);
                    __builtin_amdgcn_sched_barrier(0);      // one group at a time: keeps register pressure flat
                }
            zero_acc(acc);
        }
        lds_barrier();
        loaded = ahead;
        if (q + 1 < total) cur = advance(cur);
    };
    for (int q = 0; q < total; q += 2) {
        run_stage(std::integral_constant<int, 0>{}, q);
        if (q + 1 < total) run_stage(std::integral_constant<int, 1>{}, q + 1);
    }
    // one partial per (row, stream): stream = (col * WV + wv) * 2 + half
    const int nsr = hg.gw * C::WV * 2;
    const int sidx = (col * C::WV + wv) * 2 + half;
    constexpr int REC = 3 + 3 * L;
#pragma unroll
    for (int rt = 0; rt < C::TR; ++rt) {
        const int row = row0 + (wr * C::TR + rt) * 32 + l32;
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

// ---------------------------------------------------------------------------
// launchers

using CfgMid = TileCfg<2, 2, 2, 4>;      // 128 rows x 256 columns per block, rows > 64
using CfgSmall = TileCfg<1, 4, 2, 2>;    //  64 rows; also the down-projection tile

int mfma_rows_per_tile(int rows) { return rows > 64 ? CfgMid::RT : CfgSmall::RT; }
int mfma_streams_per_block(int rows) { return 2 * (rows > 64 ? CfgMid::WV : CfgSmall::WV); }
int mfma_cols_per_wave(int rows) { return rows > 64 ? CfgMid::TV : CfgSmall::TV; }

template <class C>
static hipError_t set_lds(const void *fn) {
    return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
}

hipError_t launch_down_gemm(const uint16_t *h, const uint16_t *A, float *part, int rows, int rows_pad, int d, int r,
                            int slices, int kslice, hipStream_t st)
{
    using C = CfgSmall;
    auto fn = down_gemm_kernel<C>;
    hipError_t e = set_lds<C>(reinterpret_cast<const void *>(fn));
    if (e != hipSuccess) return e;
    dim3 grid((r + kNT - 1) / kNT, (rows + C::RT - 1) / C::RT, slices);
    fn<<<grid, C::THREADS, C::LDS_BYTES, st>>>(h, A, part, rows, rows_pad, d, r, kslice);
    return hipGetLastError();
}

hipError_t launch_down_finish(const float *part, int slices, int rows, int rows_pad, int r,
                              float *t32, void *t16, float2 *stat, const uint16_t *B, int V, float *brms,
                              int xmode, hipStream_t st)
{
    dim3 grid(rows_pad / 64 + 1, 2 * ((r + 63) / 64));
    down_finish_kernel<<<grid, 256, 0, st>>>(part, slices, rows, rows_pad, r, t32,
                                             static_cast<uint4 *>(t16), stat, B, V, brms, xmode);
    return hipGetLastError();
}

template <class C, bool F16, bool XROW, int L>
static hipError_t launch_head_cfg(const uint16_t *X, const uint16_t *M, float *part, int rows, int rows_pad,
                                  int K, int V, int n_rb, int gw, hipStream_t st)
{
    auto fn = head_mfma_kernel<C, F16, XROW, L>;
    hipError_t e = set_lds<C>(reinterpret_cast<const void *>(fn));
    if (e != hipSuccess) return e;
    HeadGrid hg{n_rb, gw, (V + kNT - 1) / kNT};
    fn<<<n_rb * gw, C::THREADS, C::LDS_BYTES, st>>>(X, M, part, rows, rows_pad, K, V, hg);
    return hipGetLastError();
}

hipError_t launch_head_mfma(const uint16_t *X, bool x_row_major, const uint16_t *M, float *part,
                            int rows, int rows_pad, int K, int V, int n_rb, int gw, hipStream_t st)
{
    constexpr int L = kStreamList;
#define SLIMSPEC_HEAD(C)                                                                              \
    (x_row_major ? launch_head_cfg<C, false, true, L>(X, M, part, rows, rows_pad, K, V, n_rb, gw, st)  \
                 : launch_head_cfg<C, true, false, L>(X, M, part, rows, rows_pad, K, V, n_rb, gw, st))
    if (rows > 64) return SLIMSPEC_HEAD(CfgMid);
    return SLIMSPEC_HEAD(CfgSmall);
#undef SLIMSPEC_HEAD
}

}  // namespace slimspec

// Down-projection t = h A for calls with many rows (paper section 4.1, the first of the two dense products).
//
//   down_gemm_kernel     partial sums of t over a slice of d (bf16 MFMA, fp32 accumulate)
//   down_finish_kernel   fixed-order sum of the slices -> fp32 t, the 16-bit t in the k-grouped layout the
//                        up-projection kernel reads, per-row rounding statistics, an rms estimate of B
#include "mfma_core.hpp"
#include "launch.hpp"
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
    load_x_regs<C>(xr, h, kend, d, rows, kbeg, row0, tid);
    store_m_lds<C>(mr, lds, tid);
    store_x_lds<C>(xr, lds + C::M_VECS, tid);
    __syncthreads();
    for (int kb = 0; kb < nkb; ++kb) {
        uint4 *cur = lds + (kb & 1) * C::STAGE_VECS, *nxt = lds + ((kb + 1) & 1) * C::STAGE_VECS;
        const bool more = kb + 1 < nkb;
        if (more) {
            load_m_regs<C>(mr, A, kend, r, kbeg + (kb + 1) * kKB, n0, tid);
            load_x_regs<C>(xr, h, kend, d, rows, kbeg + (kb + 1) * kKB, row0, tid);
        }
        mma_stage<C>(acc, cur, cur + C::M_VECS, wr, wv, lane, kb == 0);
        if (more) {
            store_m_lds<C>(mr, nxt, tid);
            store_x_lds<C>(xr, nxt + C::M_VECS, tid);
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
//   t16   [8 ceil(r / 64), rows_pad]   16-byte vectors of 8 values t log2(e) in bf16 or f16 (round to nearest even),
//                                      zero for k >= r
//   stat  [2 ceil(r / 64), rows_pad]   per block column: (sum of (t - its 16-bit value)^2, sum of t^2) of its 32 entries
//   brms  [1]                 sqrt(mean of B^2 over a fixed sample of entries)
constexpr int kBrmsPositions = 4;

__global__ __launch_bounds__(256) void down_finish_kernel(
    const float *__restrict__ part, int slices, int rows, int rows_pad, int r,
    float *__restrict__ t32, uint4 *__restrict__ t16, float2 *__restrict__ stat,
    const uint16_t *__restrict__ B, int V, float *__restrict__ brms, bool as_f16)
{
    __shared__ float red_a[4][64], red_b[4][64];
    const int tid = threadIdx.x, lane = tid & 63, kgl = tid >> 6;
    if ((int)blockIdx.x * 64 >= rows_pad) {
        if (blockIdx.y != 0) return;
        // sample: 8 adjacent entries of every row of B at a few column positions spread over V
        // (the sample is cold in HBM: eight independent loads per thread at a time, not one after the other)
        float a = 0.f;
        const int n_sample = r * kBrmsPositions;
        for (int q0 = tid; q0 < n_sample; q0 += 8 * 256) {
            uint4 w[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int q = min(q0 + u * 256, n_sample - 1);
                const int j = q / kBrmsPositions, pos = q % kBrmsPositions;
                const int col = (int)(((long long)pos * (V / 8)) / kBrmsPositions) * 8;
                w[u] = *reinterpret_cast<const uint4 *>(B + (size_t)j * V + col);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (q0 + u * 256 >= n_sample) continue;
                const float f[8] = {bf16_lo(w[u].x), bf16_hi(w[u].x), bf16_lo(w[u].y), bf16_hi(w[u].y),
                                    bf16_lo(w[u].z), bf16_hi(w[u].z), bf16_lo(w[u].w), bf16_hi(w[u].w)};
#pragma unroll
                for (int e = 0; e < 8; ++e) a += f[e] * f[e];
            }
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
            // fixed order of the adds; the loads of 16 slices are in flight together (they come from the
            // memory-side cache: a round trip per slice would cost more than the sums)
            constexpr int SB = 16;
            for (int s0 = 0; s0 < slices; s0 += SB) {
                float w[SB][8];
#pragma unroll
                for (int u = 0; u < SB; ++u) {
                    const float *src = part + ((size_t)min(s0 + u, slices - 1) * r + kg * 8) * rows_pad + row;
#pragma unroll
                    for (int e = 0; e < 8; ++e) w[u][e] = src[(size_t)e * rows_pad];
                }
#pragma unroll
                for (int u = 0; u < SB; ++u)
                    if (s0 + u < slices) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] += w[u][e];
                    }
            }
        }
        float4 *o = reinterpret_cast<float4 *>(t32 + (size_t)row * r + kg * 8);
        o[0] = make_float4(v[0], v[1], v[2], v[3]);
        o[1] = make_float4(v[4], v[5], v[6], v[7]);
        if (!as_f16) {
            uint32_t hb[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                // bf16 operand of the head kernel, in base-2 units: t log2(e)
                const uint32_t u = __float_as_uint(v[e] * kLog2e);
                hb[e] = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;            // round to nearest even
                const float dlt = v[e] - __uint_as_float(hb[e] << 16) * kLn2;
                a += dlt * dlt;
                b += v[e] * v[e];
            }
            t16[(size_t)kg * rows_pad + row] = make_uint4(hb[0] | (hb[1] << 16), hb[2] | (hb[3] << 16),
                                                          hb[4] | (hb[5] << 16), hb[6] | (hb[7] << 16));
        } else {
            // f16 operand, also t log2(e)
            f16x8 hv;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                hv[e] = (_Float16)(v[e] * kLog2e);
                const float dlt = v[e] - (float)hv[e] * kLn2;
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

// ---------------------------------------------------------------------------
// launchers

using CfgSmall = TileCfg<1, 4, 2, 2>;    // 64 rows x 256 columns of t per block, 4 wavefronts

template <class C>
static hipError_t set_lds(const void *fn) {
    static LdsLimit lds_limit;
    return lds_limit.raise(fn, C::LDS_BYTES);
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
                              bool as_f16, hipStream_t st)
{
    dim3 grid(rows_pad / 64 + 1, 2 * ((r + 63) / 64));
    down_finish_kernel<<<grid, 256, 0, st>>>(part, slices, rows, rows_pad, r, t32,
                                             static_cast<uint4 *>(t16), stat, B, V, brms, as_f16);
    return hipGetLastError();
}

}  // namespace slimspec

// Streaming ("lane owns columns") kernels for calls with few rows, where the head
// is bound by reading the weight matrix once from HBM (paper section 4.1: the
// O(rd + Vr) low-rank head and the O(Vd) full head).
//
//   down_items_kernel     t = h A as slices over d, one block per (64 columns of A) x (slice of d)
//   widen_rows_kernel     bf16 h -> fp32 (contraction input of the full head)
//   stream_topk_kernel    z[:, chunk] = x M[:, chunk] for a 512-column chunk, then the
//                         chunk's running max, sum of exp and top-k, one partial per
//                         (row, chunk); no logit is written to memory
#include "gemv_parts.hpp"
#include "launch.hpp"

namespace slimspec {

// ---------------------------------------------------------------------------
// t = h A for up to R rows, as slices: block = one item (64 columns of A x a slice of d, read as
// full 128-byte lines); tpart is [nds][R][r] and the consumer adds the nds slices in order.
constexpr int kDownThreads = 1024;

template <int R, bool POS>
__global__ __launch_bounds__(kDownThreads) void down_items_kernel(
    const uint16_t *__restrict__ h, const uint16_t *__restrict__ A, float *__restrict__ tpart,
    int rows_here, int d, int r, int n_cb, int slice, RowMats mats)
{
    __shared__ float redd[kDownThreads / 64][R][kItemCols];
    down_item<R, kDownThreads, POS>(redd, h, A, tpart, blockIdx.x, n_cb, slice, rows_here, d, r, threadIdx.x, mats);
}

__global__ __launch_bounds__(256) void widen_rows_kernel(
    const uint16_t *__restrict__ h, float *__restrict__ x, int n)
{
    int e = blockIdx.x * 256 + threadIdx.x;
    if (e < n) x[e] = bf16_to_float(h[e]);
}

// ---------------------------------------------------------------------------
// One block per 512-column chunk of the vocabulary.  x is the fp32 contraction
// input [R, K] (t or h), M the [K, V] weight matrix (bf16 or fp32).  The NW
// wavefronts split K; every lane owns 8 adjacent columns and keeps R x 8 fp32
// accumulators.  After a fixed-order sum over the wavefronts, wavefront i % NW
// reduces row i of the chunk to (max, sum of exp, top-k) and writes the partial.
//
// SLICES: x is not the contraction input itself but nds partial sums of it, [nds][R][K] (the
// slices of t left by down_items_kernel); the block first adds them, in slice order, into shared
// memory.  The first weight rows are requested before that, so the adds hide behind them.
template <int R, int NW, typename WT, bool SLICES>
__global__ __launch_bounds__(NW * 64) void stream_topk_kernel(
    const float *__restrict__ x, int nds, const WT *__restrict__ M,
    float2 *__restrict__ part_ms, float *__restrict__ part_val, int *__restrict__ part_id,
    int rows_here, int row0, int K, int V, int chunks, int lanes, int k,
    float4 *__restrict__ part_smp, uint32_t seed_lo, uint32_t seed_hi)
{
    extern __shared__ __align__(16) unsigned char dyn[];         // ChunkLds, then (SLICES) t as fp32 [R][K]
    ChunkLds<R, NW> &L = *reinterpret_cast<ChunkLds<R, NW> *>(dyn);
    float *xs = reinterpret_cast<float *>(dyn + sizeof(ChunkLds<R, NW>));
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int chunk = blockIdx.x;
    const int col = (chunk * lanes + lane) * 8;             // the chunk covers 8 * lanes adjacent columns
    const bool active = lane < lanes && col < V;          // V is a multiple of 8: all 8 columns valid or none

    float acc[R][8];
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[i][e] = 0.f;

    // rows [j0, j1) of M for this wavefront
    const int per = ((K + NW - 1) / NW + 7) & ~7;            // multiple of 8: keeps 8-wide reads of x aligned
    const int j0 = min(K, wave * per), j1 = min(K, j0 + per);
    constexpr int U = (sizeof(WT) == 2 && R <= 2) ? 16 : 8;
    using RawT = decltype(load_raw8(static_cast<const WT *>(nullptr)));
    const WT *base = M + (active ? col : 0);

    if constexpr (SLICES) {
        // slices of t first (they come from L2), then the first batch of weight rows, then the adds
        constexpr int NT = NW * 64;
        constexpr int PER_T = 8;
        const size_t stride = (size_t)R * K;
        RawT q0[U];
        const bool first_full = active && (j0 + U <= j1);
        for (int e0 = 0; e0 < R * K; e0 += NT) {
            const int e = e0 + threadIdx.x;
            float s = 0.f;
            if (e < R * K) {
                int ds = 0;
                for (; ds + PER_T <= nds; ds += PER_T) {
                    float v[PER_T];
#pragma unroll
                    for (int u = 0; u < PER_T; ++u) v[u] = x[(size_t)(ds + u) * stride + e];
#pragma unroll
                    for (int u = 0; u < PER_T; ++u) s += v[u];
                }
                for (; ds < nds; ++ds) s += x[(size_t)ds * stride + e];
                xs[e] = s;
            }
        }
        if (first_full) {
#pragma unroll
            for (int u = 0; u < U; ++u) q0[u] = load_raw8(base + (size_t)(j0 + u) * V);
        }
        __syncthreads();
        auto fma_batch = [&](const RawT (&q)[U], int j) {
#pragma unroll
            for (int g = 0; g < U / 8; ++g) {
                float xv[R][8];
#pragma unroll
                for (int i = 0; i < R; ++i) {
                    const float4 *p = reinterpret_cast<const float4 *>(xs + i * K + j + 8 * g);
                    const float4 a = p[0], b = p[1];
                    xv[i][0] = a.x; xv[i][1] = a.y; xv[i][2] = a.z; xv[i][3] = a.w;
                    xv[i][4] = b.x; xv[i][5] = b.y; xv[i][6] = b.z; xv[i][7] = b.w;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    float f[8];
                    widen8(q[8 * g + u], f);
#pragma unroll
                    for (int i = 0; i < R; ++i)
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[i][e] = fmaf(xv[i][u], f[e], acc[i][e]);
                }
            }
        };
        if (active) {
            int j = j0;
            if (first_full) { fma_batch(q0, j); j += U; }
            for (; j + U <= j1; j += U) {
                RawT q[U];
#pragma unroll
                for (int u = 0; u < U; ++u) q[u] = load_raw8(base + (size_t)(j + u) * V);
                fma_batch(q, j);
            }
            for (; j < j1; ++j) {
                float f[8];
                widen8(load_raw8(base + (size_t)j * V), f);
#pragma unroll
                for (int i = 0; i < R; ++i) {
                    const float xv = xs[i * K + j];
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[i][e] = fmaf(xv, f[e], acc[i][e]);
                }
            }
        }
    } else if (active) {
        int j = j0;
        for (; j + U <= j1; j += U) {
            RawT q[U];
#pragma unroll
            for (int u = 0; u < U; ++u) q[u] = load_raw8(base + (size_t)(j + u) * V);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float f[8];
                widen8(q[u], f);
#pragma unroll
                for (int i = 0; i < R; ++i) {
                    float xv = x[(size_t)i * K + j + u];
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[i][e] = fmaf(xv, f[e], acc[i][e]);
                }
            }
        }
        for (; j < j1; ++j) {
            float f[8];
            widen8(load_raw8(base + (size_t)j * V), f);
#pragma unroll
            for (int i = 0; i < R; ++i) {
                float xv = x[(size_t)i * K + j];
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[i][e] = fmaf(xv, f[e], acc[i][e]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < R; ++i) {
        float4 *dst = reinterpret_cast<float4 *>(&L.red[wave][i][lane * 8]);
        dst[0] = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
        dst[1] = make_float4(acc[i][4], acc[i][5], acc[i][6], acc[i][7]);
    }
    __syncthreads();
    for (int i = wave; i < rows_here; i += NW)
        chunk_row_epilogue<R, NW>(L, i, wave, lane, active, col, k, (size_t)(row0 + i) * chunks + chunk,
                                  part_ms, part_val, part_id, part_smp, gumbel_key(seed_lo, seed_hi, (uint32_t)(row0 + i)));
}

// ---------------------------------------------------------------------------
// launchers

template <int R>
static hipError_t launch_down(const uint16_t *h, const uint16_t *A, float *tpart,
                              int rows_here, int d, int r, const DownPlan &fp, const int *mat_of_row, hipStream_t st)
{
    RowMats mats{};
    bool one_matrix = true;
    for (int i = 0; i < rows_here && i < 8; ++i) {
        mats.m[i] = mat_of_row ? mat_of_row[i] : 0;
        one_matrix = one_matrix && mats.m[i] == mats.m[0];
    }
    if (one_matrix)        // every row uses the same matrix: the weights are loaded once for all rows
        down_items_kernel<R, false><<<fp.n_items, kDownThreads, 0, st>>>(h, A + (size_t)mats.m[0] * d * r, tpart, rows_here, d, r,
                                                                         fp.n_cb, fp.slice, mats);
    else
        down_items_kernel<R, true><<<fp.n_items, kDownThreads, 0, st>>>(h, A, tpart, rows_here, d, r, fp.n_cb, fp.slice, mats);
    return hipGetLastError();
}

hipError_t launch_down_projection(const uint16_t *h, const uint16_t *A, float *tpart,
                                  int rows_here, int d, int r, const DownPlan &fp, const int *mat_of_row, hipStream_t st)
{
    if (rows_here <= 1) return launch_down<1>(h, A, tpart, rows_here, d, r, fp, mat_of_row, st);
    if (rows_here <= 2) return launch_down<2>(h, A, tpart, rows_here, d, r, fp, mat_of_row, st);
    if (rows_here <= 4) return launch_down<4>(h, A, tpart, rows_here, d, r, fp, mat_of_row, st);
    return launch_down<8>(h, A, tpart, rows_here, d, r, fp, mat_of_row, st);
}

hipError_t launch_widen_rows(const uint16_t *h, float *x, int n, hipStream_t st)
{
    widen_rows_kernel<<<(n + 255) / 256, 256, 0, st>>>(h, x, n);
    return hipGetLastError();
}

constexpr size_t kStreamLdsLimit = 150 * 1024;      // of the CU's 160 KB

template <int R, int NW>
constexpr size_t stream_lds_bytes(bool slices, int K) {
    return sizeof(ChunkLds<R, NW>) + (slices ? sizeof(float) * (size_t)R * K : 0);
}

template <int R, int NW, typename WT>
static hipError_t launch_stream(const float *x, int nds, const WT *M, float2 *ms, float *pv, int *pi,
                                int rows_here, int row0, int K, int V, int chunks, int lanes, int k,
                                float4 *smp, uint32_t seed_lo, uint32_t seed_hi, hipStream_t st)
{
    static_assert(sizeof(ChunkLds<R, NW>) % 16 == 0, "t follows the struct in shared memory");
    const size_t dyn = stream_lds_bytes<R, NW>(nds > 0, K);
    const void *fn = nds > 0 ? reinterpret_cast<const void *>(stream_topk_kernel<R, NW, WT, true>)
                             : reinterpret_cast<const void *>(stream_topk_kernel<R, NW, WT, false>);
    if (dyn > 32 * 1024) {
        static LdsLimit lds_limit[2];
        hipError_t e = lds_limit[nds > 0 ? 1 : 0].raise(fn, (int)dyn);
        if (e != hipSuccess) return e;
    }
    if (nds > 0)
        stream_topk_kernel<R, NW, WT, true><<<chunks, NW * 64, dyn, st>>>(x, nds, M, ms, pv, pi, rows_here, row0, K, V, chunks, lanes, k,
                                                                          smp, seed_lo, seed_hi);
    else
        stream_topk_kernel<R, NW, WT, false><<<chunks, NW * 64, dyn, st>>>(x, 0, M, ms, pv, pi, rows_here, row0, K, V, chunks, lanes, k,
                                                                           smp, seed_lo, seed_hi);
    return hipGetLastError();
}

template <typename WT>
static hipError_t launch_stream_rows(const float *x, int nds, const WT *M, float2 *ms, float *pv, int *pi,
                                     int rows_here, int row0, int K, int V, int chunks, int lanes, int nw1, int k,
                                     float4 *smp, uint32_t seed_lo, uint32_t seed_hi, hipStream_t st)
{
#define SLIMSPEC_STREAM(R, NW) launch_stream<R, NW, WT>(x, nds, M, ms, pv, pi, rows_here, row0, K, V, chunks, lanes, k, smp, seed_lo, seed_hi, st)
#define SLIMSPEC_FITS(R, NW) (stream_lds_bytes<R, NW>(nds > 0, K) <= kStreamLdsLimit)
    // One row: the block size the chunk geometry asks for.  More rows: as many wavefronts as the shared memory of
    // the partial sums (NW * R * 2 KB) allows; they split the contraction, and every one of them keeps loads in flight.
    if (rows_here <= 1) return nw1 == 4 ? SLIMSPEC_STREAM(1, 4) : nw1 == 8 ? SLIMSPEC_STREAM(1, 8) : SLIMSPEC_STREAM(1, 16);
    if (rows_here <= 2) return SLIMSPEC_FITS(2, 16) ? SLIMSPEC_STREAM(2, 16) : SLIMSPEC_STREAM(2, 8);
    if (rows_here <= 4) return SLIMSPEC_FITS(4, 8) ? SLIMSPEC_STREAM(4, 8) : SLIMSPEC_STREAM(4, 4);
    return SLIMSPEC_FITS(8, 4) ? SLIMSPEC_STREAM(8, 4) : SLIMSPEC_STREAM(8, 2);
#undef SLIMSPEC_FITS
#undef SLIMSPEC_STREAM
}

// nds > 0: x holds nds slices [nds][R][K] of the contraction input (R = 1, 2, 4 or 8 as chosen for rows_here)
hipError_t launch_stream_topk(const float *x, int nds, const void *M, bool m_is_f32, float2 *ms, float *pv, int *pi,
                              int rows_here, int row0, int K, int V, int chunks, int lanes, int nw1, int k,
                              float4 *smp, uint32_t seed_lo, uint32_t seed_hi, hipStream_t st)
{
    if (m_is_f32)
        return launch_stream_rows<float>(x, nds, (const float *)M, ms, pv, pi, rows_here, row0, K, V, chunks, lanes, nw1, k, smp, seed_lo, seed_hi, st);
    return launch_stream_rows<uint16_t>(x, nds, (const uint16_t *)M, ms, pv, pi, rows_here, row0, K, V, chunks, lanes, nw1, k, smp, seed_lo, seed_hi, st);
}

}  // namespace slimspec

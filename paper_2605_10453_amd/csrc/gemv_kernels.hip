// Streaming ("lane owns columns") kernels for calls with few rows, where the head
// is bound by reading the weight matrix once from HBM (paper section 4.1: the
// O(rd + Vr) low-rank head and the O(Vd) full head).
//
//   down_partial_kernel   t = h A, split over d into partial sums
//   down_reduce_kernel    fixed-order sum of the partials -> fp32 t
//   widen_rows_kernel     bf16 h -> fp32 (contraction input of the full head)
//   stream_topk_kernel    z[:, chunk] = x M[:, chunk] for a 512-column chunk, then the
//                         chunk's running max, sum of exp and top-k, one partial per
//                         (row, chunk); no logit is written to memory
#include "device_utils.hpp"
#include "launch.hpp"

namespace slimspec {

// ---------------------------------------------------------------------------
// t = h A, partial over a slice of d.  A is [d, r] row-major bf16; a lane owns 8
// adjacent columns of A (one 128-bit load per row), a wavefront covers 512
// columns, the four wavefronts of a block take interleaved rows of the slice.
// part is [splits, kGemvMaxRows, r] fp32.
template <int R>
__global__ __launch_bounds__(256) void down_partial_kernel(
    const uint16_t *__restrict__ h, const uint16_t *__restrict__ A, float *__restrict__ part,
    int rows_here, int d, int r)
{
    __shared__ float hs[R][kDownSplitRows];
    __shared__ float red[4][kChunkCols];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int c0 = blockIdx.x * kDownSplitRows;
    const int nc = min(kDownSplitRows, d - c0);
    const int col = (blockIdx.y * kWave + lane) * 8;
    const bool active = col < r;

    for (int e = threadIdx.x; e < R * kDownSplitRows; e += 256) {
        int i = e / kDownSplitRows, c = e % kDownSplitRows;
        hs[i][c] = (i < rows_here && c < nc) ? bf16_to_float(h[(size_t)i * d + c0 + c]) : 0.f;
    }
    __syncthreads();

    float acc[R][8];
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[i][e] = 0.f;

    if (active) {
        constexpr int PER_WAVE = kDownSplitRows / 4;
        uint4 w[PER_WAVE];
#pragma unroll
        for (int u = 0; u < PER_WAVE; ++u) {
            int c = wave + 4 * u;
            w[u] = (c < nc) ? *reinterpret_cast<const uint4 *>(A + (size_t)(c0 + c) * r + col)
                            : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < PER_WAVE; ++u) {
            int c = wave + 4 * u;
            float f[8] = {bf16_lo(w[u].x), bf16_hi(w[u].x), bf16_lo(w[u].y), bf16_hi(w[u].y),
                          bf16_lo(w[u].z), bf16_hi(w[u].z), bf16_lo(w[u].w), bf16_hi(w[u].w)};
#pragma unroll
            for (int i = 0; i < R; ++i) {
                float hv = hs[i][c];
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[i][e] = fmaf(hv, f[e], acc[i][e]);
            }
        }
    }
    // fixed-order sum over the four wavefronts, one row of t at a time
#pragma unroll
    for (int i = 0; i < R; ++i) {
#pragma unroll
        for (int e = 0; e < 8; ++e) red[wave][lane * 8 + e] = acc[i][e];
        __syncthreads();
        for (int cc = threadIdx.x; cc < kChunkCols; cc += 256) {
            int j = blockIdx.y * kChunkCols + cc;
            if (j < r) {
                float s = ((red[0][cc] + red[1][cc]) + red[2][cc]) + red[3][cc];
                part[((size_t)blockIdx.x * kGemvMaxRows + i) * r + j] = s;
            }
        }
        __syncthreads();
    }
}

// t[i][j] = sum over splits, in split order.  t is fp32 [kGemvMaxRows, r].
__global__ __launch_bounds__(256) void down_reduce_kernel(
    const float *__restrict__ part, float *__restrict__ t, int splits, int r, int rows_here)
{
    int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= rows_here * r) return;
    int i = e / r, j = e % r;
    float s = 0.f;
    for (int sp = 0; sp < splits; ++sp) s += part[((size_t)sp * kGemvMaxRows + i) * r + j];
    t[(size_t)i * r + j] = s;
}

__global__ __launch_bounds__(256) void widen_rows_kernel(
    const uint16_t *__restrict__ h, float *__restrict__ x, int n)
{
    int e = blockIdx.x * 256 + threadIdx.x;
    if (e < n) x[e] = bf16_to_float(h[e]);
}

// ---------------------------------------------------------------------------
// Load 8 adjacent columns of one matrix row as floats.
__device__ __forceinline__ void load8(const uint16_t *p, float (&f)[8]) {
    uint4 w = *reinterpret_cast<const uint4 *>(p);
    f[0] = bf16_lo(w.x); f[1] = bf16_hi(w.x); f[2] = bf16_lo(w.y); f[3] = bf16_hi(w.y);
    f[4] = bf16_lo(w.z); f[5] = bf16_hi(w.z); f[6] = bf16_lo(w.w); f[7] = bf16_hi(w.w);
}
__device__ __forceinline__ void load8(const float *p, float (&f)[8]) {
    float4 a = *reinterpret_cast<const float4 *>(p);
    float4 b = *reinterpret_cast<const float4 *>(p + 4);
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
}

// One block per 512-column chunk of the vocabulary.  x is the fp32 contraction
// input [R, K] (t or h), M the [K, V] weight matrix (bf16 or fp32).  The NW
// wavefronts split K; every lane owns 8 adjacent columns and keeps R x 8 fp32
// accumulators.  After a fixed-order sum over the wavefronts, wavefront i % NW
// reduces row i of the chunk to (max, sum of exp, top-k) and writes the partial.
template <int R, int NW, typename WT>
__global__ __launch_bounds__(NW * 64) void stream_topk_kernel(
    const float *__restrict__ x, const WT *__restrict__ M,
    float2 *__restrict__ part_ms, float *__restrict__ part_val, int *__restrict__ part_id,
    int rows_here, int row0, int K, int V, int chunks, int k)
{
    __shared__ float red[NW][R][kChunkCols];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int chunk = blockIdx.x;
    const int col = chunk * kChunkCols + lane * 8;
    const bool active = col < V;          // V is a multiple of 8: all 8 columns valid or none

    float acc[R][8];
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[i][e] = 0.f;

    // rows [j0, j1) of M for this wavefront
    const int per = (K + NW - 1) / NW;
    const int j0 = min(K, wave * per), j1 = min(K, j0 + per);
    if (active) {
        constexpr int U = 8;
        const WT *base = M + col;
        int j = j0;
        for (; j + U <= j1; j += U) {
            float f[U][8];
#pragma unroll
            for (int u = 0; u < U; ++u) load8(base + (size_t)(j + u) * V, f[u]);
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < R; ++i) {
                    float xv = x[(size_t)i * K + j + u];
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[i][e] = fmaf(xv, f[u][e], acc[i][e]);
                }
        }
        for (; j < j1; ++j) {
            float f[8];
            load8(base + (size_t)j * V, f);
#pragma unroll
            for (int i = 0; i < R; ++i) {
                float xv = x[(size_t)i * K + j];
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[i][e] = fmaf(xv, f[e], acc[i][e]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) red[wave][i][lane * 8 + e] = acc[i][e];
    __syncthreads();

    for (int i = wave; i < rows_here; i += NW) {
        float z[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float s = red[0][i][lane * 8 + e];
#pragma unroll
            for (int w = 1; w < NW; ++w) s += red[w][i][lane * 8 + e];
            z[e] = active ? s : kNegInf;
        }
        // running max and sum of exp of the chunk
        float m = z[0];
#pragma unroll
        for (int e = 1; e < 8; ++e) m = fmaxf(m, z[e]);
        m = wave_max(m);
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s += fast_exp(z[e] - m);     // exp(-inf) = 0 for padding lanes
        s = wave_sum(s);

        // top-k of the chunk: k rounds of "first in order among what is left"
        unsigned alive = active ? 0xffu : 0u;
        float keep_v = kNegInf;
        int keep_i = kNoId;
        for (int p = 0; p < k; ++p) {
            float bv = kNegInf;
            int bi = kNoId;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                bool ok = (alive >> e) & 1u;
                if (ok && ranks_before(z[e], col + e, bv, bi)) { bv = z[e]; bi = col + e; }
            }
            wave_first(bv, bi);
            if (lane == p) { keep_v = bv; keep_i = bi; }
            if (bi != kNoId && (bi >> 3) == (col >> 3)) alive &= ~(1u << (bi & 7));
        }
        const size_t slot = (size_t)(row0 + i) * chunks + chunk;
        if (lane < k) {
            part_val[slot * k + lane] = keep_v;
            part_id[slot * k + lane] = keep_i;
        }
        if (lane == 0) part_ms[slot] = make_float2(m, s);
    }
}

// ---------------------------------------------------------------------------
// launchers

template <int R>
static hipError_t launch_down(const uint16_t *h, const uint16_t *A, float *part, float *t,
                              int rows_here, int d, int r, int splits, hipStream_t st)
{
    dim3 grid(splits, (r / 8 + kWave - 1) / kWave);
    down_partial_kernel<R><<<grid, 256, 0, st>>>(h, A, part, rows_here, d, r);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    int n = rows_here * r;
    down_reduce_kernel<<<(n + 255) / 256, 256, 0, st>>>(part, t, splits, r, rows_here);
    return hipGetLastError();
}

hipError_t launch_down_projection(const uint16_t *h, const uint16_t *A, float *part, float *t,
                                  int rows_here, int d, int r, int splits, hipStream_t st)
{
    if (rows_here <= 1) return launch_down<1>(h, A, part, t, rows_here, d, r, splits, st);
    if (rows_here <= 2) return launch_down<2>(h, A, part, t, rows_here, d, r, splits, st);
    if (rows_here <= 4) return launch_down<4>(h, A, part, t, rows_here, d, r, splits, st);
    return launch_down<8>(h, A, part, t, rows_here, d, r, splits, st);
}

hipError_t launch_widen_rows(const uint16_t *h, float *x, int n, hipStream_t st)
{
    widen_rows_kernel<<<(n + 255) / 256, 256, 0, st>>>(h, x, n);
    return hipGetLastError();
}

template <int R, int NW, typename WT>
static hipError_t launch_stream(const float *x, const WT *M, float2 *ms, float *pv, int *pi,
                                int rows_here, int row0, int K, int V, int chunks, int k, hipStream_t st)
{
    stream_topk_kernel<R, NW, WT><<<chunks, NW * 64, 0, st>>>(x, M, ms, pv, pi, rows_here, row0, K, V, chunks, k);
    return hipGetLastError();
}

template <typename WT>
static hipError_t launch_stream_rows(const float *x, const WT *M, float2 *ms, float *pv, int *pi,
                                     int rows_here, int row0, int K, int V, int chunks, int k, hipStream_t st)
{
    // shared memory is NW * R * 2 KB: keep it at 32 KB
    if (rows_here <= 1) return launch_stream<1, 16, WT>(x, M, ms, pv, pi, rows_here, row0, K, V, chunks, k, st);
    if (rows_here <= 2) return launch_stream<2, 8, WT>(x, M, ms, pv, pi, rows_here, row0, K, V, chunks, k, st);
    if (rows_here <= 4) return launch_stream<4, 4, WT>(x, M, ms, pv, pi, rows_here, row0, K, V, chunks, k, st);
    return launch_stream<8, 2, WT>(x, M, ms, pv, pi, rows_here, row0, K, V, chunks, k, st);
}

hipError_t launch_stream_topk(const float *x, const void *M, bool m_is_f32, float2 *ms, float *pv, int *pi,
                              int rows_here, int row0, int K, int V, int chunks, int k, hipStream_t st)
{
    if (m_is_f32)
        return launch_stream_rows<float>(x, (const float *)M, ms, pv, pi, rows_here, row0, K, V, chunks, k, st);
    return launch_stream_rows<uint16_t>(x, (const uint16_t *)M, ms, pv, pi, rows_here, row0, K, V, chunks, k, st);
}

}  // namespace slimspec

// Streaming ("lane owns columns") kernels for calls with few rows, where the head
// is bound by reading the weight matrix once from HBM (paper section 4.1: the
// O(rd + Vr) low-rank head and the O(Vd) full head).
//
//   down_strip_kernel     t = h A, one block per strip of 8 columns of A over all of d
//   widen_rows_kernel     bf16 h -> fp32 (contraction input of the full head)
//   stream_topk_kernel    z[:, chunk] = x M[:, chunk] for a 512-column chunk, then the
//                         chunk's running max, sum of exp and top-k, one partial per
//                         (row, chunk); no logit is written to memory
#include "gemv_parts.hpp"
#include "launch.hpp"

namespace slimspec {

// ---------------------------------------------------------------------------
// t = h A for up to R rows.  A is [d, r] row-major bf16.  Block b owns columns
// [8b, 8b + 8) (one 128-bit load per row of A); its 1024 threads take the rows of A
// c = tid, tid + 1024, ... and the partial sums are combined in a fixed order: lanes
// of a wavefront by the DPP butterfly, wavefronts in index order.  t is fp32 [R, r].
constexpr int kDownThreads = 1024;

template <int R>
__global__ __launch_bounds__(kDownThreads) void down_strip_kernel(
    const uint16_t *__restrict__ h, const uint16_t *__restrict__ A, float *__restrict__ t,
    int rows_here, int d, int r)
{
    __shared__ float red[kDownThreads / 64][R * 8];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    // blocks are dealt round-robin to the 8 XCDs: give each XCD a contiguous run of strips
    // so that the 128-byte lines of A it touches are used in full inside its own L2
    const int nstrips = r / 8;
    const int per_xcd = gridDim.x / 8;              // the grid is 8 * ceil(nstrips / 8) blocks
    const int strip = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (strip >= nstrips) return;
    const int col = strip * 8;

    float acc[R][8];
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[i][e] = 0.f;

    constexpr int U = 4;
    for (int c0 = tid; c0 < d; c0 += kDownThreads * U) {
        uint4 w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int c = c0 + u * kDownThreads;
            w[u] = (c < d) ? *reinterpret_cast<const uint4 *>(A + (size_t)c * r + col) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int c = c0 + u * kDownThreads;
            float f[8] = {bf16_lo(w[u].x), bf16_hi(w[u].x), bf16_lo(w[u].y), bf16_hi(w[u].y),
                          bf16_lo(w[u].z), bf16_hi(w[u].z), bf16_lo(w[u].w), bf16_hi(w[u].w)};
#pragma unroll
            for (int i = 0; i < R; ++i) {
                float hv = (c < d && i < rows_here) ? bf16_to_float(h[(size_t)i * d + c]) : 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[i][e] = fmaf(hv, f[e], acc[i][e]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float s = wave_sum(acc[i][e]);
            if (lane == 0) red[wave][i * 8 + e] = s;
        }
    __syncthreads();
    if (tid < R * 8) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < kDownThreads / 64; ++w) s += red[w][tid];
        int i = tid >> 3, e = tid & 7;
        if (i < rows_here) t[(size_t)i * r + col + e] = s;
    }
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
template <int R, int NW, typename WT>
__global__ __launch_bounds__(NW * 64) void stream_topk_kernel(
    const float *__restrict__ x, const WT *__restrict__ M,
    float2 *__restrict__ part_ms, float *__restrict__ part_val, int *__restrict__ part_id,
    int rows_here, int row0, int K, int V, int chunks, int k)
{
    __shared__ ChunkLds<R, NW> L;
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
        constexpr int U = (sizeof(WT) == 2 && R <= 2) ? 16 : 8;
        const WT *base = M + col;
        int j = j0;
        for (; j + U <= j1; j += U) {
            decltype(load_raw8(base)) q[U];
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
                                  part_ms, part_val, part_id);
}

// ---------------------------------------------------------------------------
// launchers

template <int R>
static hipError_t launch_down(const uint16_t *h, const uint16_t *A, float *t,
                              int rows_here, int d, int r, hipStream_t st)
{
    down_strip_kernel<R><<<8 * ((r / 8 + 7) / 8), kDownThreads, 0, st>>>(h, A, t, rows_here, d, r);
    return hipGetLastError();
}

hipError_t launch_down_projection(const uint16_t *h, const uint16_t *A, float *t,
                                  int rows_here, int d, int r, hipStream_t st)
{
    if (rows_here <= 1) return launch_down<1>(h, A, t, rows_here, d, r, st);
    if (rows_here <= 2) return launch_down<2>(h, A, t, rows_here, d, r, st);
    if (rows_here <= 4) return launch_down<4>(h, A, t, rows_here, d, r, st);
    return launch_down<8>(h, A, t, rows_here, d, r, st);
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

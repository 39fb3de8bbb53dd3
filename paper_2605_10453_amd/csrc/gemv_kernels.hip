// Streaming ("lane owns columns") kernels for calls with few rows, where the head
// is bound by reading the weight matrix once from HBM (paper section 4.1: the
// O(rd + Vr) low-rank head and the O(Vd) full head).
//
//   down_strip_kernel     t = h A, one block per strip of 8 columns of A over all of d
//   widen_rows_kernel     bf16 h -> fp32 (contraction input of the full head)
//   stream_topk_kernel    z[:, chunk] = x M[:, chunk] for a 512-column chunk, then the
//                         chunk's running max, sum of exp and top-k, one partial per
//                         (row, chunk); no logit is written to memory
#include "device_utils.hpp"
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
// 8 adjacent columns of one matrix row: kept as loaded (raw) while in flight, widened
// to fp32 only when consumed, so that many loads can be outstanding per lane.
struct Raw8Bf16 { uint4 w; };
struct Raw8F32 { float4 a, b; };
__device__ __forceinline__ Raw8Bf16 load_raw8(const uint16_t *p) { return {*reinterpret_cast<const uint4 *>(p)}; }
__device__ __forceinline__ Raw8F32 load_raw8(const float *p) {
    return {*reinterpret_cast<const float4 *>(p), *reinterpret_cast<const float4 *>(p + 4)};
}
__device__ __forceinline__ void widen8(const Raw8Bf16 &q, float (&f)[8]) {
    f[0] = bf16_lo(q.w.x); f[1] = bf16_hi(q.w.x); f[2] = bf16_lo(q.w.y); f[3] = bf16_hi(q.w.y);
    f[4] = bf16_lo(q.w.z); f[5] = bf16_hi(q.w.z); f[6] = bf16_lo(q.w.w); f[7] = bf16_hi(q.w.w);
}
__device__ __forceinline__ void widen8(const Raw8F32 &q, float (&f)[8]) {
    f[0] = q.a.x; f[1] = q.a.y; f[2] = q.a.z; f[3] = q.a.w; f[4] = q.b.x; f[5] = q.b.y; f[6] = q.b.z; f[7] = q.b.w;
}

// One block per 512-column chunk of the vocabulary.  x is the fp32 contraction
// input [R, K] (t or h), M the [K, V] weight matrix (bf16 or fp32).  The NW
// wavefronts split K; every lane owns 8 adjacent columns and keeps R x 8 fp32
// accumulators.  After a fixed-order sum over the wavefronts, wavefront i % NW
// reduces row i of the chunk to (max, sum of exp, top-k) and writes the partial.
//
// Top-k of a chunk in three steps whose cost does not grow with k: the k-th largest
// of the 64 lane maxima (by all-pairs counting) bounds the answer from below; the
// few elements that reach the bound are gathered in shared memory; they are ranked
// among themselves by (logit desc, id asc), again by counting.  Lanes own increasing
// columns, so ordering lane maxima by (value, lane) is consistent with ordering
// elements by (value, id): an element below the bound is preceded by k lane maxima.
template <int R, int NW, typename WT>
__global__ __launch_bounds__(NW * 64) void stream_topk_kernel(
    const float *__restrict__ x, const WT *__restrict__ M,
    float2 *__restrict__ part_ms, float *__restrict__ part_val, int *__restrict__ part_id,
    int rows_here, int row0, int K, int V, int chunks, int k)
{
    __shared__ float red[NW][R][kChunkCols];
    constexpr int EW = (R < NW) ? R : NW;           // wavefronts that run the per-row epilogue
    __shared__ uint64_t sel_keys[EW][64];
    __shared__ uint64_t sel_cand[EW][kChunkCols];
    __shared__ uint64_t sel_bound[EW];
    __shared__ uint32_t sel_cnt[EW];
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
        float4 *dst = reinterpret_cast<float4 *>(&red[wave][i][lane * 8]);
        dst[0] = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
        dst[1] = make_float4(acc[i][4], acc[i][5], acc[i][6], acc[i][7]);
    }
    __syncthreads();

    for (int i = wave; i < rows_here; i += NW) {
        float z[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {          // fixed order: wavefront 0 first
            const float4 *src = reinterpret_cast<const float4 *>(&red[w][i][lane * 8]);
            float4 a = src[0], b = src[1];
            z[0] += a.x; z[1] += a.y; z[2] += a.z; z[3] += a.w;
            z[4] += b.x; z[5] += b.y; z[6] += b.z; z[7] += b.w;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = active ? z[e] : kNegInf;

        // running max and sum of exp of the chunk
        float lm = z[0];
#pragma unroll
        for (int e = 1; e < 8; ++e) lm = fmaxf(lm, z[e]);
        const float m = wave_max(lm);
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s += fast_exp(z[e] - m);     // exp(-inf) = 0 for padding lanes
        s = wave_sum(s);

        // top-k of the chunk, without k serial rounds
        // (1) bound: the k-th largest of the 64 lane maxima, as keys (value, lane)
        uint64_t *lane_keys = sel_keys[wave];
        uint64_t *cand = sel_cand[wave];
        const uint64_t my_lane_key = active ? make_key(lm, (uint32_t)lane) : kNoKey;
        lane_keys[lane] = my_lane_key;
        if (lane == 0) { sel_cnt[wave] = 0u; sel_bound[wave] = kNoKey; }
        lds_wave_sync();
        int rank = 0;
#pragma unroll 8
        for (int q = 0; q < 64; ++q) rank += (lane_keys[q] > my_lane_key) ? 1 : 0;
        if (rank == k - 1 && my_lane_key != kNoKey) sel_bound[wave] = my_lane_key;   // keys are unique: one lane at most
        lds_wave_sync();
        const uint64_t bound = sel_bound[wave];          // kNoKey when fewer than k lanes hold columns: keep everything
        // (2) every element whose (value, lane) key reaches the bound is a candidate
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (active && make_key(z[e], (uint32_t)lane) >= bound) {
                uint32_t pos = atomicAdd(&sel_cnt[wave], 1u);
                cand[pos] = make_key(z[e], (uint32_t)(col + e));
            }
        }
        lds_wave_sync();
        const int n_cand = (int)sel_cnt[wave];
        // (3) rank the candidates among themselves by (value desc, id asc); ranks below k are the answer
        const size_t slot = (size_t)(row0 + i) * chunks + chunk;
        for (int c0 = 0; c0 < n_cand; c0 += 64) {
            const int c = c0 + lane;
            const uint64_t mine = (c < n_cand) ? cand[c] : kNoKey;
            int rk = 0;
            for (int q = 0; q < n_cand; ++q) rk += (cand[q] > mine) ? 1 : 0;
            if (c < n_cand && rk < k) {
                part_val[slot * k + rk] = key_value(mine);
                part_id[slot * k + rk] = (int)key_tiebreak(mine);
            }
        }
        if (lane >= n_cand && lane < k) {                  // fewer than k columns in this chunk
            part_val[slot * k + lane] = kNegInf;
            part_id[slot * k + lane] = kNoId;
        }
        if (lane == 0) part_ms[slot] = make_float2(m, s);
        lds_wave_sync();                                   // the buffers are reused by this wavefront's next row
    }
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

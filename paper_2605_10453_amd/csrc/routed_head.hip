// Router-then-exact head (the dynamic vocabulary selection the paper compares with, section 2): the low-rank head
// scores the whole vocabulary, the k_route best ids of every row are kept (slimspec_head_topk does that part), and the
// full head z = h W is evaluated exactly on those ids only; softmax and top-k then run over that subset.
//
//   routed_partial_kernel   block (slice of d, row): partial dot products h[row, slice] . W[slice, id] for the row's
//                           k_route ids.  A column of W is one element per row of W, each in a cache line of its own,
//                           so the gathers of one row are spread over many blocks and every thread keeps 16 in flight.
//   routed_finish_kernel    one wavefront per row: fixed-order sum of the slices, log-sum-exp over the subset, rank by
//                           (logit descending, id ascending), the k best.
#include "device_utils.hpp"
#include "launch.hpp"

namespace slimspec {

namespace {
constexpr int kRoutedThreads = 256;
constexpr int kRoutedLoads = 16;      // gathers in flight per thread
}

// route_ids [rows, k_route]; part [rows, slices, k_route]
template <typename WT>
__global__ __launch_bounds__(kRoutedThreads) void routed_partial_kernel(
    const uint16_t *__restrict__ h, const WT *__restrict__ W, const int32_t *__restrict__ route_ids,
    float *__restrict__ part, int d, int V, int k_route, int slices, int per_slice)
{
    const int slice = blockIdx.x, row = blockIdx.y, tid = threadIdx.x;
    const int c0 = min(d, slice * per_slice), c1 = min(d, c0 + per_slice);
    __shared__ float red[kRoutedThreads / 64][64];
    // thread (id slot q = tid % 64, row phase tid / 64): rows c0 + phase, c0 + phase + 4, ... of W at column id_q
    const int q = tid & 63, phase = tid >> 6;
    const int id = route_ids[(size_t)row * k_route + min(q, k_route - 1)];
    const bool ok = q < k_route && (unsigned)id < (unsigned)V;
    const WT *col = W + (ok ? id : 0);
    const uint16_t *hr = h + (size_t)row * d;
    float acc = 0.f;
    for (int c = c0 + phase; c < c1; c += 4 * kRoutedLoads) {
        WT w[kRoutedLoads];
#pragma unroll
        for (int u = 0; u < kRoutedLoads; ++u) w[u] = col[(size_t)min(c + 4 * u, c1 - 1) * V];
#pragma unroll
        for (int u = 0; u < kRoutedLoads; ++u) {
            const int cc = c + 4 * u;
            float wf;
            if constexpr (sizeof(WT) == 2) wf = bf16_to_float(w[u]); else wf = w[u];
            acc = fmaf(cc < c1 ? bf16_to_float(hr[cc]) : 0.f, wf, acc);
        }
    }
    red[phase][q] = acc;
    __syncthreads();
    if (tid < k_route)
        part[((size_t)row * slices + slice) * k_route + tid] = ((red[0][tid] + red[1][tid]) + red[2][tid]) + red[3][tid];
}

// The same partial sums from a token-major copy of W, Wt [V, d] (the layout an LM head's weight is usually stored in):
// the row of an id is d adjacent elements.  Block (group of 8 ids, row): wavefront w takes ids 2 w and 2 w + 1 of the
// group, a lane 8 adjacent elements of h and of the id's row per step; lanes are added in order inside the DPP tree.
// y [rows, k_route] (one "slice").
template <typename WT>
__global__ __launch_bounds__(kRoutedThreads) void routed_rows_kernel(
    const uint16_t *__restrict__ h, const WT *__restrict__ Wt, const int32_t *__restrict__ route_ids,
    float *__restrict__ y, int d, int V, int k_route)
{
    const int row = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint16_t *hr = h + (size_t)row * d;
    constexpr int IPW = 2;                        // ids per wavefront
    const WT *wrow[IPW];
    float acc[IPW];
#pragma unroll
    for (int q = 0; q < IPW; ++q) {
        const int slot = min(blockIdx.x * 8 + wave * IPW + q, k_route - 1);
        const int id = route_ids[(size_t)row * k_route + slot];
        wrow[q] = Wt + (size_t)((unsigned)id < (unsigned)V ? id : 0) * d;
        acc[q] = 0.f;
    }
    for (int j = lane * 8; j < d; j += 512) {     // d is a multiple of 8
        const uint4 hq = *reinterpret_cast<const uint4 *>(hr + j);
        const float hv[8] = {bf16_lo(hq.x), bf16_hi(hq.x), bf16_lo(hq.y), bf16_hi(hq.y),
                             bf16_lo(hq.z), bf16_hi(hq.z), bf16_lo(hq.w), bf16_hi(hq.w)};
        float wv[IPW][8];
#pragma unroll
        for (int q = 0; q < IPW; ++q) {
            if constexpr (sizeof(WT) == 2) {
                const uint4 wq = *reinterpret_cast<const uint4 *>(wrow[q] + j);
                wv[q][0] = bf16_lo(wq.x); wv[q][1] = bf16_hi(wq.x); wv[q][2] = bf16_lo(wq.y); wv[q][3] = bf16_hi(wq.y);
                wv[q][4] = bf16_lo(wq.z); wv[q][5] = bf16_hi(wq.z); wv[q][6] = bf16_lo(wq.w); wv[q][7] = bf16_hi(wq.w);
            } else {
                const float4 a = *reinterpret_cast<const float4 *>(wrow[q] + j), b = *reinterpret_cast<const float4 *>(wrow[q] + j + 4);
                wv[q][0] = a.x; wv[q][1] = a.y; wv[q][2] = a.z; wv[q][3] = a.w;
                wv[q][4] = b.x; wv[q][5] = b.y; wv[q][6] = b.z; wv[q][7] = b.w;
            }
        }
#pragma unroll
        for (int q = 0; q < IPW; ++q)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[q] = fmaf(hv[e], wv[q][e], acc[q]);
    }
#pragma unroll
    for (int q = 0; q < IPW; ++q) {
        const float z = wave_sum(acc[q]);
        const int slot = blockIdx.x * 8 + wave * IPW + q;
        if (lane == 0 && slot < k_route) y[(size_t)row * k_route + slot] = z;
    }
}

__global__ __launch_bounds__(64) void routed_finish_kernel(
    const float *__restrict__ part, const int32_t *__restrict__ route_ids, int k_route, int slices, int k,
    int32_t *__restrict__ out_ids, float *__restrict__ out_logprobs)
{
    const int row = blockIdx.x, lane = threadIdx.x;
    __shared__ uint64_t keys[64];
    float y = kNegInf;
    int id = kNoId;
    if (lane < k_route) {
        y = 0.f;
        for (int s = 0; s < slices; ++s) y += part[((size_t)row * slices + s) * k_route + lane];      // fixed order
        id = route_ids[(size_t)row * k_route + lane];
    }
    const float m = wave_max(y);
    const float sum = wave_sum(lane < k_route ? fast_exp(y - m) : 0.f);
    const float lse = m + fast_log(sum);
    const uint64_t mine = lane < k_route ? make_key(y, (uint32_t)id) : kNoKey;
    keys[lane] = mine;
    lds_wave_sync();
    int rank = 0;
#pragma unroll 8
    for (int q = 0; q < 64; ++q) rank += (keys[q] > mine) ? 1 : 0;
    if (lane < k_route && rank < k) {
        out_ids[(size_t)row * k + rank] = id;
        out_logprobs[(size_t)row * k + rank] = y - lse;
    }
}

int routed_slices(int d) {
    int s = d / 64;                      // at least 64 rows of W per slice: 16 gathers per thread and phase
    if (s > 64) s = 64;
    if (s < 1) s = 1;
    return s;
}

hipError_t launch_routed_exact(const uint16_t *h, const void *W, bool w_is_f32, const int32_t *route_ids, float *part,
                               int rows, int d, int V, int k_route, int k, int32_t *out_ids, float *out_logprobs, hipStream_t st)
{
    const int slices = routed_slices(d);
    const int per_slice = ((d + slices - 1) / slices + 3) & ~3;
    dim3 grid(slices, rows);
    if (w_is_f32)
        routed_partial_kernel<float><<<grid, kRoutedThreads, 0, st>>>(h, static_cast<const float *>(W), route_ids, part, d, V, k_route, slices, per_slice);
    else
        routed_partial_kernel<uint16_t><<<grid, kRoutedThreads, 0, st>>>(h, static_cast<const uint16_t *>(W), route_ids, part, d, V, k_route, slices, per_slice);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    routed_finish_kernel<<<rows, 64, 0, st>>>(part, route_ids, k_route, slices, k, out_ids, out_logprobs);
    return hipGetLastError();
}

hipError_t launch_routed_exact_token_major(const uint16_t *h, const void *Wt, bool w_is_f32, const int32_t *route_ids, float *y,
                                           int rows, int d, int V, int k_route, int k, int32_t *out_ids, float *out_logprobs, hipStream_t st)
{
    dim3 grid((k_route + 7) / 8, rows);
    if (w_is_f32)
        routed_rows_kernel<float><<<grid, kRoutedThreads, 0, st>>>(h, static_cast<const float *>(Wt), route_ids, y, d, V, k_route);
    else
        routed_rows_kernel<uint16_t><<<grid, kRoutedThreads, 0, st>>>(h, static_cast<const uint16_t *>(Wt), route_ids, y, d, V, k_route);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    routed_finish_kernel<<<rows, 64, 0, st>>>(y, route_ids, k_route, 1, k, out_ids, out_logprobs);
    return hipGetLastError();
}

}  // namespace slimspec

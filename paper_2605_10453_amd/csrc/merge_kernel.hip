// Cross-workgroup merge for the streaming path: one block per row combines the row's
// partials (running max m_c, sum of exp s_c, sorted top-k list per vocabulary chunk) into
//     lse = M + ln sum_c s_c exp(m_c - M),   M = max_c m_c
// and the k globally first (logit desc, id asc) candidates, and writes
// out_ids / out_logprobs = logit - lse.  The order of every reduction is fixed, so
// the output does not depend on scheduling.
//
// Partials of one row cover increasing, disjoint id ranges and each list is
// already in output order, so "smaller list position c * k + p" breaks ties exactly
// like "smaller id".  Thread t owns the lists c = t, t + 256, ...; it offers the head
// of its best list, the block takes the best offer k times (one barrier per round).
#include "device_utils.hpp"
#include "launch.hpp"

namespace slimspec {

constexpr int kMergeWaves = kMergeThreads / 64;

__global__ __launch_bounds__(kMergeThreads) void merge_kernel(
    const float2 *__restrict__ part_ms, const float *__restrict__ part_val, const int *__restrict__ part_id,
    int chunks, int k, int32_t *__restrict__ out_ids, float *__restrict__ out_logprobs)
{
    extern __shared__ unsigned char lds_raw[];
    float *vals = reinterpret_cast<float *>(lds_raw);                       // [chunks * k]
    int *cursor = reinterpret_cast<int *>(vals + (size_t)chunks * k);       // [chunks]
    __shared__ float red_f[kMergeWaves];
    __shared__ uint64_t offer[2][kMergeWaves];
    __shared__ uint32_t winners[SLIMSPEC_KMAX_INTERNAL];

    const int row = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float2 *ms = part_ms + (size_t)row * chunks;
    const float *pv = part_val + (size_t)row * chunks * k;
    const int *pi = part_id + (size_t)row * chunks * k;

    const int n = chunks * k;
    for (int e = tid; e < n; e += kMergeThreads) vals[e] = pv[e];
    for (int c = tid; c < chunks; c += kMergeThreads) cursor[c] = 0;

    // log-sum-exp over the chunks
    float M = kNegInf;
    for (int c = tid; c < chunks; c += kMergeThreads) M = fmaxf(M, ms[c].x);
    M = wave_max(M);
    if (lane == 0) red_f[wave] = M;
    __syncthreads();
    M = red_f[0];
#pragma unroll
    for (int w = 1; w < kMergeWaves; ++w) M = fmaxf(M, red_f[w]);
    __syncthreads();
    float S = 0.f;
    for (int c = tid; c < chunks; c += kMergeThreads) {
        float2 p = ms[c];
        S += p.y * fast_exp(p.x - M);
    }
    S = wave_sum(S);
    if (lane == 0) red_f[wave] = S;
    __syncthreads();
    S = red_f[0];
#pragma unroll
    for (int w = 1; w < kMergeWaves; ++w) S += red_f[w];
    const float lse = M + fast_log(S);

    // this thread's best head
    auto best_of_mine = [&]() {
        uint64_t b = kNoKey;
        for (int c = tid; c < chunks; c += kMergeThreads) {
            int cur = cursor[c];
            if (cur < k) {
                float v = vals[c * k + cur];
                if (v != kNegInf) b = u64_max(b, make_key(v, (uint32_t)(c * k + cur)));
            }
        }
        return b;
    };
    uint64_t mine = best_of_mine();
    for (int p = 0; p < k; ++p) {
        uint64_t w = wave_max_key(mine);
        if (lane == 0) offer[p & 1][wave] = w;
        __syncthreads();
        uint64_t best = offer[p & 1][0];
#pragma unroll
        for (int q = 1; q < kMergeWaves; ++q) best = u64_max(best, offer[p & 1][q]);
        if (best == kNoKey) break;                  // cannot happen when k <= V
        if (mine == best) {                         // keys are unique: exactly one thread
            uint32_t e = key_tiebreak(best);
            winners[p] = e;
            cursor[e / (uint32_t)k] += 1;
            mine = best_of_mine();
        }
    }
    __syncthreads();
    if (tid < k) {
        uint32_t e = winners[tid];
        out_ids[(size_t)row * k + tid] = pi[e];
        out_logprobs[(size_t)row * k + tid] = vals[e] - lse;
    }
}

hipError_t launch_merge(const float2 *part_ms, const float *part_val, const int *part_id,
                        int rows, int chunks, int k, int32_t *out_ids, float *out_logprobs, hipStream_t st)
{
    size_t lds = merge_lds_bytes(chunks, k);
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(merge_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    merge_kernel<<<rows, kMergeThreads, lds, st>>>(part_ms, part_val, part_id, chunks, k, out_ids, out_logprobs);
    return hipGetLastError();
}

}  // namespace slimspec

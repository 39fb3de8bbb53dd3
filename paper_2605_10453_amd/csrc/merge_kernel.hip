// Cross-workgroup merge for the streaming path: one block per row combines the row's
// partials (running max m_c, sum of exp s_c, sorted top-k list per vocabulary chunk) into
//     lse = M + ln sum_c s_c exp(m_c - M),   M = max_c m_c
// and the k globally first (logit desc, id asc) candidates, and writes
// out_ids / out_logprobs = logit - lse.  The order of every reduction is fixed and the
// selection works on unique keys, so the output does not depend on scheduling.
//
// Partials of one row cover increasing, disjoint id ranges and each list is already in
// output order, so "smaller list position e = c * k + p" breaks ties exactly like
// "smaller id".  Selection, in steps whose cost does not grow with k:
//   (1) the k-th largest list head (by all-pairs counting) bounds the answer from below;
//   (2) the entries that reach the bound (at most k lists, k entries each) are gathered;
//   (3) they are ranked among themselves by counting; ranks below k are the output.
#include "device_utils.hpp"
#include "launch.hpp"

namespace slimspec {

constexpr int kMergeWaves = kMergeThreads / 64;

__global__ __launch_bounds__(kMergeThreads) void merge_kernel(
    const float2 *__restrict__ part_ms, const float *__restrict__ part_val, const int *__restrict__ part_id,
    int chunks, int k, int32_t *__restrict__ out_ids, float *__restrict__ out_logprobs)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    uint64_t *heads = reinterpret_cast<uint64_t *>(lds_raw);                 // [chunks]
    uint64_t *cand = heads + chunks;                                          // [k * k]
    float *vals = reinterpret_cast<float *>(cand + (size_t)k * k);           // [chunks * k]
    __shared__ float red_m[kMergeWaves], red_s[kMergeWaves];
    __shared__ uint64_t bound_sh;
    __shared__ uint32_t cnt_sh;
    __shared__ uint32_t winners[SLIMSPEC_KMAX_INTERNAL];

    const int row = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float2 *ms = part_ms + (size_t)row * chunks;
    const float *pv = part_val + (size_t)row * chunks * k;
    const int *pi = part_id + (size_t)row * chunks * k;

    const int n = chunks * k;
    for (int e = tid; e < n; e += kMergeThreads) vals[e] = pv[e];
    if (tid == 0) { bound_sh = kNoKey; cnt_sh = 0u; }

    // log-sum-exp: every thread folds its chunks in increasing order, then the block combines
    float m_t = kNegInf, s_t = 0.f;
    for (int c = tid; c < chunks; c += kMergeThreads) {
        heads[c] = make_key(pv[(size_t)c * k], (uint32_t)(c * k));
        float2 p = ms[c];
        float m_new = fmaxf(m_t, p.x);
        s_t = s_t * fast_exp(m_t - m_new) + p.y * fast_exp(p.x - m_new);
        m_t = m_new;
    }
    const float m_w = wave_max(m_t);
    float s_w = (m_t == kNegInf) ? 0.f : s_t * fast_exp(m_t - m_w);
    s_w = wave_sum(s_w);
    if (lane == 0) { red_m[wave] = m_w; red_s[wave] = s_w; }
    __syncthreads();
    float M = red_m[0];
#pragma unroll
    for (int w = 1; w < kMergeWaves; ++w) M = fmaxf(M, red_m[w]);
    float S = 0.f;
#pragma unroll
    for (int w = 0; w < kMergeWaves; ++w) S += (red_m[w] == kNegInf) ? 0.f : red_s[w] * fast_exp(red_m[w] - M);
    const float lse = M + fast_log(S);

    // (1) the k-th largest head
    for (int c = tid; c < chunks; c += kMergeThreads) {
        const uint64_t mine = heads[c];
        int rank = 0;
        for (int q = 0; q < chunks; ++q) rank += (heads[q] > mine) ? 1 : 0;
        if (rank == k - 1) bound_sh = mine;             // keys are unique: one writer at most
    }
    __syncthreads();
    const uint64_t bound = bound_sh;                    // kNoKey when there are fewer than k lists: keep everything
    // (2) gather what reaches the bound
    for (int c = tid; c < chunks; c += kMergeThreads) {
        if (heads[c] < bound) continue;
        for (int p = 0; p < k; ++p) {
            const float v = vals[c * k + p];
            const uint64_t key = make_key(v, (uint32_t)(c * k + p));
            if (v == kNegInf || key < bound) break;     // lists are sorted
            cand[atomicAdd(&cnt_sh, 1u)] = key;
        }
    }
    __syncthreads();
    // (3) rank the gathered entries
    const int n_cand = (int)cnt_sh;
    for (int c = tid; c < n_cand; c += kMergeThreads) {
        const uint64_t mine = cand[c];
        int rank = 0;
        for (int q = 0; q < n_cand; ++q) rank += (cand[q] > mine) ? 1 : 0;
        if (rank < k) winners[rank] = key_tiebreak(mine);
    }
    __syncthreads();
    if (tid < k) {                                      // n_cand >= k whenever k <= V
        const uint32_t e = winners[tid];
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

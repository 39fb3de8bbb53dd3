// Cross-workgroup merge: one wavefront per row combines the row's partials
// (running max m_c, sum of exp s_c, sorted top-k list per vocabulary chunk) into
//     lse = M + ln sum_c s_c exp(m_c - M),   M = max_c m_c
// and the k globally first (logit desc, id asc) candidates, and writes
// out_ids / out_logprobs = logit - lse.  The order of every reduction is fixed, so
// the output does not depend on scheduling.
//
// Partials of one row cover increasing, disjoint id ranges and each list is
// already in output order, so "smaller partial index, then smaller position"
// breaks ties exactly like "smaller id".
#include "device_utils.hpp"
#include "launch.hpp"

namespace slimspec {

__global__ __launch_bounds__(64) void merge_kernel(
    const float2 *__restrict__ part_ms, const float *__restrict__ part_val, const int *__restrict__ part_id,
    int chunks, int k, int32_t *__restrict__ out_ids, float *__restrict__ out_logprobs)
{
    extern __shared__ unsigned char lds_raw[];
    float *vals = reinterpret_cast<float *>(lds_raw);                       // [chunks * k]
    int *cursor = reinterpret_cast<int *>(vals + (size_t)chunks * k);       // [chunks]
    int *win = cursor + chunks;                                              // [64] winning partial per rank

    const int row = blockIdx.x;
    const int lane = threadIdx.x;
    const float2 *ms = part_ms + (size_t)row * chunks;
    const float *pv = part_val + (size_t)row * chunks * k;
    const int *pi = part_id + (size_t)row * chunks * k;

    const int n = chunks * k;
    for (int e = lane; e < n; e += kWave) vals[e] = pv[e];
    for (int c = lane; c < chunks; c += kWave) cursor[c] = 0;

    float M = kNegInf;
    for (int c = lane; c < chunks; c += kWave) M = fmaxf(M, ms[c].x);
    M = wave_max(M);
    float S = 0.f;
    for (int c = lane; c < chunks; c += kWave) {
        float2 p = ms[c];
        S += p.y * fast_exp(p.x - M);
    }
    S = wave_sum(S);
    const float lse = M + fast_log(S);
    __syncthreads();

    int my_c = -1, my_p = 0;        // lane p keeps the p-th winner
    for (int p = 0; p < k; ++p) {
        float bv = kNegInf;
        int bc = kNoId;
        for (int c = lane; c < chunks; c += kWave) {
            int cur = cursor[c];
            if (cur < k) {
                float v = vals[c * k + cur];
                if (ranks_before(v, c, bv, bc)) { bv = v; bc = c; }
            }
        }
        wave_first(bv, bc);
        if (bc == kNoId) break;                     // fewer than k candidates in total (cannot happen when k <= V)
        int cur = cursor[bc];                       // same value in every lane
        if (lane == p) { my_c = bc; my_p = cur; }
        __syncthreads();
        if (lane == 0) cursor[bc] = cur + 1;
        __syncthreads();
    }
    (void)win;
    if (lane < k && my_c >= 0) {
        size_t e = (size_t)my_c * k + my_p;
        out_ids[(size_t)row * k + lane] = pi[e];
        out_logprobs[(size_t)row * k + lane] = vals[e] - lse;
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
    merge_kernel<<<rows, 64, lds, st>>>(part_ms, part_val, part_id, chunks, k, out_ids, out_logprobs);
    return hipGetLastError();
}

}  // namespace slimspec

// Cross-workgroup merge for the streaming path: one block per row combines the row's chunk
// partials into the final ids and log-probabilities (see merge_row in gemv_parts.hpp).
#include "gemv_parts.hpp"
#include "launch.hpp"

namespace slimspec {

constexpr int kRowMergeThreads = 1024;   // one block per row: the more threads, the shorter the load and rank phases

__global__ __launch_bounds__(kRowMergeThreads) void merge_kernel(
    const float2 *__restrict__ part_ms, const float *__restrict__ part_val, const int *__restrict__ part_id,
    int chunks, int k, int cache_ids, int32_t *__restrict__ out_ids, float *__restrict__ out_logprobs,
    const int32_t *__restrict__ id_map, SampleOut so, const float4 *__restrict__ part_smp)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    __shared__ MergeSmall small;
    const int row = blockIdx.x;
    merge_row<kRowMergeThreads>(lds_raw, cache_ids != 0, small, threadIdx.x, part_ms + (size_t)row * chunks,
                             part_val + (size_t)row * chunks * k, part_id + (size_t)row * chunks * k,
                             chunks, k, out_ids + (size_t)row * k, out_logprobs + (size_t)row * k, id_map,
                             so.on ? part_smp + (size_t)row * chunks : nullptr, so.lse + row, so.sample_ids + row, so.sample_logprobs + row);
}

hipError_t launch_merge(const float2 *part_ms, const float *part_val, const int *part_id,
                        int rows, int chunks, int k, int32_t *out_ids, float *out_logprobs, const int32_t *id_map,
                        const SampleOut &so, const float4 *part_smp, hipStream_t st)
{
    const bool cache_ids = merge_lds_bytes(chunks, k, true) <= 64 * 1024;
    size_t lds = merge_lds_bytes(chunks, k, cache_ids);
    if (lds > 48 * 1024) {
        static LdsLimit lds_limit;
        hipError_t e = lds_limit.raise(reinterpret_cast<const void *>(merge_kernel), (int)lds);
        if (e != hipSuccess) return e;
    }
    merge_kernel<<<rows, kRowMergeThreads, lds, st>>>(part_ms, part_val, part_id, chunks, k, cache_ids ? 1 : 0, out_ids, out_logprobs, id_map, so, part_smp);
    return hipGetLastError();
}

}  // namespace slimspec

// Host-callable launchers of the gfx950 kernels (one per kernel family).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "plan.hpp"

namespace slimspec {

// t = h A (fp32) for up to kGemvMaxRows rows.
hipError_t launch_down_projection(const uint16_t *h, const uint16_t *A, float *t,
                                  int rows_here, int d, int r, hipStream_t st);

// x = float(h) for the full head.
hipError_t launch_widen_rows(const uint16_t *h, float *x, int n, hipStream_t st);

// One partial (max, sum of exp, top-k) per (row, 512-column chunk) from x [rows_here, K] and M [K, V].
hipError_t launch_stream_topk(const float *x, const void *M, bool m_is_f32,
                              float2 *part_ms, float *part_val, int *part_id,
                              int rows_here, int row0, int K, int V, int chunks, int k, hipStream_t st);

// Combine the partials of every row into the final ids and log-probabilities.
hipError_t launch_merge(const float2 *part_ms, const float *part_val, const int *part_id,
                        int rows, int chunks, int k, int32_t *out_ids, float *out_logprobs, hipStream_t st);

}  // namespace slimspec

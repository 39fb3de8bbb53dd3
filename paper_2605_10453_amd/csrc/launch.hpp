// Host-callable launchers of the gfx950 kernels (one per kernel family).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "plan.hpp"

namespace slimspec {

// slices of t = h A (fp32, [nds][R][r] with R = 1, 2, 4 or 8 >= rows_here) for up to kGemvMaxRows rows
hipError_t launch_down_projection(const uint16_t *h, const uint16_t *A, float *tpart,
                                  int rows_here, int d, int r, const DownPlan &dp, hipStream_t st);

// x = float(h) for the full head.
hipError_t launch_widen_rows(const uint16_t *h, float *x, int n, hipStream_t st);

// One partial (max, sum of exp, top-k) per (row, 512-column chunk) from x [rows_here, K] (nds = 0) or
// from nds slices of it (the output of launch_down_projection), and M [K, V].
hipError_t launch_stream_topk(const float *x, int nds, const void *M, bool m_is_f32,
                              float2 *part_ms, float *part_val, int *part_id,
                              int rows_here, int row0, int K, int V, int chunks, int k, hipStream_t st);

// Combine the partials of every row into the final ids and log-probabilities.
hipError_t launch_merge(const float2 *part_ms, const float *part_val, const int *part_id,
                        int rows, int chunks, int k, int32_t *out_ids, float *out_logprobs, hipStream_t st);

// ---- matrix-core path (rows > kGemvMaxRows, bf16 weights) ----
constexpr int kStreamList = 3;          // groups kept per lane stream
constexpr int kStreamRec = 3 + 3 * kStreamList;   // floats per stream partial

int mfma_cols_per_wave(int rows);       // MFMA tiles (of the 8 in a 256-wide tile) owned by one wavefront

// partial sums of t = h A over `slices` slices of d (kslice entries each, a multiple of 64)
hipError_t launch_down_gemm(const uint16_t *h, const uint16_t *A, float *part, int rows, int rows_pad, int d, int r,
                            int slices, int kslice, hipStream_t st);
// slices -> fp32 t, f16 t (k-grouped), per-row rounding statistics, rms estimate of B
hipError_t launch_down_finish(const float *part, int slices, int rows, int rows_pad, int r,
                              float *t32, void *t16, float2 *stat, const uint16_t *B, int V, float *brms,
                              int xmode, hipStream_t st);   // xmode 0: f16 t; 1: bf16 t log2(e); 2: f16 t log2(e)
// vocabulary projection with the fused epilogue; X is f16 k-grouped (x_row_major = false, M converted to
// f16 on the fly) or bf16 row-major [rows, K] (x_row_major = true, bf16 MFMA)
hipError_t launch_head_mfma(const uint16_t *X, bool x_row_major, const uint16_t *M, float *part,
                            int rows, int rows_pad, int K, int V, int n_rb, int gw, hipStream_t st);

// the same projection from stages loaded straight into LDS; X is bf16 in 16-byte vectors of 8 contraction
// elements, [ceil(K / 64) * 8][rows_pad], rows_pad a multiple of 128; columns of an MFMA tile are contiguous
// x_is_f16: X holds f16 t log2(e) and the kernel turns the M tiles into f16 inside LDS (an 8 times
// finer operand than bf16); otherwise X holds bf16 t log2(e)
hipError_t launch_head_tile(const void *X, bool x_is_f16, const uint16_t *M, float *part, int rows, int rows_pad,
                            int K, int V, int n_rb, int gw, hipStream_t st);

// stream partials -> final ids / log-probabilities, with exact fp32 re-evaluation of uncertain ranks
hipError_t launch_merge_streams(const float *part, int rows, int nsr, int gw, int n_wv, int tv, int n_vt,
                                const void *xexact, bool x_is_bf16, int ldx, const uint16_t *M, int K, int V,
                                const float2 *stat, int n_stat, int rows_pad, const float *brms, int k,
                                bool contiguous_tiles, float unit, float tiny_w, int32_t *out_ids, float *out_logprobs, hipStream_t st);

}  // namespace slimspec

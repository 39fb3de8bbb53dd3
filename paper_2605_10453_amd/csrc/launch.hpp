// Host-callable launchers of the gfx950 kernels (one per kernel family).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "plan.hpp"
#include <atomic>
#include <mutex>

namespace slimspec {

// The dynamic shared memory limit of a kernel is raised once per process and device (and again only if a later call
// needs more), not on every launch: the attribute call is host work on a path that takes tens of microseconds.
// One LdsLimit object per kernel instantiation (a function-local static of its launcher).
struct LdsLimit {
    static constexpr int kDevices = 16;
    std::atomic<int> bytes[kDevices] = {};
    hipError_t raise(const void *fn, int need) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        const bool tracked = dev >= 0 && dev < kDevices;
        if (tracked && bytes[dev].load(std::memory_order_acquire) >= need) return hipSuccess;
        // the limit only ever grows: two host threads that raise it at the same time must not leave the smaller value
        std::lock_guard<std::mutex> lock(raising);
        if (tracked && bytes[dev].load(std::memory_order_acquire) >= need) return hipSuccess;
        e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, need);
        if (e == hipSuccess && tracked) bytes[dev].store(need, std::memory_order_release);
        return e;
    }
    std::mutex raising;
};

// slices of t = h A (fp32, [nds][R][r] with R = 1, 2, 4 or 8 >= rows_here) for up to kGemvMaxRows rows
// A: a stack of [d, r] matrices; mat_of_row (host, rows_here entries, or null: matrix 0) names each row's
hipError_t launch_down_projection(const uint16_t *h, const uint16_t *A, float *tpart,
                                  int rows_here, int d, int r, const DownPlan &dp, const int *mat_of_row, hipStream_t st);

// x = float(h) for the full head.
hipError_t launch_widen_rows(const uint16_t *h, float *x, int n, hipStream_t st);

// One partial (max, sum of exp, top-k) per (row, 512-column chunk) from x [rows_here, K] (nds = 0) or
// from nds slices of it (the output of launch_down_projection), and M [K, V].
// part_smp (null: off): one Gumbel-max winner per (row, chunk) for sampling with the seed (seed_lo, seed_hi)
hipError_t launch_stream_topk(const float *x, int nds, const void *M, bool m_is_f32,
                              float2 *part_ms, float *part_val, int *part_id,
                              int rows_here, int row0, int K, int V, int chunks, int lanes, int nw1, int k,
                              float4 *part_smp, uint32_t seed_lo, uint32_t seed_hi, hipStream_t st);

// Combine the partials of every row into the final ids and log-probabilities.
// Outputs of stochastic decoding (on: asked for): the noise seed, and per row the log-sum-exp over the vocabulary
// and one Gumbel-max draw from the softmax with its log-probability.
struct SampleOut {
    int on = 0;
    uint32_t seed_lo = 0, seed_hi = 0;
    float *lse = nullptr;
    int32_t *sample_ids = nullptr;
    float *sample_logprobs = nullptr;
};

// id_map (may be null): the vocabulary id of every column, for heads over a kept subset of the vocabulary
// part_smp [rows, chunks]: the chunks' Gumbel-max winners (when so.on)
hipError_t launch_merge(const float2 *part_ms, const float *part_val, const int *part_id,
                        int rows, int chunks, int k, int32_t *out_ids, float *out_logprobs, const int32_t *id_map,
                        const SampleOut &so, const float4 *part_smp, hipStream_t st);

// ---- matrix-core path (rows > kGemvMaxRows, bf16 weights) ----
constexpr int kStreamList = 3;          // groups kept per lane stream
constexpr int kStreamRec = 3 + 3 * kStreamList;   // floats per stream partial
constexpr int kStreamRecSample = kStreamRec + 8;  // ... of a sampling call
static_assert(kStreamList == kStreamListPlan && kStreamRecSample == kStreamRecPlan, "the workspace plan is sized for these records");

// t = h A for up to 512 rows: 64 x 64 tiles over slices of the contraction (partial tiles in `part`), then the
// fixed-order sum of the slices: fp32 t, the 16-bit operand t log2(e) (bf16, or f16 when as_f16) in the k-grouped
// layout of head_tile_kernel (zero beyond r and beyond the last row), per-row rounding statistics per 32 columns,
// and per 256-column vocabulary tile (the largest column rms, the mean square) of B over a sample of its rows
// (tilescale [ceil(V / 256)])
// (A: the stack of down-projection matrices, [d, r] each; the grid names the rows and the matrix of every group)
hipError_t launch_down_projection_tiles(const uint16_t *h, const uint16_t *A, float *part, const DownGrid &g,
                                        int rows_pad, int d, int r,
                                        float *t32, void *t16, float2 *stat, const uint16_t *B, int V, float2 *tilescale,
                                        bool as_f16, hipStream_t st);

// vocabulary projection with the fused epilogue, stages loaded straight into LDS; X is 16-byte vectors of 8 contraction
// elements, [ceil(K / 64) * 8][rows_pad], rows_pad a multiple of 128; columns of an MFMA tile are contiguous
// x_is_f16: X holds f16 t log2(e) and the kernel turns the M tiles into f16 inside LDS (an 8 times
// finer operand than bf16); otherwise X holds bf16 t log2(e)
// natural_units: X holds the bf16 contraction input itself (full head) and the records carry natural-log values
// so.on: the records also carry every stream's Gumbel-max candidates (kStreamRecSample floats per record); row_base:
// index of the launch's first row in the call (the noise is a function of the row's index in the call)
hipError_t launch_head_tile(const void *X, bool x_is_f16, bool natural_units, const uint16_t *M, float *part, int rows, int rows_pad,
                            int K, int V, int n_rb, int gw, const SampleOut &so, int row_base, hipStream_t st);
// true only in an experiment build (-DSLIMSPEC_DIAG_DBG=n) where a timing-only variant replaces the kernel: its
// output is not a result and the calls then return SLIMSPEC_UNSUPPORTED
bool head_tile_timing_only();
// bf16 rows [rows, K] -> that X layout ([8 ceil(K / 64)][rows_pad] 16-byte vectors, zero padded)
hipError_t launch_regroup_rows(const uint16_t *h, void *X, int rows, int rows_pad, int K, hipStream_t st);

// stream partials -> final ids / log-probabilities, with exact fp32 re-evaluation of uncertain ranks
// nsr records per row (4, 2 or 1 for each of the gw column blocks of the head kernel's grid); unit: factor from the
// records' values to natural-log logits; tiny_w: magnitude below which the kernel flushed weights to zero;
// operand16: 0 the head kernel's row operand was exact, 1 it was t log2(e) rounded to bf16, 2 to f16 (the merge then
// recomputes, from the same rounding, the logit the head kernel saw for a column that has no recorded value);
// Mt: null, or the column-major copy of M, [V, K] (an exact logit then reads K adjacent elements; rows are not parked);
// defer_buf: merge_defer_bytes(rows) of scratch, or null: with it, rows that need exact re-evaluations are finished by
// two more launches that spread the column gathers over many CUs (worth it for long contractions only)
hipError_t launch_merge_streams(const float *part, int rows, int nsr, int gw, int n_vt,
                                const void *xexact, bool x_is_bf16, int ldx, int operand16,
                                const uint16_t *M, int K, int V, const uint16_t *Mt,
                                const float2 *stat, int n_stat, int rows_pad, const float2 *tilescale, int k,
                                float unit, float tiny_w, int32_t *out_ids, float *out_logprobs, const int32_t *id_map,
                                void *defer_buf, const SampleOut &so, int row_base, hipStream_t st);

// Mt[V, K] = the transpose of M[K, V] (bf16): the column-major copy launch_merge_streams can take
hipError_t launch_transpose_weights(const uint16_t *M, int K, int V, uint16_t *Mt, hipStream_t st);

// ---- router-then-exact head: exact full-head logits on each row's k_route routed ids, softmax and top-k over them
// part: rows * routed_slices(d) * k_route floats of scratch
int routed_slices(int d);
hipError_t launch_routed_exact(const uint16_t *h, const void *W, bool w_is_f32, const int32_t *route_ids, float *part,
                               int rows, int d, int V, int k_route, int k, int32_t *out_ids, float *out_logprobs, hipStream_t st);
// ... from a token-major copy of W, Wt [V, d]; y: rows * k_route floats of scratch
hipError_t launch_routed_exact_token_major(const uint16_t *h, const void *Wt, bool w_is_f32, const int32_t *route_ids, float *y,
                                           int rows, int d, int V, int k_route, int k, int32_t *out_ids, float *out_logprobs, hipStream_t st);

}  // namespace slimspec

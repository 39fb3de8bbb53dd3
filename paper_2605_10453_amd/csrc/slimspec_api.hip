// C ABI of the library (see include/slimspec.h): argument checks, workspace
// layout, and the launch sequence for each head.  Everything before the first
// launch is plain host arithmetic, so validation works without a GPU.
#include "../../include/slimspec.h"
#include "launch.hpp"
#include <string.h>
#include <atomic>

using namespace slimspec;
namespace slimspec { bool head_tile_f16(int k); }

namespace {

// Scratch of slimspec_head_topk_static: device memory that belongs to the library's code object, so the entry point
// needs no allocation and no workspace argument.  Every GPU the library runs on holds its own copy at its own
// address; in host code the array's name is only a handle for hipGetSymbolAddress, never a device pointer.
static __device__ __align__(256) unsigned char scratch[SLIMSPEC_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 16;
std::atomic<void *> g_scratch_ptr[kMaxDevices] = {};      // device address of `scratch`, per device, looked up once

thread_local char g_hip_error[256] = "";
thread_local hipEvent_t g_ev_start = nullptr, g_ev_stop = nullptr;

int fail_hip(hipError_t e)
{
    const char *s = hipGetErrorString(e);
    strncpy(g_hip_error, s ? s : "unknown HIP error", sizeof(g_hip_error) - 1);
    g_hip_error[sizeof(g_hip_error) - 1] = 0;
    return SLIMSPEC_HIP_ERROR;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Shape / k checks common to both heads.  Returns SLIMSPEC_OK or the error.
int check_shape(HeadKind kind, const slimspec_shape *s, int32_t k)
{
    if (!s) return SLIMSPEC_INVALID_ARGUMENT;
    if (s->rows <= 0 || s->d <= 0 || s->V <= 0) return SLIMSPEC_INVALID_ARGUMENT;
    if (kind == HeadKind::LowRank && s->r <= 0) return SLIMSPEC_INVALID_ARGUMENT;
    if (k < 1 || k > s->V) return SLIMSPEC_INVALID_ARGUMENT;
    if (k > SLIMSPEC_KMAX) return SLIMSPEC_UNSUPPORTED;
    if ((s->d & 7) || (s->V & 7)) return SLIMSPEC_UNSUPPORTED;
    if (kind == HeadKind::LowRank && (s->r & 7)) return SLIMSPEC_UNSUPPORTED;
    // Index arithmetic inside the kernels: 32-bit ids, 64-bit base addresses, 32-bit lane offsets of a few rows of a
    // weight matrix (up to four rows of V bf16 values) and of an element of A (d * r).
    if ((int64_t)s->V > (int64_t)1 << 28) return SLIMSPEC_UNSUPPORTED;
    if (kind == HeadKind::LowRank && (int64_t)s->d * s->r >= (int64_t)1 << 31) return SLIMSPEC_UNSUPPORTED;
    // ... and of a row of h inside one launch's 512 rows, and of 32 rows of A (the many-row down-projection)
    if (kind == HeadKind::LowRank && (s->d > (1 << 21) || s->r > (1 << 24))) return SLIMSPEC_UNSUPPORTED;
    const int chunks = make_chunk_geom(s->rows, s->V).chunks;
    if (merge_lds_bytes(chunks, k) > kMergeLdsLimit) return SLIMSPEC_UNSUPPORTED;
    return SLIMSPEC_OK;
}

constexpr int kMfmaMaxK = 16;      // the lane streams keep 3 groups: enough for k <= 16 (larger k: streaming path)
constexpr int kMfmaMinRows = 5;    // from here on the matrix-core path is faster than streaming rows in lock step (measured at C2's shape)

// The launches of one call share the workspace in stream order; a last, smaller batch has a plan of its own
// (fewer row blocks, more slices of d), so the call needs the larger of the two plans.
size_t mfma_workspace_bytes(HeadKind kind, const slimspec_shape *s)
{
    const int per = mfma_max_rows_per_launch(s->rows);
    const int rows0 = s->rows < per ? s->rows : per;
    size_t need = make_mfma_plan(kind, rows0, s->d, s->r, s->V).bytes;
    const int tail = s->rows % per;
    if (s->rows > per && tail != 0) {
        const size_t t = make_mfma_plan(kind, tail, s->d, s->r, s->V).bytes;
        if (t > need) need = t;
    }
    return need;
}

// Device address of this device's copy of `scratch` (looked up at the first call on the device).
int static_scratch_address(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e);
    if (dev < 0 || dev >= kMaxDevices) return SLIMSPEC_UNSUPPORTED;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail_hip(e != hipSuccess ? e : hipErrorInvalidSymbol);
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return SLIMSPEC_OK;
}

// One down-projection matrix per drafted position: rows [off[p], off[p + 1]) use matrix p of the stack (host array).
struct Positions { int n = 0; const int32_t *off = nullptr; };

int position_of_row(const Positions &pos, int row)
{
    int p = 0;
    while (p + 1 < pos.n && row >= pos.off[p + 1]) ++p;
    return p;
}

int run_head_mfma(HeadKind kind, const void *h, const void *A, const void *M, const void *Mt,
                  const slimspec_shape *shape, int32_t k, int32_t *out_ids, float *out_logprobs, const int32_t *id_map,
                  const Positions &pos, const SampleOut &so, void *workspace, size_t workspace_bytes, void *stream)
{
    if (workspace_bytes < mfma_workspace_bytes(kind, shape)) return SLIMSPEC_WORKSPACE_TOO_SMALL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    const int d = shape->d, r = shape->r, V = shape->V;
    const int per = mfma_max_rows_per_launch(shape->rows);
    const uint16_t *hb = static_cast<const uint16_t *>(h);
    const uint16_t *Mb = static_cast<const uint16_t *>(M);
    const uint16_t *Mtb = static_cast<const uint16_t *>(Mt);      // column-major copy of M, or null
    for (int row0 = 0; row0 < shape->rows; row0 += per) {
        const int rows = (shape->rows - row0 < per) ? shape->rows - row0 : per;
        // a last, smaller batch may fall below the matrix-core threshold; it still runs here
        MfmaPlan p = make_mfma_plan(kind, rows, d, r, V);
        if (kind == HeadKind::LowRank && pos.n > 0) {
            // this launch's rows in groups by position (empty groups dropped); the workspace is sized for any grouping
            int g_first[kMaxPositions + 1], g_mat[kMaxPositions], n_groups = 0;
            for (int q = 0; q < pos.n; ++q) {
                const int lo = pos.off[q] > row0 ? pos.off[q] : row0;
                const int hi = pos.off[q + 1] < row0 + rows ? pos.off[q + 1] : row0 + rows;
                if (hi > lo) { g_first[n_groups] = lo - row0; g_mat[n_groups] = q; ++n_groups; }
            }
            g_first[n_groups] = rows;
            p.down = make_down_grid(rows, p.rows_pad, d, r, n_groups, g_first, g_mat);
        }
        float *streams = reinterpret_cast<float *>(ws + p.off_streams);
        const uint16_t *hrow = hb + (size_t)row0 * d;
        hipError_t e;
        const bool timed = g_ev_start && row0 == 0;
        if (kind == HeadKind::LowRank) {
            float *t32 = reinterpret_cast<float *>(ws + p.off_t32);
            void *t16 = ws + p.off_t16;
            float2 *stat = reinterpret_cast<float2 *>(ws + p.off_stat);
            float2 *tilescale = reinterpret_cast<float2 *>(ws + p.off_tilescale);
            // (with a column-major copy the re-evaluations the finer operand saves cost little: bf16 as it is)
            const bool tile_f16 = head_tile_f16(k) && Mtb == nullptr;
            e = launch_down_projection_tiles(hrow, static_cast<const uint16_t *>(A), reinterpret_cast<float *>(ws + p.off_down_part), p.down,
                                             p.rows_pad, d, r, t32, t16, stat, Mb, V, tilescale, tile_f16, s);
            if (e != hipSuccess) return fail_hip(e);
            if (timed && (e = hipEventRecord(g_ev_start, s)) != hipSuccess) return fail_hip(e);
            e = launch_head_tile(t16, tile_f16, false, Mb, streams, rows, p.rows_pad, r, V, p.n_rb, p.gw, so, row0, s);
            if (e != hipSuccess) return fail_hip(e);
            if (timed && (e = hipEventRecord(g_ev_stop, s)) != hipSuccess) return fail_hip(e);
            if (head_tile_timing_only()) return SLIMSPEC_UNSUPPORTED;      // diagnostic build, timing-only kernel: no result
            // the records are in base-2 units (t was scaled by log2 e); f16 mode flushes weights below 2^-25 to zero
            e = launch_merge_streams(streams, rows, p.nsr, p.gw, p.n_vt, t32, false, r, tile_f16 ? 2 : 1, Mb, r, V, Mtb, stat, 2 * ((r + 63) / 64), p.rows_pad, tilescale, k,
                                     0.6931471805599453f, tile_f16 ? 2.9802322e-8f : 0.f, out_ids + (size_t)row0 * k, out_logprobs + (size_t)row0 * k, id_map,
                                     (p.defer && merge_parks_rows(r, tile_f16)) ? ws + p.off_defer : nullptr, so, row0, s);
            if (e != hipSuccess) return fail_hip(e);
        } else {
            // the full head runs the same kernel on h itself (bf16 exact, natural units): no rounding statistics
            void *hx = ws + p.off_t16;
            if ((e = launch_regroup_rows(hrow, hx, rows, p.rows_pad, d, s)) != hipSuccess) return fail_hip(e);
            if (timed && (e = hipEventRecord(g_ev_start, s)) != hipSuccess) return fail_hip(e);
            e = launch_head_tile(hx, false, true, Mb, streams, rows, p.rows_pad, d, V, p.n_rb, p.gw, so, row0, s);
            if (e != hipSuccess) return fail_hip(e);
            if (timed && (e = hipEventRecord(g_ev_stop, s)) != hipSuccess) return fail_hip(e);
            if (head_tile_timing_only()) return SLIMSPEC_UNSUPPORTED;
            e = launch_merge_streams(streams, rows, p.nsr, p.gw, p.n_vt, hrow, true, d, 0, Mb, d, V, Mtb, nullptr, 0, 0, nullptr, k,
                                     1.0f, 0.f, out_ids + (size_t)row0 * k, out_logprobs + (size_t)row0 * k, id_map,
                                     (p.defer && merge_parks_rows(d, true)) ? ws + p.off_defer : nullptr, so, row0, s);
            if (e != hipSuccess) return fail_hip(e);
        }
    }
    return SLIMSPEC_OK;
}

int run_head(HeadKind kind, const void *h, const void *A, const void *M, bool m_is_f32,
             const slimspec_shape *shape, int32_t k, int32_t *out_ids, float *out_logprobs,
             void *workspace, size_t workspace_bytes, void *stream, const int32_t *id_map = nullptr,
             const Positions &pos = Positions(), const SampleOut &so = SampleOut(), const void *Mt = nullptr)
{
    int st = check_shape(kind, shape, k);
    if (st != SLIMSPEC_OK) return st;
    if (!h || !M || !out_ids || !out_logprobs || !workspace) return SLIMSPEC_INVALID_ARGUMENT;
    if (kind == HeadKind::LowRank && !A) return SLIMSPEC_INVALID_ARGUMENT;
    if (!aligned16(h) || !aligned16(M) || (A && !aligned16(A)) || !aligned16(workspace) || !aligned16(Mt))
        return SLIMSPEC_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(out_ids) & 3u) || (reinterpret_cast<uintptr_t>(out_logprobs) & 3u))
        return SLIMSPEC_UNSUPPORTED;
    if (so.on && (!so.lse || !so.sample_ids || !so.sample_logprobs)) return SLIMSPEC_INVALID_ARGUMENT;
    const bool use_mfma = shape->rows >= kMfmaMinRows && !m_is_f32 && k <= kMfmaMaxK;
    if (use_mfma)
        return run_head_mfma(kind, h, A, M, Mt, shape, k, out_ids, out_logprobs, id_map, pos, so, workspace, workspace_bytes, stream);
    const Plan p = make_plan(kind, shape->rows, shape->d, shape->r, shape->V, k);
    if (workspace_bytes < p.bytes) return SLIMSPEC_WORKSPACE_TOO_SMALL;

    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    float *x = reinterpret_cast<float *>(ws + p.off_x);
    float2 *part_ms = reinterpret_cast<float2 *>(ws + p.off_part_ms);
    float *part_val = reinterpret_cast<float *>(ws + p.off_part_val);
    int *part_id = reinterpret_cast<int *>(ws + p.off_part_id);
    float4 *part_smp = so.on ? reinterpret_cast<float4 *>(ws + p.off_part_smp) : nullptr;
    const uint16_t *hb = static_cast<const uint16_t *>(h);

    // Rows are processed in groups of kGemvMaxRows by the streaming kernels; the groups reuse the small
    // scratch in stream order; one merge launch serves all rows.
    const DownPlan dp = make_down_plan(kind == HeadKind::LowRank, p.d, p.r);
    float *tpart = reinterpret_cast<float *>(ws + p.off_tpart);
    for (int row0 = 0; row0 < p.rows; row0 += kGemvMaxRows) {
        const int rows_here = (p.rows - row0 < kGemvMaxRows) ? p.rows - row0 : kGemvMaxRows;
        hipError_t e;
        if (kind == HeadKind::LowRank) {
            int mat_of_row[kGemvMaxRows];
            for (int i = 0; i < rows_here; ++i) mat_of_row[i] = pos.n > 0 ? position_of_row(pos, row0 + i) : 0;
            e = launch_down_projection(hb + (size_t)row0 * p.d, static_cast<const uint16_t *>(A),
                                       tpart, rows_here, p.d, p.r, dp, mat_of_row, s);
        }
        else
            e = launch_widen_rows(hb + (size_t)row0 * p.d, x, rows_here * p.d, s);
        if (e != hipSuccess) return fail_hip(e);
        const bool timed = g_ev_start && row0 == 0;
        if (timed && (e = hipEventRecord(g_ev_start, s)) != hipSuccess) return fail_hip(e);
        e = launch_stream_topk(kind == HeadKind::LowRank ? tpart : x, kind == HeadKind::LowRank ? dp.nds : 0, M, m_is_f32,
                               part_ms, part_val, part_id,
                               rows_here, row0, p.K, p.V, p.chunks, p.lanes, p.nw1, k, part_smp, so.seed_lo, so.seed_hi, s);
        if (e != hipSuccess) return fail_hip(e);
        if (timed && (e = hipEventRecord(g_ev_stop, s)) != hipSuccess) return fail_hip(e);
    }
    hipError_t e = launch_merge(part_ms, part_val, part_id, p.rows, p.chunks, k, out_ids, out_logprobs, id_map, so, part_smp, s);
    if (e != hipSuccess) return fail_hip(e);
    return SLIMSPEC_OK;
}

SampleOut sample_out(uint64_t seed, float *out_lse, int32_t *out_sample_ids, float *out_sample_logprobs)
{
    SampleOut so;
    so.on = 1;
    so.seed_lo = (uint32_t)(seed & 0xffffffffu);
    so.seed_hi = (uint32_t)(seed >> 32);
    so.lse = out_lse; so.sample_ids = out_sample_ids; so.sample_logprobs = out_sample_logprobs;
    return so;
}

// Scratch one call of `kind` needs (the query slimspec_workspace_bytes reports the larger of the two heads).
size_t head_workspace_bytes(HeadKind kind, const slimspec_shape *shape, int32_t k)
{
    if (check_shape(kind, shape, k) != SLIMSPEC_OK) return 0;
    size_t need = make_plan(kind, shape->rows, shape->d, shape->r, shape->V, k).bytes;
    if (shape->rows >= kMfmaMinRows) {
        const size_t m = mfma_workspace_bytes(kind, shape);
        if (m > need) need = m;
    }
    return need;
}

}  // namespace

namespace slimspec {
bool head_tile_f16(int k) {
    // The direct-to-LDS kernel takes bf16 operands as they are, or turns the weight tiles into f16 inside LDS and
    // takes an f16 t (8 times finer).  The conversion costs the projection kernel about 12 %; the finer operand
    // saves most of the merge's exact re-evaluations, which grow with k: measured break-even at k = 10, 5-9 % of
    // the call in favour of f16 at k = 16.
#ifdef SLIMSPEC_DIAG_OPERAND_F16      // experiment builds only: force the operand mode (1 f16, 0 bf16)
    return SLIMSPEC_DIAG_OPERAND_F16 != 0;
#endif
    return k > 12;
}
}  // namespace slimspec

extern "C" {

int slimspec_version(void) { return SLIMSPEC_VERSION; }

size_t slimspec_workspace_bytes(const slimspec_shape *shape, int32_t k)
{
    if (!shape) return 0;
    // the larger of: streaming path (also serves fp32 W and large k), matrix-core path, for both heads
    const size_t full = head_workspace_bytes(HeadKind::Full, shape, k);
    const size_t low = head_workspace_bytes(HeadKind::LowRank, shape, k);
    return full > low ? full : low;
}

int slimspec_head_topk(const void *h, const void *A, const void *B,
                       const slimspec_shape *shape, int32_t k,
                       int32_t *out_ids, float *out_logprobs,
                       void *workspace, size_t workspace_bytes, void *stream)
{
    return run_head(HeadKind::LowRank, h, A, B, false, shape, k, out_ids, out_logprobs,
                    workspace, workspace_bytes, stream);
}

int slimspec_transpose_weights(const void *M, int32_t K, int32_t V, void *Mt, void *stream)
{
    if (!M || !Mt || K <= 0 || V <= 0) return SLIMSPEC_INVALID_ARGUMENT;
    if ((K & 7) || (V & 7) || (int64_t)V > (int64_t)1 << 28) return SLIMSPEC_UNSUPPORTED;
    if (!aligned16(M) || !aligned16(Mt)) return SLIMSPEC_UNSUPPORTED;
    const hipError_t e = launch_transpose_weights(static_cast<const uint16_t *>(M), K, V, static_cast<uint16_t *>(Mt),
                                                  static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SLIMSPEC_OK : fail_hip(e);
}

int slimspec_head_topk_prepared(const void *h, const void *A, const void *B, const void *Bt,
                                const slimspec_shape *shape, int32_t k,
                                int32_t *out_ids, float *out_logprobs,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    if (!Bt) return SLIMSPEC_INVALID_ARGUMENT;
    return run_head(HeadKind::LowRank, h, A, B, false, shape, k, out_ids, out_logprobs,
                    workspace, workspace_bytes, stream, nullptr, Positions(), SampleOut(), Bt);
}

int slimspec_head_topk_static(const void *h, const void *A, const void *B,
                              const slimspec_shape *shape, int32_t k,
                              int32_t *out_ids, float *out_logprobs, void *stream)
{
    const int st = check_shape(HeadKind::LowRank, shape, k);
    if (st != SLIMSPEC_OK) return st;
    if (head_workspace_bytes(HeadKind::LowRank, shape, k) > (size_t)SLIMSPEC_STATIC_SCRATCH_BYTES)
        return SLIMSPEC_SCRATCH_LIMIT;
    if (!h || !A || !B || !out_ids || !out_logprobs) return SLIMSPEC_INVALID_ARGUMENT;      // before any HIP call
    void *ptr = nullptr;
    const int sa = static_scratch_address(&ptr);
    if (sa != SLIMSPEC_OK) return sa;
    return run_head(HeadKind::LowRank, h, A, B, false, shape, k, out_ids, out_logprobs,
                    ptr, (size_t)SLIMSPEC_STATIC_SCRATCH_BYTES, stream);
}

int full_head_topk(const void *h, const void *W, slimspec_dtype w_dtype,
                   const slimspec_shape *shape, int32_t k,
                   int32_t *out_ids, float *out_logprobs,
                   void *workspace, size_t workspace_bytes, void *stream)
{
    if (w_dtype != SLIMSPEC_BF16 && w_dtype != SLIMSPEC_F32) return SLIMSPEC_INVALID_ARGUMENT;
    return run_head(HeadKind::Full, h, nullptr, W, w_dtype == SLIMSPEC_F32, shape, k, out_ids, out_logprobs,
                    workspace, workspace_bytes, stream);
}

int slimspec_head_sample(const void *h, const void *A, const void *B,
                         const slimspec_shape *shape, int32_t k, uint64_t seed,
                         int32_t *out_ids, float *out_logprobs,
                         float *out_lse, int32_t *out_sample_ids, float *out_sample_logprobs,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    return run_head(HeadKind::LowRank, h, A, B, false, shape, k, out_ids, out_logprobs, workspace, workspace_bytes, stream,
                    nullptr, Positions(), sample_out(seed, out_lse, out_sample_ids, out_sample_logprobs));
}

int slimspec_head_sample_prepared(const void *h, const void *A, const void *B, const void *Bt,
                                  const slimspec_shape *shape, int32_t k, uint64_t seed,
                                  int32_t *out_ids, float *out_logprobs,
                                  float *out_lse, int32_t *out_sample_ids, float *out_sample_logprobs,
                                  void *workspace, size_t workspace_bytes, void *stream)
{
    if (!Bt) return SLIMSPEC_INVALID_ARGUMENT;
    return run_head(HeadKind::LowRank, h, A, B, false, shape, k, out_ids, out_logprobs, workspace, workspace_bytes, stream,
                    nullptr, Positions(), sample_out(seed, out_lse, out_sample_ids, out_sample_logprobs), Bt);
}

int full_head_sample(const void *h, const void *W, slimspec_dtype w_dtype,
                     const slimspec_shape *shape, int32_t k, uint64_t seed,
                     int32_t *out_ids, float *out_logprobs,
                     float *out_lse, int32_t *out_sample_ids, float *out_sample_logprobs,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    if (w_dtype != SLIMSPEC_BF16 && w_dtype != SLIMSPEC_F32) return SLIMSPEC_INVALID_ARGUMENT;
    return run_head(HeadKind::Full, h, nullptr, W, w_dtype == SLIMSPEC_F32, shape, k, out_ids, out_logprobs,
                    workspace, workspace_bytes, stream, nullptr, Positions(),
                    sample_out(seed, out_lse, out_sample_ids, out_sample_logprobs));
}

size_t routed_workspace_bytes(const slimspec_shape *shape, int32_t k_route)
{
    if (!shape) return 0;
    const size_t router = head_workspace_bytes(HeadKind::LowRank, shape, k_route);
    if (router == 0) return 0;
    const size_t n = (size_t)shape->rows * k_route;
    return align_up(router) + align_up(4 * n) + align_up(4 * n) + align_up(4 * n * routed_slices(shape->d));
}

namespace {
// W: [d, V], or (token_major) its copy [V, d]; Bt: null, or the column-major copy of B for the router
int run_routed(const void *h, const void *A, const void *B, const void *Bt, const void *W, bool token_major, slimspec_dtype w_dtype,
               const slimspec_shape *shape, int32_t k_route, int32_t k,
               int32_t *out_ids, float *out_logprobs,
               void *workspace, size_t workspace_bytes, void *stream)
{
    if (w_dtype != SLIMSPEC_BF16 && w_dtype != SLIMSPEC_F32) return SLIMSPEC_INVALID_ARGUMENT;
    const int st = check_shape(HeadKind::LowRank, shape, k_route);
    if (st != SLIMSPEC_OK) return st;
    if (k < 1 || k > k_route) return SLIMSPEC_INVALID_ARGUMENT;
    if (!W || !out_ids || !out_logprobs || !workspace) return SLIMSPEC_INVALID_ARGUMENT;
    if (!aligned16(W)) return SLIMSPEC_UNSUPPORTED;
    if (workspace_bytes < routed_workspace_bytes(shape, k_route)) return SLIMSPEC_WORKSPACE_TOO_SMALL;
    char *ws = static_cast<char *>(workspace);
    const size_t router = align_up(head_workspace_bytes(HeadKind::LowRank, shape, k_route));
    const size_t n = (size_t)shape->rows * k_route;
    int32_t *route_ids = reinterpret_cast<int32_t *>(ws + router);
    float *route_lp = reinterpret_cast<float *>(ws + router + align_up(4 * n));
    float *part = reinterpret_cast<float *>(ws + router + 2 * align_up(4 * n));
    // the router: the low-rank head's k_route best ids of every row
    const int rs = run_head(HeadKind::LowRank, h, A, B, false, shape, k_route, route_ids, route_lp, workspace, router, stream,
                            nullptr, Positions(), SampleOut(), Bt);
    if (rs != SLIMSPEC_OK) return rs;
    const hipError_t e = token_major
        ? launch_routed_exact_token_major(static_cast<const uint16_t *>(h), W, w_dtype == SLIMSPEC_F32, route_ids, part,
                                          shape->rows, shape->d, shape->V, k_route, k, out_ids, out_logprobs,
                                          static_cast<hipStream_t>(stream))
        : launch_routed_exact(static_cast<const uint16_t *>(h), W, w_dtype == SLIMSPEC_F32, route_ids, part,
                              shape->rows, shape->d, shape->V, k_route, k, out_ids, out_logprobs,
                              static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SLIMSPEC_OK : fail_hip(e);
}
}  // namespace

int routed_head_topk(const void *h, const void *A, const void *B, const void *W, slimspec_dtype w_dtype,
                     const slimspec_shape *shape, int32_t k_route, int32_t k,
                     int32_t *out_ids, float *out_logprobs,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    return run_routed(h, A, B, nullptr, W, false, w_dtype, shape, k_route, k, out_ids, out_logprobs, workspace, workspace_bytes, stream);
}

int routed_head_topk_prepared(const void *h, const void *A, const void *B, const void *Bt, const void *Wt, slimspec_dtype w_dtype,
                              const slimspec_shape *shape, int32_t k_route, int32_t k,
                              int32_t *out_ids, float *out_logprobs,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    return run_routed(h, A, B, Bt, Wt, true, w_dtype, shape, k_route, k, out_ids, out_logprobs, workspace, workspace_bytes, stream);
}

namespace {
int run_positions(const void *h, const void *A_stack, int32_t n_pos, const int32_t *pos_offsets,
                  const void *B, const void *Bt, const slimspec_shape *shape, int32_t k,
                  int32_t *out_ids, float *out_logprobs,
                  void *workspace, size_t workspace_bytes, void *stream)
{
    if (!shape || !pos_offsets) return SLIMSPEC_INVALID_ARGUMENT;
    if (n_pos < 1) return SLIMSPEC_INVALID_ARGUMENT;
    if (n_pos > SLIMSPEC_MAX_POSITIONS) return SLIMSPEC_UNSUPPORTED;
    if (pos_offsets[0] != 0 || pos_offsets[n_pos] != shape->rows) return SLIMSPEC_INVALID_ARGUMENT;
    for (int p = 0; p < n_pos; ++p)
        if (pos_offsets[p + 1] < pos_offsets[p]) return SLIMSPEC_INVALID_ARGUMENT;
    // the stack is addressed as one array of n_pos * d * r elements with the kernels' 32-bit element offsets
    if (shape->d > 0 && shape->r > 0 && (int64_t)n_pos * shape->d * shape->r >= (int64_t)1 << 31) return SLIMSPEC_UNSUPPORTED;
    Positions pos;
    pos.n = n_pos; pos.off = pos_offsets;
    return run_head(HeadKind::LowRank, h, A_stack, B, false, shape, k, out_ids, out_logprobs,
                    workspace, workspace_bytes, stream, nullptr, pos, SampleOut(), Bt);
}
}  // namespace

int slimspec_head_topk_positions(const void *h, const void *A_stack, int32_t n_pos, const int32_t *pos_offsets,
                                 const void *B, const slimspec_shape *shape, int32_t k,
                                 int32_t *out_ids, float *out_logprobs,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    return run_positions(h, A_stack, n_pos, pos_offsets, B, nullptr, shape, k, out_ids, out_logprobs, workspace, workspace_bytes, stream);
}

int slimspec_head_topk_positions_prepared(const void *h, const void *A_stack, int32_t n_pos, const int32_t *pos_offsets,
                                          const void *B, const void *Bt, const slimspec_shape *shape, int32_t k,
                                          int32_t *out_ids, float *out_logprobs,
                                          void *workspace, size_t workspace_bytes, void *stream)
{
    if (!Bt) return SLIMSPEC_INVALID_ARGUMENT;
    return run_positions(h, A_stack, n_pos, pos_offsets, B, Bt, shape, k, out_ids, out_logprobs, workspace, workspace_bytes, stream);
}

int truncated_head_topk(const void *h, const void *W_tr, slimspec_dtype w_dtype, const int32_t *id_map,
                        const slimspec_shape *shape, int32_t k,
                        int32_t *out_ids, float *out_logprobs,
                        void *workspace, size_t workspace_bytes, void *stream)
{
    if (w_dtype != SLIMSPEC_BF16 && w_dtype != SLIMSPEC_F32) return SLIMSPEC_INVALID_ARGUMENT;
    if (!id_map) return SLIMSPEC_INVALID_ARGUMENT;
    if (reinterpret_cast<uintptr_t>(id_map) & 3u) return SLIMSPEC_UNSUPPORTED;
    return run_head(HeadKind::Full, h, nullptr, W_tr, w_dtype == SLIMSPEC_F32, shape, k, out_ids, out_logprobs,
                    workspace, workspace_bytes, stream, id_map);
}

const char *slimspec_status_string(int status)
{
    switch (status) {
    case SLIMSPEC_OK: return "ok";
    case SLIMSPEC_INVALID_ARGUMENT: return "invalid argument";
    case SLIMSPEC_UNSUPPORTED: return "unsupported shape, k or alignment";
    case SLIMSPEC_WORKSPACE_TOO_SMALL: return "workspace too small";
    case SLIMSPEC_HIP_ERROR: return "HIP error";
    case SLIMSPEC_SCRATCH_LIMIT: return "shape needs more scratch than the library's static buffer holds";
    default: return "unknown status";
    }
}

const char *slimspec_last_hip_error(void) { return g_hip_error; }

int slimspec_set_timing_events(void *start_event, void *stop_event)
{
    if ((start_event == nullptr) != (stop_event == nullptr)) return SLIMSPEC_INVALID_ARGUMENT;
    g_ev_start = static_cast<hipEvent_t>(start_event);
    g_ev_stop = static_cast<hipEvent_t>(stop_event);
    return SLIMSPEC_OK;
}

}  // extern "C"

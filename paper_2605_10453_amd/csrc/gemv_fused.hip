// Whole head in ONE launch for calls with few rows (paper section 4.1, both heads), where every
// extra kernel boundary costs as much as a fifth of the weight streaming itself.
//
// Block b owns the 512-column vocabulary chunk b, as in stream_topk_kernel.  In order:
//   (0) the first loads of its chunk of B / W are issued (they do not depend on t);
//   (1) low-rank head only: the blocks share out the down-projection t = h A in items of
//       (64 columns of A) x (a slice of d), each read as full 128-byte lines; an item's partial
//       sums go to scratch and a flag word is set to this call's tag;
//   (2) every block waits (bounded spin) until all flags carry the tag, then sums the slices of t
//       in a fixed order into shared memory.  A block that loses patience computes the missing
//       items itself: same code, same bits, so a duplicate write is harmless.  Blocks are
//       dispatched in index order and the items sit on the lowest indices, so no block ever
//       waits for a block that has not started;
//   (3) the chunk is streamed and reduced to its partial (max, sum of exp, top-k) per row;
//   (4) the last block to finish (atomic ticket) merges all partials into the final ids and
//       log-probabilities and clears the flags.
//
// The flag words live in caller scratch whose contents are arbitrary on entry, hence the tag: a
// fresh non-zero 32-bit number per call.  The last block zeroes the flags again, so a replay of the
// same launch (same tag) from a captured graph also starts from a clean state.
#include "gemv_parts.hpp"
#include "launch.hpp"
#include <atomic>

namespace slimspec {

#ifdef SLIMSPEC_TRACE
__device__ unsigned long long g_trace[1024 * 8];
#define TRACE(slot) do { if (threadIdx.x == 0) g_trace[blockIdx.x * 8 + (slot)] = wall_clock64(); } while (0)
extern "C" void slimspec_read_trace(unsigned long long *dst) { (void)hipMemcpyFromSymbol(dst, HIP_SYMBOL(g_trace), sizeof(g_trace)); }
#else
#define TRACE(slot) do { } while (0)
#endif

namespace {

constexpr int kFusedMergeBytes = 32 * 1024;     // shared memory the last block may use for the merge
constexpr unsigned kSpinLimit = 1u << 22;

// Polls are relaxed (an acquire load would invalidate the XCD's L2 on every spin); one acquire fence
// follows the wait.
__device__ __forceinline__ uint32_t load_flag(const uint32_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_flag(uint32_t *p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace

template <int R, int NW, int PF, bool LOWRANK, typename WT>
__global__ __launch_bounds__(NW * 64) void fused_head_kernel(
    const uint16_t *__restrict__ h, const uint16_t *__restrict__ A, const WT *__restrict__ M,
    float *__restrict__ tpart, uint32_t *__restrict__ flags, uint32_t *__restrict__ ticket, uint32_t tag,
    float2 *__restrict__ part_ms, float *__restrict__ part_val, int *__restrict__ part_id,
    int rows_here, int d, int K, int V, int chunks, int k,
    int n_items, int n_cb, int nds, int slice,
    int32_t *__restrict__ out_ids, float *__restrict__ out_logprobs)
{
    constexpr int NT = NW * 64;
    __shared__ union { ChunkLds<R, NW> L; unsigned char merge_bytes[kFusedMergeBytes]; } lds_u;
    ChunkLds<R, NW> &L = lds_u.L;
    __shared__ MergeSmall small;
    __shared__ uint32_t sh_flag;
    extern __shared__ __align__(16) unsigned char dyn[];         // low-rank: t as fp32 [R][K]
    float *xs = reinterpret_cast<float *>(dyn);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int chunk = blockIdx.x;
    const int col = chunk * kChunkCols + lane * 8;
    const bool active = col < V;          // V is a multiple of 8: all 8 columns valid or none
    const int per = ((K + NW - 1) / NW + 7) & ~7;            // multiple of 8: keeps the 8-wide x reads aligned
    const int j0 = min(K, wave * per), j1 = min(K, j0 + per);
    constexpr int U = (sizeof(WT) == 2 && R <= 2) ? 16 : 8;
    const WT *base = M + (active ? col : 0);

    // Vector memory returns in issue order per wavefront, so a wavefront that has weight rows in
    // flight sees every later load (a flag poll, a slice of t) only after those rows.  Hence the
    // order below: the down-projection items first, then the weight prefetch, with wavefront 0
    // polling the flags BEFORE it issues its own prefetch.
    using RawT = decltype(load_raw8(static_cast<const WT *>(nullptr)));
    RawT q0[PF][U];                                             // PF batches of U rows kept in flight ahead of t
    const int n_first = active ? min(PF, (j1 - j0) / U) : 0;    // wavefront-uniform
    auto prefetch_first = [&]() {
#pragma unroll
        for (int b = 0; b < PF; ++b)
            if (b < n_first) {
#pragma unroll
                for (int u = 0; u < U; ++u) q0[b][u] = load_raw8(base + (size_t)(j0 + b * U + u) * V);
            }
    };

    TRACE(0);
    if (blockIdx.x == 0 && tid == 0) {
        __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (!LOWRANK) store_flag(&flags[0], tag);               // tells the others that the ticket is zero
    }
    if constexpr (LOWRANK) {
        // (1) this block's share of the down-projection
        auto redd = reinterpret_cast<float (*)[R][kItemCols]>(&L.red[0][0][0]);     // 16 KB at most; red is free until (3)
        static_assert(sizeof(float) * NW * R * kItemCols <= sizeof(L.red), "item scratch must fit");
        for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
            down_item<R, NT>(redd, h, A, tpart, item, n_cb, slice, rows_here, d, K, tid);   // ends with a barrier
            if (tid == 0) store_flag(&flags[item], tag);        // one release per block: an L2 write-back is not cheap
        }
        TRACE(1);
        // (0) first batch of weight rows, in flight while the flags are awaited; (2) wavefront 0 polls
        bool missing = false;
        if (wave != 0) {
            prefetch_first();
        } else {
            for (int item = lane; item < n_items; item += 64) {
                unsigned spins = 0;
                while (load_flag(&flags[item]) != tag) {
                    if (++spins > kSpinLimit) { missing = true; break; }
                    __builtin_amdgcn_s_sleep(2);
                }
            }
        }
        if (__syncthreads_or(missing ? 1 : 0)) {
            for (int item = 0; item < n_items; ++item) {
                if (tid == 0) sh_flag = load_flag(&flags[item]);
                __syncthreads();
                const bool todo = sh_flag != tag;
                __syncthreads();
                if (todo) down_item<R, NT>(redd, h, A, tpart, item, n_cb, slice, rows_here, d, K, tid);
            }
        }
        TRACE(2);
        if (tid == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");     // one cache invalidate per block
        __syncthreads();
        if (wave == 0) prefetch_first();
        // t = sum of the slices, in slice order (loads batched 8 at a time, the sum stays sequential)
        for (int e = tid; e < R * K; e += NT) {
            const int i = e / K, j = e % K;
            const float *src = tpart + (size_t)i * K + j;
            const size_t stride = (size_t)R * K;
            float s = 0.f;
            int ds = 0;
            for (; ds + 8 <= nds; ds += 8) {
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = src[(size_t)(ds + u) * stride];
#pragma unroll
                for (int u = 0; u < 8; ++u) s += v[u];
            }
            for (; ds < nds; ++ds) s += src[(size_t)ds * stride];
            xs[e] = s;
        }
        __syncthreads();
    } else {
        prefetch_first();
    }

    TRACE(3);
    // (3) stream the chunk
    float acc[R][8];
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[i][e] = 0.f;
    // 8 consecutive entries of row i of the contraction input (j is a multiple of 8)
    auto x8_at = [&](int i, int j, float (&xv)[8]) {
        if constexpr (LOWRANK) {
            const float4 *p = reinterpret_cast<const float4 *>(xs + i * K + j);
            const float4 a = p[0], b = p[1];
            xv[0] = a.x; xv[1] = a.y; xv[2] = a.z; xv[3] = a.w; xv[4] = b.x; xv[5] = b.y; xv[6] = b.z; xv[7] = b.w;
        } else {
            uint4 w = make_uint4(0, 0, 0, 0);
            if (i < rows_here) w = *reinterpret_cast<const uint4 *>(h + (size_t)i * K + j);
            xv[0] = bf16_lo(w.x); xv[1] = bf16_hi(w.x); xv[2] = bf16_lo(w.y); xv[3] = bf16_hi(w.y);
            xv[4] = bf16_lo(w.z); xv[5] = bf16_hi(w.z); xv[6] = bf16_lo(w.w); xv[7] = bf16_hi(w.w);
        }
    };
    auto x_at = [&](int i, int j) -> float {
        if constexpr (LOWRANK) return xs[i * K + j];
        else return (i < rows_here) ? bf16_to_float(h[(size_t)i * K + j]) : 0.f;
    };
    auto fma_batch = [&](const RawT (&q)[U], int j) {
#pragma unroll
        for (int g = 0; g < U / 8; ++g) {
            float xv[R][8];
#pragma unroll
            for (int i = 0; i < R; ++i) x8_at(i, j + 8 * g, xv[i]);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                float f[8];
                widen8(q[8 * g + u], f);
#pragma unroll
                for (int i = 0; i < R; ++i)
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[i][e] = fmaf(xv[i][u], f[e], acc[i][e]);
            }
        }
    };
    if (active) {
        int j = j0;
#pragma unroll
        for (int b = 0; b < PF; ++b)
            if (b < n_first) {
                fma_batch(q0[b], j);
                j += U;
            }
        for (; j + U <= j1; j += U) {
            RawT q[U];
#pragma unroll
            for (int u = 0; u < U; ++u) q[u] = load_raw8(base + (size_t)(j + u) * V);
            fma_batch(q, j);
        }
        for (; j < j1; ++j) {
            float f[8];
            widen8(load_raw8(base + (size_t)j * V), f);
#pragma unroll
            for (int i = 0; i < R; ++i) {
                const float xv = x_at(i, j);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[i][e] = fmaf(xv, f[e], acc[i][e]);
            }
        }
    }
    TRACE(4);
#pragma unroll
    for (int i = 0; i < R; ++i) {
        float4 *dst = reinterpret_cast<float4 *>(&L.red[wave][i][lane * 8]);
        dst[0] = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
        dst[1] = make_float4(acc[i][4], acc[i][5], acc[i][6], acc[i][7]);
    }
    __syncthreads();
    for (int i = wave; i < rows_here; i += NW)
        chunk_row_epilogue<R, NW>(L, i, wave, lane, active, col, k, (size_t)i * chunks + chunk,
                                  part_ms, part_val, part_id);

    TRACE(5);
    // (4) ticket; the last block merges.  The barrier orders every thread's partial writes before
    // thread 0's release; one write-back / invalidate per block.
    __syncthreads();
    if (tid == 0) {
        if (!LOWRANK) {                                         // the ticket must have been zeroed by block 0
            unsigned spins = 0;
            while (load_flag(&flags[0]) != tag && ++spins < (kSpinLimit << 4)) __builtin_amdgcn_s_sleep(4);
        }
        sh_flag = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    TRACE(6);
    if (sh_flag != gridDim.x - 1) return;
    unsigned char *mdyn = lds_u.merge_bytes;                    // merge scratch: the chunk buffers are free now
    for (int i = 0; i < rows_here; ++i)
        merge_row<NT>(mdyn, false, small, tid, part_ms + (size_t)i * chunks, part_val + (size_t)i * chunks * k,
                      part_id + (size_t)i * chunks * k, chunks, k, out_ids + (size_t)i * k, out_logprobs + (size_t)i * k);
    TRACE(7);
    const int n_flags = LOWRANK ? n_items : 1;
    for (int e = tid; e < n_flags; e += NT) store_flag(&flags[e], 0u);
}

// ---------------------------------------------------------------------------

namespace {
std::atomic<uint32_t> g_tag{0x5a17u};
uint32_t next_tag() {
    uint32_t t = g_tag.fetch_add(0x9e3779b9u, std::memory_order_relaxed) + 0x9e3779b9u;
    return t ? t : 0x1u;
}
}  // namespace

bool fused_head_fits(int rows_here, int chunks, int k) {
    (void)rows_here;
    return merge_lds_bytes(chunks, k) <= (size_t)kFusedMergeBytes;
}

FusedPlan make_fused_plan(bool low_rank, int d, int r) {
    FusedPlan p;
    if (low_rank) {
        p.n_cb = (r + kItemCols - 1) / kItemCols;
        // about 240 items in all (one round of blocks on 256 CUs), at most 32 slices, slices a multiple of 8 rows
        int want = 240 / p.n_cb;
        if (want > 32) want = 32;
        if (want < 1) want = 1;
        int slice = ((d + want - 1) / want + 7) / 8 * 8;
        if (slice < 64) slice = 64;
        p.slice = slice;
        p.nds = (d + slice - 1) / slice;
        p.n_items = p.n_cb * p.nds;
    }
    return p;
}

template <int R, int NW, int PF, bool LOWRANK, typename WT>
static hipError_t launch_fused_cfg(const uint16_t *h, const uint16_t *A, const WT *M, float *tpart, uint32_t *flags,
                                   uint32_t *ticket, float2 *ms, float *pv, int *pi, int rows_here, int d, int K, int V,
                                   int chunks, int k, const FusedPlan &fp, int32_t *out_ids, float *out_lp, hipStream_t st)
{
    auto fn = fused_head_kernel<R, NW, PF, LOWRANK, WT>;
    const size_t dyn = LOWRANK ? sizeof(float) * (size_t)R * K : 0;
    if (dyn > 16 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);
        if (e != hipSuccess) return e;
    }
    fn<<<chunks, NW * 64, dyn, st>>>(h, A, M, tpart, flags, ticket, next_tag(), ms, pv, pi, rows_here, d, K, V, chunks, k,
                                     fp.n_items, fp.n_cb, fp.nds, fp.slice, out_ids, out_lp);
    return hipGetLastError();
}

template <bool LOWRANK, typename WT>
static hipError_t launch_fused_rows(const uint16_t *h, const uint16_t *A, const WT *M, float *tpart, uint32_t *flags,
                                    uint32_t *ticket, float2 *ms, float *pv, int *pi, int rows_here, int d, int K, int V,
                                    int chunks, int k, const FusedPlan &fp, int32_t *out_ids, float *out_lp, hipStream_t st)
{
#define SLIMSPEC_FUSED(R, NW, PF) launch_fused_cfg<R, NW, PF, LOWRANK, WT>(h, A, M, tpart, flags, ticket, ms, pv, pi, rows_here, d, K, V, chunks, k, fp, out_ids, out_lp, st)
    // one row: 8 wavefronts (256 registers each) so that three batches of 16 rows can be in flight per lane
    if (rows_here <= 1) {
        if constexpr (sizeof(WT) == 2) return SLIMSPEC_FUSED(1, 8, 3);
        else return SLIMSPEC_FUSED(1, 16, 1);
    }
    if (rows_here <= 2) return SLIMSPEC_FUSED(2, 8, 1);
    if (rows_here <= 4) return SLIMSPEC_FUSED(4, 4, 1);
    return SLIMSPEC_FUSED(8, 2, 1);
#undef SLIMSPEC_FUSED
}

hipError_t launch_fused_head(bool low_rank, const uint16_t *h, const uint16_t *A, const void *M, bool m_is_f32,
                             float *tpart, uint32_t *flags, uint32_t *ticket, float2 *ms, float *pv, int *pi,
                             int rows_here, int d, int K, int V, int chunks, int k, const FusedPlan &fp,
                             int32_t *out_ids, float *out_lp, hipStream_t st)
{
    if (low_rank)
        return launch_fused_rows<true, uint16_t>(h, A, (const uint16_t *)M, tpart, flags, ticket, ms, pv, pi, rows_here, d, K, V,
                                                 chunks, k, fp, out_ids, out_lp, st);
    if (m_is_f32)
        return launch_fused_rows<false, float>(h, A, (const float *)M, tpart, flags, ticket, ms, pv, pi, rows_here, d, K, V,
                                               chunks, k, fp, out_ids, out_lp, st);
    return launch_fused_rows<false, uint16_t>(h, A, (const uint16_t *)M, tpart, flags, ticket, ms, pv, pi, rows_here, d, K, V,
                                              chunks, k, fp, out_ids, out_lp, st);
}

}  // namespace slimspec

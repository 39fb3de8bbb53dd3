// Device-side pieces shared by the streaming ("lane owns columns") kernels: raw weight loads,
// the per-chunk epilogue (running max, sum of exp, top-k of one 512-column chunk) and the
// per-row merge of the chunk partials.
#pragma once
#include "device_utils.hpp"
#include "plan.hpp"

namespace slimspec {

// 8 adjacent columns of one matrix row: kept as loaded (raw) while in flight, widened
// to fp32 only when consumed, so that many loads can be outstanding per lane.
struct Raw8Bf16 { uint4 w; };
struct Raw8F32 { float4 a, b; };
__device__ __forceinline__ Raw8Bf16 load_raw8(const uint16_t *p) { return {*reinterpret_cast<const uint4 *>(p)}; }
__device__ __forceinline__ Raw8F32 load_raw8(const float *p) {
    return {*reinterpret_cast<const float4 *>(p), *reinterpret_cast<const float4 *>(p + 4)};
}
__device__ __forceinline__ void widen8(const Raw8Bf16 &q, float (&f)[8]) {
    f[0] = bf16_lo(q.w.x); f[1] = bf16_hi(q.w.x); f[2] = bf16_lo(q.w.y); f[3] = bf16_hi(q.w.y);
    f[4] = bf16_lo(q.w.z); f[5] = bf16_hi(q.w.z); f[6] = bf16_lo(q.w.w); f[7] = bf16_hi(q.w.w);
}
__device__ __forceinline__ void widen8(const Raw8F32 &q, float (&f)[8]) {
    f[0] = q.a.x; f[1] = q.a.y; f[2] = q.a.z; f[3] = q.a.w; f[4] = q.b.x; f[5] = q.b.y; f[6] = q.b.z; f[7] = q.b.w;
}

// ---------------------------------------------------------------------------
// Down-projection t = h A shared out in items of (64 columns of A) x (a slice of d).
constexpr int kItemCols = 64;           // columns of A per item: one 128-byte line per row of A

// Which matrix of a stack of down-projection matrices each of up to 8 rows uses (one matrix per drafted position).
struct RowMats { int m[8]; };

// One down-projection item: columns [64 cb, 64 cb + 64) x rows [ds * slice, ds * slice + slice) of A.
// Thread = (row slot tid / 8, 16-byte piece tid % 8).  tpart is [nds][R][r].
// POS: A is a stack of [d, r] matrices and row i uses matrix mats.m[i] (every row then loads its own weights).
template <int R, int NT, bool POS>
__device__ __forceinline__ void down_item(float (*redd)[R][kItemCols], const uint16_t *__restrict__ h,
                                          const uint16_t *__restrict__ A, float *__restrict__ tpart,
                                          int item, int n_cb, int slice, int rows_here, int d, int r, int tid,
                                          const RowMats &mats)
{
    constexpr int NW = NT / 64;
    const int cb = item % n_cb, ds = item / n_cb;
    const int piece = tid & 7, slot = tid >> 3;
    const int col = cb * kItemCols + piece * 8;
    const int c_beg = ds * slice, c_end = min(d, c_beg + slice);
    float acc[R][8];
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[i][e] = 0.f;
    if (col < r) {
        for (int c = c_beg + slot; c < c_end; c += NT / 8) {
            if constexpr (!POS) {
                const uint4 w = *reinterpret_cast<const uint4 *>(A + (size_t)c * r + col);
                const float f[8] = {bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y),
                                    bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w)};
#pragma unroll
                for (int i = 0; i < R; ++i) {
                    const float hv = (i < rows_here) ? bf16_to_float(h[(size_t)i * d + c]) : 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[i][e] = fmaf(hv, f[e], acc[i][e]);
                }
            } else {
                uint4 w[R];
#pragma unroll
                for (int i = 0; i < R; ++i)
                    w[i] = *reinterpret_cast<const uint4 *>(A + (size_t)mats.m[i & 7] * d * r + (size_t)c * r + col);
#pragma unroll
                for (int i = 0; i < R; ++i) {
                    const float f[8] = {bf16_lo(w[i].x), bf16_hi(w[i].x), bf16_lo(w[i].y), bf16_hi(w[i].y),
                                        bf16_lo(w[i].z), bf16_hi(w[i].z), bf16_lo(w[i].w), bf16_hi(w[i].w)};
                    const float hv = (i < rows_here) ? bf16_to_float(h[(size_t)i * d + c]) : 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[i][e] = fmaf(hv, f[e], acc[i][e]);
                }
            }
        }
    }
    // lanes with equal (lane % 8) hold the same columns: butterfly over lane bits 3, 4, 5
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = acc[i][e];
            v += dpp_f32<0x128>(v);                             // row_ror:8  = lane ^ 8 inside a row of 16
            uint32_t a, b;
            swap_pair<16>(__float_as_uint(v), a, b);
            v = __uint_as_float(a) + __uint_as_float(b);
            swap_pair<32>(__float_as_uint(v), a, b);
            v = __uint_as_float(a) + __uint_as_float(b);
            if (lane < 8) redd[wave][i][lane * 8 + e] = v;
        }
    __syncthreads();
    for (int q = tid; q < R * kItemCols; q += NT) {
        const int i = q / kItemCols, c = q % kItemCols;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += redd[w][i][c];        // fixed order
        if (cb * kItemCols + c < r) tpart[((size_t)ds * R + i) * r + cb * kItemCols + c] = s;
    }
    __syncthreads();
}


// ---------------------------------------------------------------------------
// Shared memory of the chunk epilogue: the partial sums of the NW wavefronts that split the
// contraction, and the selection scratch of the wavefronts that reduce a row each.
template <int R, int NW>
struct ChunkLds {
    static constexpr int EW = (R < NW) ? R : NW;
    float red[NW][R][kChunkCols];
    uint64_t sel_cand[EW][kChunkCols];
};

// Row i of the chunk: fixed-order sum of the NW partial sums, then (max, sum of exp, top-k) of its
// 512 logits, written as the partial of (row, chunk).  One wavefront; all 64 lanes must call.
//
// Top-k in three steps whose cost does not grow with k, and which stay inside the wavefront (this is the tail of
// every block, after its last weight row has arrived: nothing overlaps it).  (1) T = the k-th largest of the 64
// lane maxima, found bit by bit from the top with one ballot and one population count per bit: an element below
// T is preceded by k lane maxima, so it cannot be in the top-k.  (2) The elements >= T (k or a few more; all of
// them when values tie) are compacted into shared memory through ballots and lane prefix counts.  (3) They are
// ranked among themselves by (logit desc, id asc) by counting.
// part_smp (may be null): the chunk's best z_v + g_v with standard Gumbel noise g (Gumbel-max sampling), as
// (z + g, id, z, -) of the winner; gk: the noise key of this row.
template <int R, int NW>
__device__ __forceinline__ void chunk_row_epilogue(ChunkLds<R, NW> &L, int i, int wave, int lane, bool active,
                                                   int col, int k, size_t slot,
                                                   float2 *__restrict__ part_ms, float *__restrict__ part_val,
                                                   int *__restrict__ part_id,
                                                   float4 *__restrict__ part_smp, const GumbelKey &gk)
{
    float z[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) z[e] = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {          // fixed order: wavefront 0 first
        const float4 *src = reinterpret_cast<const float4 *>(&L.red[w][i][lane * 8]);
        float4 a = src[0], b = src[1];
        z[0] += a.x; z[1] += a.y; z[2] += a.z; z[3] += a.w;
        z[4] += b.x; z[5] += b.y; z[6] += b.z; z[7] += b.w;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) z[e] = active ? z[e] : kNegInf;

    if (part_smp) {
        // keys are unique (one per id), so exactly one lane holds the wavefront's largest
        uint64_t best = kNoKey;
        float zb = 0.f;
        if (active) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint64_t key = make_key(z[e] + gumbel_base2(gk, (uint32_t)(col + e)) * kLn2, (uint32_t)(col + e));
                if (key > best) { best = key; zb = z[e]; }
            }
        }
        const uint64_t top = wave_max_key(best);
        if (active && best == top)
            part_smp[slot] = make_float4(key_value(top), __int_as_float((int)key_tiebreak(top)), zb, 0.f);
    }
    float lm = z[0];
#pragma unroll
    for (int e = 1; e < 8; ++e) lm = fmaxf(lm, z[e]);
    const float m = wave_max(lm);
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) s += fast_exp(z[e] - m);     // exp(-inf) = 0 for padding lanes
    s = wave_sum(s);

    // (1) T: the largest 32-bit pattern with at least k lane maxima at or above it (0 if fewer than k lanes hold columns)
    uint64_t *cand = L.sel_cand[wave];
    const uint32_t lane_bits = active ? float_order_bits(lm) : 0u;
    uint32_t T = 0u;
#pragma unroll
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t trial = T | (1u << bit);
        if (__popcll(__ballot(lane_bits >= trial)) >= k) T = trial;
    }
    // (2) every element at or above T is a candidate; slot = number of candidates before it (element-major, then lane)
    int n_cand = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const bool take = active && float_order_bits(z[e]) >= T;
        const uint64_t mask = __ballot(take);
        const int before = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
        if (take) cand[n_cand + before] = make_key(z[e], (uint32_t)(col + e));
        n_cand += __popcll(mask);
    }
    lds_wave_sync();
    // (3) rank the candidates among themselves by (value desc, id asc); ranks below k are the answer
    for (int c0 = 0; c0 < n_cand; c0 += 64) {
        const int c = c0 + lane;
        const uint64_t mine = (c < n_cand) ? cand[c] : kNoKey;
        int rk = 0;
#pragma unroll 8
        for (int q = 0; q < n_cand; ++q) rk += (cand[q] > mine) ? 1 : 0;
        if (c < n_cand && rk < k) {
            part_val[slot * k + rk] = key_value(mine);
            part_id[slot * k + rk] = (int)key_tiebreak(mine);
        }
    }
    if (lane >= n_cand && lane < k) {                  // fewer than k columns in this chunk
        part_val[slot * k + lane] = kNegInf;
        part_id[slot * k + lane] = kNoId;
    }
    if (lane == 0) part_ms[slot] = make_float2(m, s);
    lds_wave_sync();                                   // the buffers are reused by this wavefront's next row
}

// ---------------------------------------------------------------------------
// Merge of one row's chunk partials (running max m_c, sum of exp s_c, sorted top-k list per chunk):
//     lse = M + ln sum_c s_c exp(m_c - M),   M = max_c m_c
// and the k globally first (logit desc, id asc) candidates.  The order of every reduction is fixed
// and the selection works on unique keys, so the output does not depend on scheduling.
//
// Partials of one row cover increasing, disjoint id ranges and each list is already in output
// order, so "smaller list position e = c * k + p" breaks ties exactly like "smaller id".
//   (1) the k-th largest list head (by all-pairs counting) bounds the answer from below;
//   (2) the entries that reach the bound (at most k lists, k entries each) are gathered;
//   (3) they are ranked among themselves by counting; ranks below k are the output.
// NT threads (a multiple of 64, at most 1024) call together; `dyn` holds merge_lds_bytes(chunks, k, cache_ids).
struct MergeSmall {
    float red_m[16], red_s[16];
    uint64_t bound;
    uint32_t cnt;
    uint32_t winners[SLIMSPEC_KMAX_INTERNAL];
    uint64_t smp_key[16];
    float smp_z[16];
};

template <int NT>
__device__ __forceinline__ void merge_row(unsigned char *dyn, bool cache_ids, MergeSmall &S, int tid,
                                          const float2 *__restrict__ ms, const float *__restrict__ pv,
                                          const int *__restrict__ pi, int chunks, int k,
                                          int32_t *__restrict__ out_ids, float *__restrict__ out_logprobs,
                                          const int32_t *__restrict__ id_map,
                                          const float4 *__restrict__ smp, float *__restrict__ out_lse,
                                          int32_t *__restrict__ out_sample_id, float *__restrict__ out_sample_lp)
{
    constexpr int NWAVES = NT / 64;
    uint64_t *heads = reinterpret_cast<uint64_t *>(dyn);                      // [chunks]
    uint64_t *cand = heads + chunks;                                           // [k * k]
    float *vals = reinterpret_cast<float *>(cand + (size_t)k * k);            // [chunks * k]
    int *ids = reinterpret_cast<int *>(vals + (size_t)chunks * k);            // [chunks * k]
    const int lane = tid & 63, wave = tid >> 6;

    const int n = chunks * k;
    // The partials were written by other CUs: every load is a trip to the memory side.  All loads of a thread are
    // therefore issued before the first of them is used (four list entries per thread and trip, and the first
    // chunk's head and (max, sum) with them), instead of one trip per loop iteration.
    const bool own_chunk = tid < chunks;
    const float head0 = own_chunk ? pv[(size_t)tid * k] : 0.f;
    const float2 ms0 = own_chunk ? ms[tid] : make_float2(kNegInf, 0.f);
    for (int e0 = tid; e0 < n; e0 += 4 * NT) {
        float v[4];
        int id[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = min(e0 + u * NT, n - 1);
            v[u] = pv[e];
            id[u] = cache_ids ? pi[e] : 0;              // when they fit: no dependent load at the end
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = e0 + u * NT;
            if (e < n) {
                vals[e] = v[u];
                if (cache_ids) ids[e] = id[u];
            }
        }
    }
    if (tid == 0) { S.bound = kNoKey; S.cnt = 0u; }

    // log-sum-exp: every thread folds its chunks in increasing order, then the block combines
    float m_t = kNegInf, s_t = 0.f;
    for (int c = tid; c < chunks; c += NT) {
        const bool first = c == tid;
        heads[c] = make_key(first ? head0 : pv[(size_t)c * k], (uint32_t)(c * k));
        float2 p = first ? ms0 : ms[c];
        float m_new = fmaxf(m_t, p.x);
        s_t = s_t * fast_exp(m_t - m_new) + p.y * fast_exp(p.x - m_new);
        m_t = m_new;
    }
    const float m_w = wave_max(m_t);
    float s_w = (m_t == kNegInf) ? 0.f : s_t * fast_exp(m_t - m_w);
    s_w = wave_sum(s_w);
    if (lane == 0) { S.red_m[wave] = m_w; S.red_s[wave] = s_w; }
    __syncthreads();
    float M = S.red_m[0];
#pragma unroll
    for (int w = 1; w < NWAVES; ++w) M = fmaxf(M, S.red_m[w]);
    float Ssum = 0.f;
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) Ssum += (S.red_m[w] == kNegInf) ? 0.f : S.red_s[w] * fast_exp(S.red_m[w] - M);
    const float lse = M + fast_log(Ssum);
    if (smp) {
        // stochastic-decoding outputs: the row's log-sum-exp and the Gumbel-max draw (largest z + g over the chunks)
        uint64_t best = kNoKey;
        float zb = 0.f;
        for (int c = tid; c < chunks; c += NT) {
            const float4 e = smp[c];
            const uint64_t key = make_key(e.x, (uint32_t)__float_as_int(e.y));
            if (key > best) { best = key; zb = e.z; }
        }
        const uint64_t top_w = wave_max_key(best);
        if (lane == 0) S.smp_key[wave] = top_w;
        if (best == top_w && best != kNoKey) S.smp_z[wave] = zb;
        __syncthreads();
        if (tid == 0) {
            int wb = 0;
            for (int w = 1; w < NWAVES; ++w) if (S.smp_key[w] > S.smp_key[wb]) wb = w;
            const int id = (int)key_tiebreak(S.smp_key[wb]);
            *out_lse = lse;
            *out_sample_id = id_map ? id_map[id] : id;
            *out_sample_lp = S.smp_z[wb] - lse;
        }
    }

    // (1) the k-th largest head: four adjacent lanes share one head, each counts a quarter of the others
    {
        const int quarter = (chunks + 3) / 4;
        const int q0 = (tid & 3) * quarter, q1 = min(chunks, q0 + quarter);
        for (int c0 = 0; c0 < chunks; c0 += NT / 4) {              // trip count uniform over the block
            const int c = c0 + (tid >> 2);
            const uint64_t mine = heads[min(c, chunks - 1)];
            int rank = 0;
#pragma unroll 8
            for (int q = q0; q < q1; ++q) rank += (heads[q] > mine) ? 1 : 0;
            rank += __shfl_xor(rank, 1);
            rank += __shfl_xor(rank, 2);
            if (c < chunks && (tid & 3) == 0 && rank == k - 1) S.bound = mine;      // keys are unique: one writer at most
        }
    }
    __syncthreads();
    const uint64_t bound = S.bound;                     // kNoKey when there are fewer than k lists: keep everything
    // (2) gather what reaches the bound
    for (int c = tid; c < chunks; c += NT) {
        if (heads[c] < bound) continue;
        for (int p = 0; p < k; ++p) {
            const float v = vals[c * k + p];
            const uint64_t key = make_key(v, (uint32_t)(c * k + p));
            if (v == kNegInf || key < bound) break;     // lists are sorted
            cand[atomicAdd(&S.cnt, 1u)] = key;
        }
    }
    __syncthreads();
    // (3) rank the gathered entries
    const int n_cand = (int)S.cnt;
    for (int c = tid; c < n_cand; c += NT) {
        const uint64_t mine = cand[c];
        int rank = 0;
#pragma unroll 8
        for (int q = 0; q < n_cand; ++q) rank += (cand[q] > mine) ? 1 : 0;
        if (rank < k) S.winners[rank] = key_tiebreak(mine);
    }
    __syncthreads();
    if (tid < k) {                                      // n_cand >= k whenever k <= V
        const uint32_t e = S.winners[tid];
        const int id = cache_ids ? ids[e] : pi[e];
        out_ids[tid] = id_map ? id_map[id] : id;                // truncated vocabulary: column -> vocabulary id
        out_logprobs[tid] = vals[e] - lse;
    }
    __syncthreads();                                    // the buffers may be reused for the next row
}

}  // namespace slimspec

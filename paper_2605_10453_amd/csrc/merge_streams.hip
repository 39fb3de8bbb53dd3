// Merge for the matrix-core path: one block per row turns the row's stream records (one per block of
// head_tile_kernel that worked on the row, see head_tile.hip) into the final top-k ids and log-probabilities.
//
// What a stream tells about its share of the row's logits (all values as computed by the
// matrix cores, i.e. with a 16-bit contraction input in the low-rank head):
//   * L listed groups of 16 logits: the group maximum x (its low 4 bits name its position in the
//     group), the second largest value y of the group, a tag naming the group;
//   * U: an upper bound of every logit in its unlisted groups.
// Let tau be the k-th largest listed maximum and eps_v a bound of |computed - exact| for column v (the same for
// all columns of a 256-column vocabulary tile: see below), eps the largest of them.  Every logit that can be among
// the exact top-k is computed >= tau - eps - eps_v, in particular >= tau - 2 eps =: theta.  The block therefore
// collects (a) listed maxima >= theta, (b) the other 15 members of listed groups whose second
// largest value reaches theta, (c) all members of unlisted groups of streams with U >= theta
// (b and c are rare), evaluates exactly, in fp32 from the fp32 contraction input, every
// collected logit whose rank is not already certain (members under b and c, and listed maxima
// within 2 eps of another collected value), and ranks the collected set by (value desc, id asc).
// If the collected set outgrows its buffer (possible only with thousands of near-ties at the
// k-th place) the block falls back to an exhaustive exact pass over the row's whole vocabulary.
//
// log-sum-exp: streams carry (max * log2 e, sum of 2^(z log2 e - max)); combined in a fixed order.  The sum is
// made of computed logits: the term of every re-evaluated logit is replaced by its exact one (a listed maximum has
// its recorded value; for any other column the computed logit is recomputed from the same 16-bit rounding of the
// contraction input).  With a wide bound the row's probable tokens are re-evaluated for that purpose alone, and two
// guards send a row whose remaining error could still be seen to the exhaustive pass (see kWideEps below).
#include "device_utils.hpp"
#include "launch.hpp"

namespace slimspec {

namespace {

constexpr int kWorkCap = 2048;          // collected logits per row before the exhaustive fallback
// The exhaustive pass scans kMergeThreads * 4 columns per step; every one of them may beat the running k-th key
// (logits rising with the column id), and the k keys kept from the step before come on top.
constexpr int kExhaustCap = kMergeThreads * 4 + SLIMSPEC_KMAX_INTERNAL;
static_assert(kMergeThreads * 4 <= kWorkCap, "a step of the exhaustive pass appends at most kWorkCap keys");
constexpr float kNoValue = -1.0e38f;    // stream fields at or below this are empty
constexpr float kExactWinnersEps = 8.0e-3f;   // largest eps at which a computed winner's log-probability is reported as is
static_assert(kStreamsPerBlock == 4, "a record's place in its block names (column half, half-wavefront)");
constexpr int kCrowdCap = 8;              // streams of a row whose unlisted groups are all listed member by member (more: exhaustive pass)
constexpr int kGatherRound = 32;          // columns of a column-major copy evaluated per round of loads
constexpr float kExhaustiveEps = 0.25f;       // from this eps on the row takes the exhaustive exact pass
// The streams' sum of exponentials is made of computed logits; the merge replaces the terms of the logits it
// re-evaluates, so what remains of its error is the probability-weighted mean error of all the others.  With a wide
// bound (eps above kWideEps) the row's probable tokens are therefore collected and re-evaluated as well, winners or
// not: every listed maximum of probability >= kMassCut / eps.  If the tokens left over still hold so much mass that
// errors of one sign at the bound would move the log-sum-exp by more than kLseGuard, the row is done exhaustively
// (a guard for bounds close to kExhaustiveEps: the exhaustive pass costs milliseconds per row, and at 2.5e-2 the
// peaked rows of a 512-row batch at r = 1024, whose real error is a tenth of that, already tripped it).
constexpr float kWideEps = 8.0e-3f;      // (= kExactWinnersEps: from here on every winner is re-evaluated anyway)
constexpr float kMassCut = 5.0e-4f;
constexpr float kLseGuard = 1.0e-1f;
constexpr float kCommonModeTol = 1.0e-2f;
constexpr int kListedBit = 1 << 30;     // marks, in the list of items to evaluate, a listed maximum (it has a computed value)
constexpr int kSampleBit = 1 << 29;     // ... an entry of the sampling contenders' list (smp_id / smp_z) instead
constexpr float kEpsSigmas = 4.0f;      // eps_v = this many standard deviations of the rounding error of t in column v
                                        // (values are re-evaluated when within eps_a + eps_b = 5.6 sigma of their difference)
constexpr int kSampleCap = 32;          // streams whose best z + g may be the row's Gumbel-max draw, at most
constexpr int kTsCap = 4096;            // vocabulary tiles whose column scale is kept in shared memory (1 M columns)
constexpr float kEpsViolation = 1.5f;   // a re-evaluated value further than this many eps_v from its computed value
                                        // shows that the bound does not hold for this input: the row is done exhaustively

// Deferred exact evaluation (long contractions, i.e. the full head).  A column of M is one 2-byte element per row,
// every row in a cache line and mostly a page of its own; one block (one CU) gets through only about 160 such lines
// per microsecond, so a row that has to re-evaluate 16 columns over K = 4096 would hold the whole launch up for
// 25 us per batch.  With a deferral buffer the merge kernel instead parks such a row (its collected set and the
// list of columns to evaluate), exact_cols_kernel spreads the row's gathers over kDeferSlices blocks, and a second
// launch of the merge kernel (resume = 1) picks the parked rows up after the evaluation.  Rows whose lists do not
// fit the buffer are evaluated in place as before.
constexpr int kDeferNeed = 1280;        // columns to evaluate per parked row, at most (a whole stream's unlisted groups
                                        // at the 512-row shape: about 1000)
constexpr int kDeferWork = 1536;        // collected logits per parked row, at most
constexpr int kDeferSlices = 16;        // blocks that share one row's gathers (slices of the contraction)
constexpr int kDeferHeader = 16;        // ints: [0] n_need (0: not parked), [1] n_work, [2] S, [3] Mx, [4] lse (floats)
constexpr size_t kDeferRowInts = kDeferHeader + kDeferNeed + 3 * kDeferWork + (size_t)kDeferSlices * kDeferNeed;

struct ParkedRow { int *hdr, *need, *id; float *val, *eps, *part; };     // part: [kDeferSlices][kDeferNeed]
__device__ __forceinline__ ParkedRow parked_row(int *defer, int row) {
    ParkedRow p{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    if (defer) {
        p.hdr = defer + (size_t)row * kDeferRowInts;
        p.need = p.hdr + kDeferHeader;
        p.id = p.need + kDeferNeed;
        p.val = reinterpret_cast<float *>(p.id + kDeferWork);
        p.eps = p.val + kDeferWork;
        p.part = p.eps + kDeferWork;
    }
    return p;
}

__device__ __forceinline__ float mask4(float v) { return __uint_as_float(__float_as_uint(v) & 0xfffffff0u); }

struct RowCtx {
    const void *x; int x_is_bf16;       // exact contraction input of this row: fp32 t or bf16 h
    const uint16_t *M; int K, V;
};

__device__ __forceinline__ float x_at(const RowCtx &c, int j) {
    return c.x_is_bf16 ? bf16_to_float(static_cast<const uint16_t *>(c.x)[j]) : static_cast<const float *>(c.x)[j];
}

// rank of every key among keys[0, n) by counting; calls f(index, key, rank) for this thread's keys
template <class F>
__device__ __forceinline__ void rank_all_pairs(const uint64_t *keys, int n, int tid, int nthreads, F f) {
    for (int c = tid; c < n; c += nthreads) {
        const uint64_t mine = keys[c];
        int rank = 0;
#pragma unroll 8
        for (int q = 0; q < n; ++q) rank += (keys[q] > mine) ? 1 : 0;
        f(c, mine, rank);
    }
}

// Sum of v over every aligned group of P adjacent lanes (P a power of two, at most 64; the same in all lanes of the
// group).  All lanes of the wavefront must be active at the call.
__device__ __forceinline__ int lanes_sum(int v, int P) {
    if (P > 1) v += (int)dpp_u32<0xB1>((uint32_t)v);
    if (P > 2) v += (int)dpp_u32<0x4E>((uint32_t)v);
    if (P > 4) v += (int)dpp_u32<0x141>((uint32_t)v);
    if (P > 8) v += (int)dpp_u32<0x140>((uint32_t)v);
    uint32_t a, b;
    if (P > 16) { swap_pair<16>((uint32_t)v, a, b); v = (int)(a + b); }
    if (P > 32) { swap_pair<32>((uint32_t)v, a, b); v = (int)(a + b); }
    return v;
}
// Lanes that share the scan for one of n items when nthreads threads work on them: the largest power of two P with
// n P <= nthreads (1 when there are more items than threads); returns log2 P.
__device__ __forceinline__ int lanes_per_item_log2(int n, int nthreads) {
    int p = 0;
    while (p < 6 && (2 * n << p) <= nthreads) ++p;
    return p;
}
// Slots of a shared list for the lanes of a wavefront that have `take` set: one atomic per wavefront instead of one per
// lane (a thousand atomics on one shared-memory counter take tens of microseconds).  Every lane of the wavefront calls.
__device__ __forceinline__ uint32_t wave_slots(uint32_t *counter, bool take, int &n_taken) {
    const uint64_t mask = __ballot(take);
    n_taken = __popcll(mask);
    uint32_t base = 0u;
    if (n_taken != 0) {
        const int before = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
        if (take && before == 0) base = atomicAdd(counter, (uint32_t)n_taken);
        base = (uint32_t)__shfl((int)base, __ffsll((unsigned long long)mask) - 1) + (uint32_t)before;
    }
    return base;
}

// rank_all_pairs with the scan for every key shared by P adjacent lanes (few keys, many threads: the ranking is a
// chain of shared-memory reads, and P lanes make it P times shorter).  Every thread of the block must call it.
template <class F>
__device__ __forceinline__ void rank_all_pairs_wide(const uint64_t *keys, int n, int tid, int nthreads, F f) {
    const int p = lanes_per_item_log2(n, nthreads), P = 1 << p;
    if (p == 0) { rank_all_pairs(keys, n, tid, nthreads, f); return; }
    const int c = tid >> p, part = tid & (P - 1);
    const uint64_t mine = (c < n) ? keys[c] : kNoKey;
    int rank = 0;
    if (c < n) {
#pragma unroll 4
        for (int q = part; q < n; q += P) rank += (keys[q] > mine) ? 1 : 0;
    }
    rank = lanes_sum(rank, P);
    if (c < n && part == 0) f(c, mine, rank);
}

// This lane's share (one of PH lanes) of the rank of `mine` among the 64 stream heads of its group
template <int PH>
__device__ __forceinline__ int head_rank_share(const uint64_t *group, int part, uint64_t mine) {
    const uint4 *grp = reinterpret_cast<const uint4 *>(group);      // 64 keys, two per 16-byte read
    int rank = 0;
#pragma unroll
    for (int q = 0; q < 32 / PH; ++q) {
        const uint4 v = grp[part + q * PH];
        rank += (u64_from(v.y, v.x) > mine ? 1 : 0) + (u64_from(v.w, v.z) > mine ? 1 : 0);
    }
    return rank;
}

}  // namespace

// so.on (sampling calls): the records have rec_stride = kStreamRecSample floats and also carry every stream's best
// and second best z + g (Gumbel noise); the row's draw is the largest over the streams, decided on exact logits
// for every stream whose best is within the rounding bound of the largest.
__global__ __launch_bounds__(kMergeThreads) void merge_streams_kernel(
    const float *__restrict__ part, int rec_stride, int nsr, int gw, int n_vt,
    const void *__restrict__ xexact, int x_is_bf16, int ldx,
    int operand16,      // 0: the head kernel's row operand was exact; 1: it was t log2(e) rounded to bf16; 2: to f16
    const uint16_t *__restrict__ M, int K, int V,
    const uint16_t *__restrict__ Mt,      // null, or the caller's column-major copy of M, [V, K]: a column is K adjacent elements
    const float2 *__restrict__ stat, int n_stat, int rows_pad, const float2 *__restrict__ tilescale,
    int k, float unit, float tiny_w, int32_t *__restrict__ out_ids, float *__restrict__ out_logprobs,
    const int32_t *__restrict__ id_map, int *__restrict__ defer, int resume, SampleOut so, int row_base)
{
    constexpr int L = kStreamList, REC = kStreamRec, NT = kMergeThreads, NWAVES = kMergeThreads / 64;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int n = nsr * L;
    const int ngroups = (nsr + 63) / 64;                                // groups of 64 stream heads
    uint64_t *keys = reinterpret_cast<uint64_t *>(lds_raw);            // [n]            every listed maximum
    uint64_t *hkeys = keys + n;                                         // [ngroups * 64] the streams' largest maxima, padded with kNoKey
    uint64_t *surv = hkeys + (size_t)ngroups * 64;                      // [max(ngroups, 3) * k]  best k of every 64 heads; then the candidates for tau
    // (the final keys and the fallback's buffer lie over the three arrays above, which are dead by then)
    uint64_t *work = keys;                                              // [kExhaustCap]  final keys / fallback buffer
    const size_t n_front = (size_t)n + (size_t)ngroups * 64 + (size_t)(ngroups > 3 ? ngroups : 3) * k;
    int *w_id = reinterpret_cast<int *>(keys + (n_front > (size_t)kExhaustCap ? n_front : (size_t)kExhaustCap));   // [kWorkCap]
    float *w_val = reinterpret_cast<float *>(w_id + kWorkCap);          // [kWorkCap]
    int *w_need = reinterpret_cast<int *>(w_val + kWorkCap);            // [kWorkCap]     0 no, 1 / 2 yes; later: list of items to evaluate
    float *w_apx = reinterpret_cast<float *>(w_need + kWorkCap);        // [kWorkCap]     change of the item's term of the sum of exp; later by rank
    float *w_eps = w_apx + kWorkCap;                                    // [kWorkCap]     the item's bound eps_v
    float *ts = w_eps + kWorkCap;                                       // [min(n_vt, kTsCap)]  column scale of B per vocabulary tile
    const bool ts_cached = n_vt <= kTsCap;                              // a larger vocabulary uses the largest scale for every tile
    float *xrow = ts + ((min(n_vt, kTsCap) + 3) & ~3);                  // [K]            the row's exact contraction input
    float *xrow16 = xrow + K;                                           // [K]            ... as the head kernel had it (operand16 != 0)
    __shared__ float red_m[NWAVES], red_s[NWAVES];
    __shared__ uint64_t tau_key;
    __shared__ uint32_t cnt_surv, cnt_work, cnt_hidden, cnt_need;
    __shared__ int tau_slot, eps_violated;
    __shared__ uint32_t cnt_crowd;                                      // streams whose best unlisted group is a candidate
    __shared__ int crowd[kCrowdCap];
    __shared__ float mass_eval_sh;
    __shared__ uint64_t smp_wkey[NWAVES];                               // sampling: per-wavefront reductions
    __shared__ float smp_wz[NWAVES], smp_w2[NWAVES], lse_out_sh;
    __shared__ int smp_id[kSampleCap];
    __shared__ float smp_z[kSampleCap];
    __shared__ uint32_t smp_cnt;
    __shared__ uint64_t thr_key;
    __shared__ uint32_t cnt_buf;
    __shared__ uint32_t winners[SLIMSPEC_KMAX_INTERNAL];

    const int row = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *rec = part + (size_t)row * nsr * rec_stride;
    const GumbelKey gk = gumbel_key(so.seed_lo, so.seed_hi, (uint32_t)(row_base + row));
    // The block's largest key and the z that goes with it, in every thread (keys are unique or kNoKey).
    const auto block_best = [&](uint64_t key, float z, float &z_out) {
        const uint64_t top_w = wave_max_key(key);
        __syncthreads();
        if (lane == 0) smp_wkey[wave] = top_w;
        if (key == top_w && key != kNoKey) smp_wz[wave] = z;
        __syncthreads();
        int wb = 0;
#pragma unroll
        for (int w = 1; w < NWAVES; ++w) if (smp_wkey[w] > smp_wkey[wb]) wb = w;
        z_out = smp_wz[wb];
        return smp_wkey[wb];
    };
    const auto write_sample = [&](uint64_t key, float z, float lse_final) {
        if (tid == 0) {
            const int id = (int)key_tiebreak(key);
            so.lse[row_base + row] = lse_final;
            so.sample_ids[row_base + row] = id_map ? id_map[id] : id;
            so.sample_logprobs[row_base + row] = z - lse_final;
        }
    };
    RowCtx ctx;
    ctx.x = x_is_bf16 ? static_cast<const void *>(static_cast<const uint16_t *>(xexact) + (size_t)row * ldx)
                      : static_cast<const void *>(static_cast<const float *>(xexact) + (size_t)row * ldx);
    ctx.x_is_bf16 = x_is_bf16; ctx.M = M; ctx.K = K; ctx.V = V;
    const ParkedRow pk = parked_row(defer, row);
    int *const park = pk.hdr, *const park_need = pk.need, *const park_id = pk.id;
    float *const park_val = pk.val, *const park_eps = pk.eps, *const park_part = pk.part;

    // The tail of the row's merge once every collected logit has its final value: rank the collected set, correct
    // the sum of exp by the changes of the re-evaluated terms (summed in rank order: a fixed order), write.
    const auto finish = [&](int n_work, float S, float Mx, float lse) {
        for (int c = tid; c < n_work; c += NT) work[c] = make_key(w_val[c], (uint32_t)w_id[c]);
        __syncthreads();
        float *by_rank = reinterpret_cast<float *>(w_need);
        rank_all_pairs_wide(work, n_work, tid, NT, [&](int c, uint64_t, int rank) {
            if (rank < k) winners[rank] = (uint32_t)c;
            by_rank[rank] = w_apx[c];
        });
        __syncthreads();
        float corr = 0.f;
        for (int q = 0; q < n_work; ++q) corr += by_rank[q];
        const float s_fixed = S + corr;
        const float lse_fixed = (s_fixed > 0.f) ? (Mx + __builtin_amdgcn_logf(s_fixed)) * kLn2 : lse;
        if (tid == 0) lse_out_sh = lse_fixed;
        if (tid < k) {
            const uint32_t c = winners[tid];
            out_ids[(size_t)row * k + tid] = id_map ? id_map[w_id[c]] : w_id[c];
            out_logprobs[(size_t)row * k + tid] = w_val[c] - lse_fixed;
        }
    };
    // A listed maximum had its computed value in the streams' sum of exp: remember by how much its term changes.
    // ... and check it against the bound that decided what to re-evaluate.
    // A member of a group that is not the listed maximum has no recorded value; z16 is its logit recomputed from the
    // 16-bit contraction input (what the head kernel added to the sum of exp, up to the order of the additions).
    const auto take_exact = [&](int entry, float z, float z16, float Mx) {
        const int item = entry & (kListedBit - 1);
        if (entry & kListedBit) {
            if (fabsf(z - w_val[item]) > kEpsViolation * w_eps[item]) eps_violated = 1;
            w_apx[item] = __builtin_amdgcn_exp2f(z * kLog2e - Mx) - __builtin_amdgcn_exp2f(w_val[item] * kLog2e - Mx);
        } else {
            if (fabsf(z - z16) > kEpsViolation * w_eps[item]) eps_violated = 1;
            w_apx[item] = __builtin_amdgcn_exp2f(z * kLog2e - Mx) - __builtin_amdgcn_exp2f(z16 * kLog2e - Mx);
        }
        w_val[item] = z;
    };

    // ---- exhaustive exact pass: every logit of the row in fp32, running top-k in `work`
    // (also recomputes the log-sum-exp, since the streams' sums may have overflowed)
    const auto exhaustive_pass = [&]() {
    __syncthreads();
    if (tid == 0) { thr_key = kNoKey; cnt_buf = 0u; }
    __syncthreads();
    float em = kNegInf, es = 0.f;
    uint64_t sbest = kNoKey;                                  // sampling: this thread's largest z + g and its z
    float sbest_z = 0.f;
    for (int c0 = 0; c0 < V; c0 += NT * 4) {
        const int col = c0 + tid * 4;
        if (col < V) {
            float z[4] = {0.f, 0.f, 0.f, 0.f};
            constexpr int NJ = 8;                              // rows of M in flight per thread (summed in row order)
            for (int j0 = 0; j0 < K; j0 += NJ) {
                uint2 w[NJ];
#pragma unroll
                for (int u = 0; u < NJ; ++u) w[u] = *reinterpret_cast<const uint2 *>(M + (size_t)min(j0 + u, K - 1) * V + col);
#pragma unroll
                for (int u = 0; u < NJ; ++u) {
                    const float xj = (j0 + u < K) ? x_at(ctx, j0 + u) : 0.f;
                    z[0] = fmaf(xj, bf16_lo(w[u].x), z[0]); z[1] = fmaf(xj, bf16_hi(w[u].x), z[1]);
                    z[2] = fmaf(xj, bf16_lo(w[u].y), z[2]); z[3] = fmaf(xj, bf16_hi(w[u].y), z[3]);
                }
            }
            const uint64_t thr = thr_key;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float m_new = fmaxf(em, z[e]);
                es = es * fast_exp(em - m_new) + fast_exp(z[e] - m_new);
                em = m_new;
                const uint64_t key = make_key(z[e], (uint32_t)(col + e));
                if (key > thr) work[atomicAdd(&cnt_buf, 1u)] = key;     // at most k + 4 NT = kExhaustCap entries: fits
                if (so.on) {
                    const uint64_t skey = make_key(z[e] + gumbel_base2(gk, (uint32_t)(col + e)) * kLn2, (uint32_t)(col + e));
                    if (skey > sbest) { sbest = skey; sbest_z = z[e]; }
                }
            }
        }
        __syncthreads();
        const int nb = (int)cnt_buf;
        constexpr int PER_X = (kExhaustCap + NT - 1) / NT;
        uint64_t mykey[PER_X];
        int myrank[PER_X];
        int cnt_mine = 0;
        rank_all_pairs(work, nb, tid, NT, [&](int, uint64_t key, int rank) { mykey[cnt_mine] = key; myrank[cnt_mine] = rank; ++cnt_mine; });
        __syncthreads();
        for (int q = 0; q < cnt_mine; ++q)
            if (myrank[q] < k) { work[myrank[q]] = mykey[q]; if (myrank[q] == k - 1) thr_key = mykey[q]; }
        if (tid == 0) cnt_buf = (uint32_t)min(nb, k);
        __syncthreads();
    }
    // exact log-sum-exp of the row
    const float em_w = wave_max(em);
    float es_w = (em == kNegInf) ? 0.f : es * fast_exp(em - em_w);
    es_w = wave_sum(es_w);
    __syncthreads();
    if (lane == 0) { red_m[wave] = em_w; red_s[wave] = es_w; }
    __syncthreads();
    float EM = red_m[0];
#pragma unroll
    for (int w = 1; w < NWAVES; ++w) EM = fmaxf(EM, red_m[w]);
    float ES = 0.f;
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) ES += (red_m[w] == kNegInf) ? 0.f : red_s[w] * fast_exp(red_m[w] - EM);
    const float lse_exact = EM + fast_log(ES);
    if (tid < k) {                                          // work[0..k) is sorted by rank
        const int id = (int)key_tiebreak(work[tid]);
        out_ids[(size_t)row * k + tid] = id_map ? id_map[id] : id;
        out_logprobs[(size_t)row * k + tid] = key_value(work[tid]) - lse_exact;
    }
    if (so.on) {
        float zs;
        const uint64_t top = block_best(sbest, sbest_z, zs);
        write_sample(top, zs, lse_exact);
    }
    };

    if (resume) {
        // second launch: only rows parked by the first one; their columns have been evaluated in between
        const int n_need = park[0];
        if (n_need == 0) return;
        const int n_work = park[1];
        const float S = __int_as_float(park[2]), Mx = __int_as_float(park[3]), lse = __int_as_float(park[4]);
        for (int c = tid; c < n_work; c += NT) { w_id[c] = park_id[c]; w_val[c] = park_val[c]; w_eps[c] = park_eps[c]; w_apx[c] = 0.f; }
        if (tid == 0) eps_violated = 0;
        __syncthreads();
        for (int i = tid; i < n_need; i += NT) {           // every entry names its own item: no two threads share a slot
            float z = 0.f;
#pragma unroll
            for (int ks = 0; ks < kDeferSlices; ++ks) z += park_part[ks * kDeferNeed + i];      // fixed order
            take_exact(park_need[i], z, z, Mx);          // (rows with unlisted members on a rounded operand are not parked)
        }
        __syncthreads();
        if (eps_violated) { exhaustive_pass(); return; }
        finish(n_work, S, Mx, lse);
        return;
    }
    if (tid == 0) {
        tau_key = kNoKey; cnt_surv = 0u; cnt_work = 0u; cnt_hidden = 0u; cnt_need = 0u; cnt_crowd = 0u; tau_slot = -1; eps_violated = 0;
        if (park) park[0] = 0;                              // not parked, unless decided otherwise below
    }

    // a stream record as three 16-byte loads; the thread's first stream stays in registers
    static_assert(REC == 12, "three float4 per record");
    typedef float f32x4 __attribute__((ext_vector_type(4)));      // native vectors stay in registers (a float4 array did not)
    // Every global load of the prologue is issued before the first of them is used (one trip to the memory side
    // instead of three): the first element(s) of the contraction input, of the column scales and of the rounding
    // statistics, then the thread's stream record.
    const float x_first = (tid < K) ? x_at(ctx, tid) : 0.f;
    float2 ts_first0 = make_float2(0.f, 0.f), ts_first1 = make_float2(0.f, 0.f);
    if (tilescale != nullptr) {
        if (tid < n_vt) ts_first0 = tilescale[tid];
        if (tid + NT < n_vt) ts_first1 = tilescale[tid + NT];
    }
    // squared norm of t - rounded t: lane q of the first wavefront adds the row's entries q, q + 64, ... in order
    float dt2_mine = 0.f, tdt_mine = 0.f;               // ... and of t . (t - rounded t)
    if (stat != nullptr && tid < 64)
        for (int q = tid; q < n_stat; q += 64) {
            const float2 sq = stat[(size_t)q * rows_pad + row];
            dt2_mine += sq.x;
            tdt_mine += sq.y;
        }
    const f32x4 *mine_src = reinterpret_cast<const f32x4 *>(rec + (size_t)min(tid, nsr - 1) * rec_stride);
    const f32x4 mine0 = mine_src[0], mine1 = mine_src[1], mine2 = mine_src[2];
    auto load_rec = [&](int sidx, float (&f)[REC]) {
        f32x4 a = mine0, b = mine1, c = mine2;
        if (sidx != tid) {
            const f32x4 *src = reinterpret_cast<const f32x4 *>(rec + (size_t)sidx * rec_stride);
            a = src[0]; b = src[1]; c = src[2];
        }
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
        f[8] = c.x; f[9] = c.y; f[10] = c.z; f[11] = c.w;
    };

    // ---- log-sum-exp of the streams, and the squared norm of the row's contraction input
    float m_t = kNegInf, s_t = 0.f, x2 = 0.f, x1 = 0.f;
    for (int sidx = tid; sidx < nsr; sidx += NT) {
        float f[REC];
        load_rec(sidx, f);
        const float mc = f[0], s = f[1];
        if (!(s <= 0.f)) {      // (a sum that overflowed in the head kernel is +inf or NaN: it must reach the check of lse below)
            const float m_new = fmaxf(m_t, mc);
            s_t = s_t * __builtin_amdgcn_exp2f(m_t - m_new) + s * __builtin_amdgcn_exp2f(mc - m_new);
            m_t = m_new;
        }
    }
    for (int j = tid; j < K; j += NT) {
        const float v = (j == tid) ? x_first : x_at(ctx, j);
        xrow[j] = v; x2 += v * v; x1 += fabsf(v);
        if (operand16) xrow16[j] = operand_value(v, operand16 == 2);
    }
    __shared__ float dt2_sh, tdt_sh;
    // Column scale of B per vocabulary tile (asked for early: by the time eps needs it, it has arrived): the largest
    // column rms of the tile, and the rms of all of B from the tiles' mean squares (added in a fixed order).
    float ts_max = 0.f, ts_msq = 0.f;
    if (tilescale != nullptr)
        for (int i = tid; i < n_vt; i += NT) {
            const float2 v = (i < NT) ? ts_first0 : (i < 2 * NT) ? ts_first1 : tilescale[i];
            if (ts_cached) ts[i] = v.x;
            ts_max = fmaxf(ts_max, v.x);
            ts_msq += v.y;
        }
    __shared__ float red_ts[NWAVES], red_tq[NWAVES];
    if (wave == 0) {                                          // (fixed order: the lanes' sums, then the DPP tree)
        const float dt2_w = wave_sum(dt2_mine), tdt_w = wave_sum(tdt_mine);
        if (lane == 0) { dt2_sh = dt2_w; tdt_sh = tdt_w; }
    }
    const float m_w = wave_max(m_t);
    float s_w = (m_t == kNegInf) ? 0.f : s_t * __builtin_amdgcn_exp2f(m_t - m_w);
    s_w = wave_sum(s_w);
    x2 = wave_sum(x2);
    x1 = wave_sum(x1);
    if (lane == 0) { red_m[wave] = m_w; red_s[wave] = s_w; }
    __shared__ float red_x[NWAVES];
    __shared__ float red_x1[NWAVES];
    ts_max = wave_max(ts_max);
    ts_msq = wave_sum(ts_msq);
    if (lane == 0) { red_x[wave] = x2; red_x1[wave] = x1; red_ts[wave] = ts_max; red_tq[wave] = ts_msq; }
    // ---- keys of the listed maxima
    for (int sidx = tid; sidx < nsr; sidx += NT) {
        float f[REC];
        load_rec(sidx, f);
#pragma unroll
        for (int l = 0; l < L; ++l) {
            const float x = f[3 + 3 * l];
            keys[sidx * L + l] = (x > kNoValue) ? make_key(mask4(x) * unit, (uint32_t)(sidx * L + l)) : kNoKey;
        }
    }
    for (int sidx = tid; sidx < ngroups * 64; sidx += NT) hkeys[sidx] = (sidx < nsr) ? keys[sidx * L] : kNoKey;   // own writes
    __syncthreads();
    float Mx = red_m[0], X2 = 0.f, X1 = 0.f;
#pragma unroll
    for (int w = 1; w < NWAVES; ++w) Mx = fmaxf(Mx, red_m[w]);
    float S = 0.f;
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) {
        S += (red_m[w] == kNegInf) ? 0.f : red_s[w] * __builtin_amdgcn_exp2f(red_m[w] - Mx);
        X2 += red_x[w];
        X1 += red_x1[w];
        ts_max = fmaxf(ts_max, red_ts[w]);
    }
    float b_rms = 0.f;
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) b_rms += red_tq[w];
    b_rms = sqrtf(b_rms / (float)n_vt);
    const float lse = (Mx + __builtin_amdgcn_logf(S)) * kLn2;

    if (X2 == 0.f) {
        // zero contraction input (for instance a padded batch slot): every logit is exactly +0
        if (tid < k) {
            out_ids[(size_t)row * k + tid] = id_map ? id_map[tid] : tid;
            out_logprobs[(size_t)row * k + tid] = -__builtin_amdgcn_logf((float)V) * kLn2;
        }
        if (so.on) {                                        // the draw: the largest noise alone
            uint64_t best = kNoKey;
            for (int v = tid; v < V; v += NT) {
                const uint64_t key = make_key(gumbel_base2(gk, (uint32_t)v) * kLn2, (uint32_t)v);
                if (key > best) best = key;
            }
            float zs;
            const uint64_t top = block_best(best, 0.f, zs);
            write_sample(top, 0.f, __builtin_amdgcn_logf((float)V) * kLn2);
        }
        return;
    }
    // ---- tau: the k-th largest listed maximum.  The lists are sorted, so first T = the k-th largest of the
    // streams' heads (best k of every 64 heads, then all pairs); every listed maximum >= T (at most 3 k of them,
    // all of them if there are fewer than k heads) is a candidate, and tau is the k-th largest candidate.
    // (with few streams, PH = 2 or 4 lanes share the 64 comparisons of one head)
    const int ph = (4 * ngroups * 64 <= NT) ? 2 : (2 * ngroups * 64 <= NT) ? 1 : 0, PH = 1 << ph;
    for (int e0 = 0; e0 < ngroups * 64; e0 += NT >> ph) {
        const int e = e0 + (tid >> ph), part = tid & (PH - 1);
        const uint64_t mine = (e < ngroups * 64) ? hkeys[e] : kNoKey;
        int rank = 0;
        if (mine != kNoKey) {
            const uint64_t *group = hkeys + (e & ~63);
            rank = (ph == 2) ? head_rank_share<4>(group, part, mine)
                 : (ph == 1) ? head_rank_share<2>(group, part, mine) : head_rank_share<1>(group, part, mine);
        }
        rank = lanes_sum(rank, PH);
        if (mine != kNoKey && part == 0 && rank < k) surv[atomicAdd(&cnt_surv, 1u)] = mine;
    }
    __syncthreads();
    const int n_surv = (int)cnt_surv;
    __shared__ uint64_t head_bound;
    __shared__ uint32_t cnt_cand;
    if (tid == 0) { head_bound = kNoKey; cnt_cand = 0u; }
    __syncthreads();
    rank_all_pairs_wide(surv, n_surv, tid, NT, [&](int, uint64_t key, int rank) { if (rank == k - 1) head_bound = key; });
    __syncthreads();
    const uint64_t T = head_bound;                                       // kNoKey (smallest): fewer than k heads
    __syncthreads();                                                     // surv is reused below
    for (int e = tid; e < n; e += NT) {
        const uint64_t mine = keys[e];
        if (mine != kNoKey && mine >= T) surv[atomicAdd(&cnt_cand, 1u)] = mine;
    }
    __syncthreads();
    rank_all_pairs_wide(surv, (int)cnt_cand, tid, NT, [&](int, uint64_t key, int rank) { if (rank == k - 1) tau_key = key; });
    __syncthreads();
    const bool have_tau = tau_key != kNoKey;
    const float tau = have_tau ? key_value(tau_key) : kNegInf;
    // eps_v = kEpsSigmas |t - rounded t| (column scale of v's vocabulary tile) + eps_abs: the rounding errors dt_j of t
    // are taken as independent, so that column v's error sum_j dt_j B[j, v] has standard deviation |dt| rms(B[:, v]);
    // eps_abs covers the fp32 accumulation, the 4 packed bits and, in f16 mode, the weights the kernel flushed to
    // zero (magnitude below tiny_w, times the 1-norm of the contraction input).
    float dt_scale = 0.f, eps_abs;
    if (stat != nullptr) {
        dt_scale = kEpsSigmas * sqrtf(dt2_sh);
        eps_abs = fabsf(tau) * 1.2e-5f + tiny_w * X1 + 1e-30f;
    }
    else eps_abs = fabsf(tau) * 1.6e-5f + 1e-6f;
    // Scale of a tile's columns: the rms of all of B (tens of thousands of sampled entries: no noise to speak of), or
    // the tile's own column scale where that is larger, i.e. where the tile holds columns well above the average (the
    // kernel that samples B has already taken the overshoot of "the largest of 256 estimates" off, or, where one column
    // stands out of its tile, left that column's estimate as it is).
    const auto tile_scale = [&](float tile_max) { return fmaxf(b_rms, tile_max); };
    const auto eps_of_tile = [&](int vt) {
        return (stat != nullptr) ? dt_scale * tile_scale(ts_cached ? ts[min(vt, n_vt - 1)] : ts_max) + eps_abs : eps_abs;
    };
    const float eps = dt_scale * tile_scale(ts_max) + eps_abs;      // the bound of the vocabulary tile with the largest columns
    const float theta = have_tau ? tau - 2.f * eps : kNegInf;
    // Overflow of the 16-bit input; or a rounding bound so wide that the streams' sum of exponentials (whose terms
    // are off by up to a factor e^eps) no longer gives the log-sum-exp to the reported precision, and the
    // correction by the re-evaluated terms could itself overflow.
    bool exhaustive = !(eps < kExhaustiveEps) || !(lse == lse) || !(fabsf(lse) < 1e30f);

    // ---- sampling: the streams whose best z + g could be the row's largest once the logits are exact
    if (so.on) {
        uint64_t best = kNoKey;
        float w2m = kNegInf;
        for (int sidx = tid; sidx < nsr; sidx += NT) {
            const float *sp = rec + (size_t)sidx * rec_stride + REC;
            const float w1 = sp[0], w3 = sp[4];
            if (w1 > kNoValue) best = u64_max(best, make_key(w1 * unit, (uint32_t)__float_as_int(sp[1])));
            if (w3 > kNoValue) w2m = fmaxf(w2m, w3 * unit);        // bounds what the stream saw beyond its two recorded ids
        }
        float unused;
        const uint64_t top = block_best(best, 0.f, unused);
        w2m = wave_max(w2m);
        if (tid == 0) smp_cnt = 0u;
        if (lane == 0) smp_w2[wave] = w2m;
        __syncthreads();
        float W2 = smp_w2[0];
#pragma unroll
        for (int w = 1; w < NWAVES; ++w) W2 = fmaxf(W2, smp_w2[w]);
        const float thr_s = key_value(top) - 2.f * eps;
        for (int sidx = tid; sidx < nsr; sidx += NT) {
            const float *sp = rec + (size_t)sidx * rec_stride + REC;
#pragma unroll
            for (int q = 0; q < 2; ++q) {                    // the stream's best and second best
                const int idq = __float_as_int(sp[2 * q + 1]);
                if (sp[2 * q] > kNoValue && sp[2 * q] * unit >= thr_s && (unsigned)idq < (unsigned)V) {
                    const uint32_t slot = atomicAdd(&smp_cnt, 1u);
                    if (slot < (uint32_t)kSampleCap) smp_id[slot] = idq;
                }
            }
        }
        __syncthreads();
        // a stream's third best within the bound (its id is not recorded), too many contenders, or none: whole row exact
        if (top == kNoKey || smp_cnt == 0u || smp_cnt > (uint32_t)kSampleCap || W2 >= thr_s) exhaustive = true;
    }

    // ---- collect
    auto push = [&](int id, float val, int need, float e_item) {
        const uint32_t slot = atomicAdd(&cnt_work, 1u);
        if (slot < (uint32_t)kWorkCap) { w_id[slot] = id; w_val[slot] = val; w_need[slot] = need; w_apx[slot] = 0.f; w_eps[slot] = e_item; }
        if (need) atomicAdd(&cnt_hidden, 1u);
        return slot;
    };
    // column of member i of a group: MFMA tile (tag & 7) of vocabulary tile (tag >> 3) covers 32 adjacent columns
    auto id_of = [&](int tag, int i, int half) {
        const int pos = 8 * (i >> 2) + 4 * half + (i & 3);
        return (tag >> 3) * 256 + 32 * (tag & 7) + pos;
    };
    const bool wide = eps > kWideEps;
    // computed logits from here on belong to tokens of probability >= kMassCut / eps
    const float v_mass = wide ? lse + __builtin_amdgcn_logf(kMassCut / eps) * kLn2 : __builtin_huge_valf();
    if (!exhaustive) {
        for (int sidx = tid; sidx < nsr; sidx += NT) {
            float r[REC];
            load_rec(sidx, r);
            int listed[L];
#pragma unroll
            for (int l = 0; l < L; ++l) {
                const float x = r[3 + 3 * l], y = r[4 + 3 * l];
                const int rawtag = __float_as_int(r[5 + 3 * l]);
                // the tag's lowest bit names the half-wavefront that held the group
                const int half = rawtag & 1, tag = rawtag >> 1;
                listed[l] = (x > kNoValue) ? rawtag : -1;
                if (!(x > kNoValue) || !(mask4(x) * unit >= fminf(theta, v_mass))) continue;
                const int imax = (int)(__float_as_uint(x) & 15u);
                const int id_max = id_of(tag, imax, half);
                if ((unsigned)id_max >= (unsigned)V) continue;      // cannot come from the head kernel: keeps the gathers in bounds whatever the records hold
                // its own tile's bound decides (theta was the bound of the widest tile)
                const float e_item = eps_of_tile(tag >> 3);
                // a candidate for the top-k, or at least a probable token whose exact value the log-sum-exp needs
                const float xv = mask4(x) * unit, yv = mask4(y) * unit;
                const bool cand = xv >= tau - eps - e_item;
                const bool mass_on = e_item > kExactWinnersEps;      // (such a token is re-evaluated: see the need pass)
                if (!cand && !(mass_on && xv >= v_mass)) continue;
                const uint32_t slot = push(id_max, xv, 0, e_item);
                if (cand && keys[sidx * L + l] == tau_key) tau_slot = (int)slot;      // one writer: keys are unique
                // the group's other members, when its second largest value is a candidate or a probable token itself
                if (y > kNoValue && ((cand && yv >= tau - eps - e_item) || (mass_on && yv >= v_mass))) {
                    for (int i = 0; i < 16; ++i) {
                        const int id = id_of(tag, i, half);
                        if (i != imax && (unsigned)id < (unsigned)V) push(id, 0.f, 1, e_item);
                    }
                }
            }
            const float U = r[2];
            if (U > kNoValue && mask4(U) * unit >= fminf(theta, v_mass)) {
                // every unlisted group of the stream is a candidate: the whole block lists their members below
                const uint32_t c = atomicAdd(&cnt_crowd, 1u);
                if (c < (uint32_t)kCrowdCap) crowd[c] = sidx;
            }
        }
        __syncthreads();
        // Column block col covers vocabulary tiles col, col + gw, ...; of a tile's 8 MFMA tiles a column half has four,
        // of an MFMA tile's 32 columns a half-wavefront 16.  A record stands for one lane stream (column half,
        // half-wavefront), for a column half, or for the whole block (see the head kernel): 256, 512 or 1024 columns
        // at four tiles per block, listed by the whole merge block (one thread alone took 0.3 ms for 1000 columns).
        const int n_crowd = (int)cnt_crowd;
        if (n_crowd > kCrowdCap) exhaustive = true;           // (the same for every thread)
        for (int c = 0; c < n_crowd && !exhaustive; ++c) {
            const int sidx = crowd[c];
            float r[REC];
            load_rec(sidx, r);
            int listed[L];
#pragma unroll
            for (int l = 0; l < L; ++l) listed[l] = (r[3 + 3 * l] > kNoValue) ? __float_as_int(r[5 + 3 * l]) : -1;
            const int spb = nsr / gw, col = sidx / spb, sub = sidx % spb;       // 4, 2 or 1 records per column block
            const int n_tiles = (n_vt - col + gw - 1) / gw;
            const int per_tile = 256 / spb, sh = (spb == 4) ? 6 : (spb == 2) ? 7 : 8;
            for (int e = tid; e < n_tiles * per_tile; e += NT) {
                const int vt = col + (e >> sh) * gw, m = e & (per_tile - 1);
                // spb 4: (column half, half-wavefront) = sub; 2: column half = sub, both half-wavefronts; 1: everything
                const int half = (spb == 4) ? (sub & 1) : ((m >> 4) & 1);
                const int j = (spb == 4) ? 4 * (sub >> 1) + ((m >> 4) & 3) : (spb == 2) ? 4 * sub + ((m >> 5) & 3) : ((m >> 5) & 7);
                const int rawtag = (vt * 8 + j) * 2 + half;
                bool is_listed = false;
#pragma unroll
                for (int l = 0; l < L; ++l) is_listed |= (listed[l] == rawtag);
                const int id = id_of(rawtag >> 1, e & 15, rawtag & 1);
                const bool take = !is_listed && id < V;           // (a wavefront's 64 values of e are all inside the range or all outside)
                int n_taken;
                const uint32_t slot = wave_slots(&cnt_work, take, n_taken);
                if (take && slot < (uint32_t)kWorkCap) { w_id[slot] = id; w_val[slot] = 0.f; w_need[slot] = 1; w_apx[slot] = 0.f; w_eps[slot] = eps_of_tile(vt); }
                if (lane == 0 && n_taken != 0) atomicAdd(&cnt_hidden, (uint32_t)n_taken);
            }
        }
    }
    __syncthreads();
    int n_work = (int)cnt_work;
    if (n_work > kWorkCap || n_work < k) exhaustive = true;

    if (!exhaustive) {
        // ---- which listed maxima need the exact value
        const bool any_hidden = cnt_hidden != 0u;
        // (PN lanes share the scan of one item: the collected set is a dozen items, the block 512 threads)
        const int pn = lanes_per_item_log2(n_work, NT), PN = 1 << pn;
        for (int c0 = 0; c0 < n_work; c0 += NT >> pn) {
            const int c = c0 + (tid >> pn), part = tid & (PN - 1);
            const bool open = c < n_work && w_need[c] == 0;
            int need = 0;
            if (open) {
                // a computed value may be off by its eps_v: beyond kExactWinnersEps a log-probability takes the exact value
                const float mine = w_val[c], e_mine = w_eps[c];
                if (any_hidden || e_mine > kExactWinnersEps) need = 1;
                else {
#pragma unroll 4
                    for (int q = part; q < n_work; q += PN)
                        need |= (q != c && fabsf(w_val[q] - mine) <= w_eps[q] + e_mine) ? 1 : 0;
                }
            }
            need = lanes_sum(need, PN);
            if (open && part == 0 && need) w_need[c] = 2;    // 2: decided in this pass (w_val still the computed value)
        }
        __syncthreads();
        if (wide) {
            // probability mass of the listed logits that get their exact value (fixed order: lanes, then the DPP tree)
            if (wave == 0) {
                float pm = 0.f;
                for (int c = lane; c < n_work; c += 64)
                    if (w_need[c] == 2) pm += __builtin_amdgcn_exp2f((w_val[c] - lse) * kLog2e);
                pm = wave_sum(pm);
                if (lane == 0) mass_eval_sh = pm;
            }
            __syncthreads();
            const float rest = 1.f - fminf(mass_eval_sh, 1.f);
            if (rest * eps > kLseGuard) exhaustive = true;
            // The part of the rounding error that lies along t itself, (t - rounded t) . t / |t|^2 =: rho, scales every
            // logit by 1 - rho: errors of one sign, proportional to the logit, which do not average out of the sum of
            // exponentials.  rho is known exactly; with a long contraction it is a few 1e-5, with a rank of a few dozen
            // it reaches 1e-3 and more.  Where it could move the log-sum-exp of the tokens left over, the row is redone.
            if (stat != nullptr && rest * fabsf(tdt_sh / X2) * fabsf(Mx * kLn2) > kCommonModeTol) exhaustive = true;
        }
    }
    if (!exhaustive) {
        // list the items to evaluate (any order: every result goes back to its own slot)
        constexpr int PER = (kWorkCap + NT - 1) / NT;       // fixed trip count: the array stays in registers
        int my_need[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = tid + i * NT;
            my_need[i] = (c < n_work && w_need[c]) ? (c | (w_need[c] == 2 ? kListedBit : 0)) : -1;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            int n_taken;
            const uint32_t slot = wave_slots(&cnt_need, my_need[i] >= 0, n_taken);
            if (my_need[i] >= 0) w_need[slot] = my_need[i];
        }
        __syncthreads();
        // No item to evaluate: the k-th listed maximum is evaluated all the same, so that every row checks the bound
        // it relied on against one exact value at least (take_exact).
        if (cnt_need == 0u && tau_slot >= 0 && tau_slot < n_work && stat != nullptr) {
            __syncthreads();
            if (tid == 0) { w_need[0] = tau_slot | kListedBit; cnt_need = 1u; }
            __syncthreads();
        }
        if (so.on) {                                         // the sampling contenders join the list of columns to evaluate
            const uint32_t base_n = cnt_need;
            __syncthreads();
            if (base_n + smp_cnt <= (uint32_t)kWorkCap) {
                if (tid < (int)smp_cnt) w_need[base_n + tid] = tid | kSampleBit;
                if (tid == 0) cnt_need = base_n + smp_cnt;
            } else if (tid == 0) eps_violated = 1;          // no room (thousands of near-ties): exhaustive pass
            __syncthreads();
        }
        // (a row with unlisted members on a bf16 operand stays here: their recomputed 16-bit logits come with the gathers)
        const bool park_ok = !(operand16 == 1 && cnt_hidden != 0u);
        if (park && park_ok && cnt_need != 0u && cnt_need <= (uint32_t)kDeferNeed && n_work <= kDeferWork) {
            // park the row: collected set, list of columns, the streams' log-sum-exp
            const int n_need = (int)cnt_need;
            for (int c = tid; c < n_work; c += NT) { park_id[c] = w_id[c]; park_val[c] = w_val[c]; park_eps[c] = w_eps[c]; }
            for (int c = tid; c < n_need; c += NT) park_need[c] = w_need[c];
            if (tid == 0) {
                park[0] = n_need; park[1] = n_work;
                park[2] = __float_as_int(S); park[3] = __float_as_int(Mx); park[4] = __float_as_int(lse);
            }
            return;
        }
        // exact fp32 logits, 16 columns at a time: a lane owns (column lane % 16, row phase lane / 16), the
        // four wavefronts interleave rows, so one load instruction touches 4 rows of M x 16 columns and the
        // whole block has 16 rows in flight per step; partial sums are combined in a fixed order
        const int n_need = (int)cnt_need;
        __shared__ float red_ex[NWAVES][16], red_ex16[NWAVES][16];
        const bool with16 = operand16 != 0;
        // Column-major copy: a column is K adjacent elements.  kGatherRound columns per round; wavefront w takes columns w,
        // w + NWAVES, ... of the round, a lane 8 adjacent elements of the column per step (K = 512: one 16-byte load
        // per lane and column, all of a wavefront's columns in flight together); lanes in order inside the DPP tree.
        // (a lane's 8 adjacent elements of the contraction input are 32 bytes from its neighbour's: reads with shared-memory
        // bank conflicts, so they are done once per step, not once per column, and once for all rounds when the
        // contraction fits one step)
        float xv[8], xv16[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { xv[e] = 0.f; xv16[e] = 0.f; }
        const bool one_step = K <= 512;
        if (Mt != nullptr && one_step && lane * 8 < K) {
#pragma unroll
            for (int e = 0; e < 8; e += 2) {                   // (xrow is 8-byte aligned)
                const float2 x2 = *reinterpret_cast<const float2 *>(xrow + lane * 8 + e);
                const float2 y2 = *reinterpret_cast<const float2 *>(xrow16 + lane * 8 + e);
                xv[e] = x2.x; xv[e + 1] = x2.y; xv16[e] = y2.x; xv16[e + 1] = y2.y;
            }
        }
        for (int g0 = 0; Mt != nullptr && g0 < n_need; g0 += kGatherRound) {
            constexpr int CPW = kGatherRound / NWAVES;
            __shared__ float z_col[kGatherRound], z16_col[kGatherRound];
            const int n_here = min(kGatherRound, n_need - g0);
            const int entry = w_need[g0 + min(lane, n_here - 1)];
            // (the second sum only in a round that holds a column without a recorded value: every wavefront sees the same
            // entries, so all of them decide alike)
            const bool round16 = with16 && __ballot(lane < n_here && (entry & (kListedBit | kSampleBit)) == 0) != 0ull;
            float zc[CPW], zc16[CPW];
            const uint16_t *col[CPW];
#pragma unroll
            for (int q = 0; q < CPW; ++q) {
                zc[q] = 0.f; zc16[q] = 0.f;
                const int ent = w_need[g0 + min(wave + q * NWAVES, n_here - 1)];
                const int it = ent & (kSampleBit - 1);
                col[q] = Mt + (size_t)((ent & kSampleBit) ? smp_id[it] : w_id[it]) * K;
            }
            for (int j = lane * 8; j < K; j += 512) {        // K is a multiple of 8
                uint4 wq[CPW];
#pragma unroll
                for (int q = 0; q < CPW; ++q)
                    if (wave + q * NWAVES < n_here) wq[q] = *reinterpret_cast<const uint4 *>(col[q] + j);
                if (!one_step) {
#pragma unroll
                    for (int e = 0; e < 8; e += 2) {
                        const float2 x2 = *reinterpret_cast<const float2 *>(xrow + j + e);
                        const float2 y2 = *reinterpret_cast<const float2 *>(xrow16 + j + e);
                        xv[e] = x2.x; xv[e + 1] = x2.y; xv16[e] = y2.x; xv16[e + 1] = y2.y;
                    }
                }
#pragma unroll
                for (int q = 0; q < CPW; ++q) {
                    if (wave + q * NWAVES >= n_here) continue;
                    const float f[8] = {bf16_lo(wq[q].x), bf16_hi(wq[q].x), bf16_lo(wq[q].y), bf16_hi(wq[q].y),
                                        bf16_lo(wq[q].z), bf16_hi(wq[q].z), bf16_lo(wq[q].w), bf16_hi(wq[q].w)};
#pragma unroll
                    for (int e = 0; e < 8; ++e) zc[q] = fmaf(xv[e], f[e], zc[q]);
                    if (round16) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) zc16[q] = fmaf(xv16[e], f[e], zc16[q]);
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < CPW; ++q) {
                if (wave + q * NWAVES >= n_here) continue;     // (the same for the whole wavefront)
                const float z = wave_sum(zc[q]), z16 = round16 ? wave_sum(zc16[q]) : 0.f;
                if (lane == 0) { z_col[wave + q * NWAVES] = z; z16_col[wave + q * NWAVES] = z16; }
            }
            __syncthreads();
            if (tid < n_here) {                                 // tid < 64: `entry` is this column's
                const float z = z_col[tid];
                if (entry & kSampleBit) smp_z[entry & (kSampleBit - 1)] = z;
                else take_exact(entry, z, round16 ? z16_col[tid] : z, Mx);
            }
            __syncthreads();
        }
        for (int g0 = 0; Mt == nullptr && g0 < n_need; g0 += 16) {
            const int u = lane & 15, jsub = lane >> 4;
            const int entry = w_need[min(g0 + u, n_need - 1)];
            const int item = entry & (kSampleBit - 1);
            const int id = (entry & kSampleBit) ? smp_id[item] : w_id[item];
            // (the second sum only in a batch that holds a column without a recorded value: every wavefront sees the same
            // 16 entries, so all of them decide alike)
            const bool batch16 = with16 && __ballot((entry & (kListedBit | kSampleBit)) == 0) != 0ull;
            float acc = 0.f, acc16 = 0.f;
            // rows wave * 4 + jsub + 4 NWAVES e, e = 0, 1, ...: batches of 16 independent loads per lane (K = 512: one round trip)
            const uint16_t *mcol = M + id;
            constexpr int RSTEP = 4 * NWAVES, NLD = 16;
            for (int j0 = wave * 4 + jsub; j0 < K; j0 += NLD * RSTEP) {
                uint16_t w[NLD];
#pragma unroll
                for (int e = 0; e < NLD; ++e) w[e] = mcol[(size_t)min(j0 + e * RSTEP, K - 1) * V];
#pragma unroll
                for (int e = 0; e < NLD; ++e) {
                    const int j = j0 + e * RSTEP;
                    acc = fmaf(j < K ? xrow[j] : 0.f, bf16_to_float(w[e]), acc);
                }
                if (batch16) {                              // (a pass of its own: the common path stays as it was)
#pragma unroll
                    for (int e = 0; e < NLD; ++e) {
                        const int j = j0 + e * RSTEP;
                        acc16 = fmaf(j < K ? xrow16[j] : 0.f, bf16_to_float(w[e]), acc16);
                    }
                }
            }
            uint32_t a, b;
            swap_pair<16>(__float_as_uint(acc), a, b);
            acc = __uint_as_float(a) + __uint_as_float(b);
            swap_pair<32>(__float_as_uint(acc), a, b);
            acc = __uint_as_float(a) + __uint_as_float(b);
            if (batch16) {
                swap_pair<16>(__float_as_uint(acc16), a, b);
                acc16 = __uint_as_float(a) + __uint_as_float(b);
                swap_pair<32>(__float_as_uint(acc16), a, b);
                acc16 = __uint_as_float(a) + __uint_as_float(b);
            }
            if (lane < 16) { red_ex[wave][lane] = acc; red_ex16[wave][lane] = acc16; }
            __syncthreads();
            if (tid < 16 && g0 + tid < n_need) {
                float z = red_ex[0][tid], z16 = red_ex16[0][tid];
#pragma unroll
                for (int w = 1; w < NWAVES; ++w) { z += red_ex[w][tid]; z16 += red_ex16[w][tid]; }
                if (entry & kSampleBit) smp_z[item] = z;
                else take_exact(entry, z, batch16 ? z16 : z, Mx);     // tid < 16: u == tid, so `entry` is this column's
            }
            __syncthreads();
        }
        __syncthreads();
        if (!eps_violated) {
            uint64_t skey = kNoKey;
            float sz = 0.f;
            if (so.on) {                                     // the draw: the contenders' exact logits plus their noise
                uint64_t mine = kNoKey;
                float zm = 0.f;
                if (tid < (int)smp_cnt) {
                    zm = smp_z[tid];
                    mine = make_key(zm + gumbel_base2(gk, (uint32_t)smp_id[tid]) * kLn2, (uint32_t)smp_id[tid]);
                }
                skey = block_best(mine, zm, sz);
            }
            finish(n_work, S, Mx, lse);
            if (so.on) {
                __syncthreads();
                write_sample(skey, sz, lse_out_sh);
            }
            return;
        }
    }
    exhaustive_pass();
}


// Partial exact logits of the parked rows: block (ks, row) covers slice ks of the contraction for every column on
// the row's list, 16 columns at a time (lane = column lane % 16, row phase lane / 16; the four wavefronts interleave
// rows), and leaves part[ks][i]; the resumed merge adds the slices in order.  Rows that are not parked cost a block
// one load.
__global__ __launch_bounds__(256) void exact_cols_kernel(
    int *__restrict__ defer, const void *__restrict__ xexact, int x_is_bf16, int ldx,
    const uint16_t *__restrict__ M, int K, int V)
{
    const int ks = blockIdx.x, row = blockIdx.y;
    const ParkedRow pk = parked_row(defer, row);
    const int n_need = pk.hdr[0];
    if (n_need == 0) return;
    RowCtx ctx;
    ctx.x = x_is_bf16 ? static_cast<const void *>(static_cast<const uint16_t *>(xexact) + (size_t)row * ldx)
                      : static_cast<const void *>(static_cast<const float *>(xexact) + (size_t)row * ldx);
    ctx.x_is_bf16 = x_is_bf16; ctx.M = M; ctx.K = K; ctx.V = V;
    const int per = ((K + kDeferSlices - 1) / kDeferSlices + 15) & ~15;
    const int kb = min(K, ks * per), ke = min(K, kb + per);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int u = lane & 15, jsub = lane >> 4;
    __shared__ float red[4][16];
    for (int g0 = 0; g0 < n_need; g0 += 16) {
        const int entry = pk.need[min(g0 + u, n_need - 1)];
        const uint16_t *mcol = M + pk.id[entry & (kListedBit - 1)];
        float acc = 0.f;
        constexpr int NB = 16, RSTEP = 16;                 // 16 loads in flight per lane, 16 rows per load instruction of the block
        for (int j0 = kb + wave * 4 + jsub; j0 < ke; j0 += NB * RSTEP) {
            uint16_t w[NB];
#pragma unroll
            for (int e = 0; e < NB; ++e) w[e] = mcol[(size_t)min(j0 + e * RSTEP, ke - 1) * V];
#pragma unroll
            for (int e = 0; e < NB; ++e) {
                const int j = j0 + e * RSTEP;
                acc = fmaf(j < ke ? x_at(ctx, j) : 0.f, bf16_to_float(w[e]), acc);
            }
        }
        uint32_t a, b;
        swap_pair<16>(__float_as_uint(acc), a, b);
        acc = __uint_as_float(a) + __uint_as_float(b);
        swap_pair<32>(__float_as_uint(acc), a, b);
        acc = __uint_as_float(a) + __uint_as_float(b);
        if (lane < 16) red[wave][lane] = acc;
        __syncthreads();
        if (tid < 16 && g0 + tid < n_need)
            pk.part[ks * kDeferNeed + g0 + tid] = ((red[0][tid] + red[1][tid]) + red[2][tid]) + red[3][tid];
        __syncthreads();
    }
}

size_t merge_defer_bytes(int rows) { return sizeof(int) * kDeferRowInts * (size_t)rows; }

size_t merge_streams_lds_bytes(int nsr, int k, int n_vt) {
    const size_t n = (size_t)nsr * kStreamList;
    const size_t ngroups = ((size_t)nsr + 63) / 64;
    const size_t n_front = n + ngroups * 64 + (ngroups > 3 ? ngroups : 3) * k;
    return sizeof(uint64_t) * (n_front > (size_t)kExhaustCap ? n_front : (size_t)kExhaustCap) + 20u * kWorkCap
           + sizeof(float) * (((size_t)(n_vt < kTsCap ? n_vt : kTsCap) + 3) & ~(size_t)3);
}

hipError_t launch_merge_streams(const float *part, int rows, int nsr, int gw, int n_vt,
                                const void *xexact, bool x_is_bf16, int ldx, int operand16,
                                const uint16_t *M, int K, int V, const uint16_t *Mt,
                                const float2 *stat, int n_stat, int rows_pad, const float2 *tilescale, int k,
                                float unit, float tiny_w, int32_t *out_ids, float *out_logprobs, const int32_t *id_map,
                                void *defer_buf, const SampleOut &so, int row_base, hipStream_t st)
{
    const size_t lds = merge_streams_lds_bytes(nsr, k, n_vt) + 2 * sizeof(float) * (size_t)K;   // + the row's contraction input, exact and as rounded
    static LdsLimit lds_limit;
    hipError_t e = lds_limit.raise(reinterpret_cast<const void *>(merge_streams_kernel), (int)lds);
    if (e != hipSuccess) return e;
    // sampling calls evaluate in place; with a column-major copy an exact logit is one short read: nothing to park
    int *defer = (so.on || Mt != nullptr) ? nullptr : static_cast<int *>(defer_buf);
    const int rec_stride = so.on ? kStreamRecSample : kStreamRec;
    merge_streams_kernel<<<rows, kMergeThreads, lds, st>>>(part, rec_stride, nsr, gw, n_vt, xexact, x_is_bf16 ? 1 : 0, ldx,
                                                           operand16, M, K, V, Mt, stat, n_stat, rows_pad, tilescale, k, unit, tiny_w, out_ids, out_logprobs, id_map,
                                                           defer, 0, so, row_base);
    if ((e = hipGetLastError()) != hipSuccess || !defer) return e;
    // parked rows: their exact columns on many CUs, then the rest of their merge
    exact_cols_kernel<<<dim3(kDeferSlices, rows), 256, 0, st>>>(defer, xexact, x_is_bf16 ? 1 : 0, ldx, M, K, V);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    merge_streams_kernel<<<rows, kMergeThreads, lds, st>>>(part, rec_stride, nsr, gw, n_vt, xexact, x_is_bf16 ? 1 : 0, ldx,
                                                           operand16, M, K, V, Mt, stat, n_stat, rows_pad, tilescale, k, unit, tiny_w, out_ids, out_logprobs, id_map,
                                                           defer, 1, so, row_base);
    return hipGetLastError();
}

}  // namespace slimspec

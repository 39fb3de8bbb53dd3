/*
 * CPU fp64 checker for the drafter LM-head with top-k / log-probability outputs.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against; nothing in the product path may call it, and
 * it shares no code, header, table or helper with the HIP sources.
 *
 * What it computes (paper section 4.1, "LM-head architecture"):
 *   full head      z = W_full h                      (first display of 4.1)
 *   low-rank head  z = W_up (W_down h)               (second display of 4.1)
 * in row-vector form with the transposed matrices the library takes:
 *   h [rows,d],  A = W_down^T [d,r],  B = W_up^T [r,V],  W = W_full^T [d,V],
 *   t = h A,  z = t B   (or z = h W),   no bias, temperature 1.
 * The reduction of each logit row to the k most likely tokens and their natural
 * log-probabilities is the plain definition of log-softmax (the softmax over the
 * whole vocabulary of section 3.2) followed by a full sort:
 *   lse = m + ln sum_v exp(z_v - m),  m = max_v z_v      (two passes, fp64)
 *   order tokens by z descending, equal z by smaller id first; emit the first k
 *   ids and z - lse.
 *
 * Every input is widened to fp64 exactly (bf16 bits -> fp32 -> fp64); the
 * intermediate t is never rounded.  No blocking, fusion or reordering beyond the
 * loop nests below.  OpenMP only distributes independent rows (or, for a single
 * row, independent vocabulary entries) over threads.
 *
 * Further down: the heads around it that the paper compares with or proposes
 * (truncated vocabulary, router-then-exact, position-specific down-projections)
 * and Gumbel-max sampling at temperature 1, each as its plain definition.
 *
 * Pins (tests/test_oracle_*.py): hand-worked example, closed forms (h = 0,
 * one hot column), brute force in pure Python on tiny inputs, (hA)B = h(AB),
 * rank(AB) <= r, sum exp(logprob) = 1, shift invariance, permutation
 * equivariance, k = 1 = argmax, k = V = sorted log-softmax, numpy/scipy
 * cross-checks.  Numerical values on random inputs are pinned only through
 * those library cross-checks (the paper prints no worked logits): beyond the
 * pins above, parity on random inputs is "parity unpinned" by any paper value.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double widen_bf16(uint16_t bits)
{
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* t[i][j] = sum_c h[i][c] * A[c][j]          (the inner product W_down h of 4.1) */
int oracle_down_projection(const uint16_t *h, const uint16_t *A,
                           int rows, int d, int r, double *t)
{
    if (!h || !A || !t || rows <= 0 || d <= 0 || r <= 0) return -1;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < rows; ++i) {
        double *ti = t + (size_t)i * r;
        for (int j = 0; j < r; ++j) ti[j] = 0.0;
        for (int c = 0; c < d; ++c) {
            double hic = widen_bf16(h[(size_t)i * d + c]);
            const uint16_t *Ac = A + (size_t)c * r;
            for (int j = 0; j < r; ++j) ti[j] += hic * widen_bf16(Ac[j]);
        }
    }
    return 0;
}

/* z[v] = sum_j x[j] * M[j][v] for one row; x is fp64 [K], M is [K,V] bf16 or fp32.
 * v is the inner loop so that each M row is read contiguously. */
static void logits_one_row(const double *x, const void *M, int m_is_f32,
                           int K, int V, double *z)
{
    for (int v = 0; v < V; ++v) z[v] = 0.0;
    for (int j = 0; j < K; ++j) {
        double xj = x[j];
        if (m_is_f32) {
            const float *Mj = (const float *)M + (size_t)j * V;
            for (int v = 0; v < V; ++v) z[v] += xj * (double)Mj[v];
        } else {
            const uint16_t *Mj = (const uint16_t *)M + (size_t)j * V;
            for (int v = 0; v < V; ++v) z[v] += xj * widen_bf16(Mj[v]);
        }
    }
}

/* Same sum, restricted to vocabulary entries [v0,v1) (used when one row is split
 * over threads; each entry still accumulates j = 0..K-1 in order). */
static void logits_one_row_range(const double *x, const void *M, int m_is_f32,
                                 int K, int V, int v0, int v1, double *z)
{
    for (int v = v0; v < v1; ++v) z[v] = 0.0;
    for (int j = 0; j < K; ++j) {
        double xj = x[j];
        if (m_is_f32) {
            const float *Mj = (const float *)M + (size_t)j * V;
            for (int v = v0; v < v1; ++v) z[v] += xj * (double)Mj[v];
        } else {
            const uint16_t *Mj = (const uint16_t *)M + (size_t)j * V;
            for (int v = v0; v < v1; ++v) z[v] += xj * widen_bf16(Mj[v]);
        }
    }
}

typedef struct { double z; int32_t id; } scored;

static int by_logit_desc_then_id(const void *pa, const void *pb)
{
    const scored *a = (const scored *)pa, *b = (const scored *)pb;
    if (a->z > b->z) return -1;
    if (a->z < b->z) return 1;
    return (a->id > b->id) - (a->id < b->id);
}

/* Exact log-softmax + sort-based top-k of one fp64 logit row.
 * ids[k], logprobs[k] (float), lse (nullable), gap[k] (nullable):
 * gap[p] = z[ids[p]] - z[next in order] (the last one is the gap to rank k+1,
 * +inf when k == V). */
int oracle_log_softmax_topk(const double *z, int V, int k,
                            int32_t *ids, float *logprobs, double *lse_out, double *gap)
{
    if (!z || !ids || !logprobs || V <= 0 || k < 1 || k > V) return -1;
    double m = z[0];
    for (int v = 1; v < V; ++v) if (z[v] > m) m = z[v];
    double s = 0.0;
    for (int v = 0; v < V; ++v) s += exp(z[v] - m);
    double lse = m + log(s);
    scored *order = (scored *)malloc((size_t)V * sizeof(scored));
    if (!order) return -2;
    for (int v = 0; v < V; ++v) { order[v].z = z[v]; order[v].id = v; }
    qsort(order, (size_t)V, sizeof(scored), by_logit_desc_then_id);   /* total order: no ties left */
    for (int p = 0; p < k; ++p) {
        ids[p] = order[p].id;
        logprobs[p] = (float)(order[p].z - lse);
        if (gap) gap[p] = (p + 1 < V) ? order[p].z - order[p + 1].z : INFINITY;
    }
    if (lse_out) *lse_out = lse;
    free(order);
    return 0;
}

/* Shared driver: x is the fp64 contraction input [rows,K] (t for the low-rank
 * head, widened h for the full head), M the [K,V] matrix. */
static int head_from_x(const double *x, const void *M, int m_is_f32,
                       int rows, int K, int V, int k,
                       int32_t *ids, float *logprobs, double *lse, double *gap, double *z_out)
{
    int status = 0;
    if (rows == 1) {
        double *z = z_out ? z_out : (double *)malloc((size_t)V * sizeof(double));
        if (!z) return -2;
#pragma omp parallel
        {
#ifdef _OPENMP
            int nt = omp_get_num_threads(), id = omp_get_thread_num();
#else
            int nt = 1, id = 0;
#endif
            int v0 = (int)((long long)V * id / nt), v1 = (int)((long long)V * (id + 1) / nt);
            logits_one_row_range(x, M, m_is_f32, K, V, v0, v1, z);
        }
        status = oracle_log_softmax_topk(z, V, k, ids, logprobs, lse, gap);
        if (!z_out) free(z);
        return status;
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < rows; ++i) {
        double *z = z_out ? z_out + (size_t)i * V : (double *)malloc((size_t)V * sizeof(double));
        if (!z) {
#pragma omp atomic write
            status = -2;
            continue;
        }
        logits_one_row(x + (size_t)i * K, M, m_is_f32, K, V, z);
        int st = oracle_log_softmax_topk(z, V, k, ids + (size_t)i * k, logprobs + (size_t)i * k,
                                         lse ? lse + i : NULL, gap ? gap + (size_t)i * k : NULL);
        if (st != 0) {
#pragma omp atomic write
            status = st;
        }
        if (!z_out) free(z);
    }
    return status;
}

/* Low-rank head: z = (h A) B, then log-softmax top-k.  Host pointers.
 * h [rows,d], A [d,r], B [r,V] are bf16 bit patterns.  Outputs ids/logprobs
 * [rows,k]; optional lse [rows], gap [rows,k], z_out [rows,V] (fp64 logits). */
int oracle_slimspec_head_topk(const uint16_t *h, const uint16_t *A, const uint16_t *B,
                              int rows, int d, int r, int V, int k,
                              int32_t *ids, float *logprobs,
                              double *lse, double *gap, double *z_out)
{
    if (!h || !A || !B || !ids || !logprobs) return -1;
    if (rows <= 0 || d <= 0 || r <= 0 || V <= 0 || k < 1 || k > V) return -1;
    double *t = (double *)malloc((size_t)rows * r * sizeof(double));
    if (!t) return -2;
    int st = oracle_down_projection(h, A, rows, d, r, t);
    if (st == 0) st = head_from_x(t, B, 0, rows, r, V, k, ids, logprobs, lse, gap, z_out);
    free(t);
    return st;
}

/* Full head: z = h W, then log-softmax top-k.  W [d,V] is bf16 bits
 * (w_is_f32 = 0) or fp32 (w_is_f32 = 1). */
int oracle_full_head_topk(const uint16_t *h, const void *W, int w_is_f32,
                          int rows, int d, int V, int k,
                          int32_t *ids, float *logprobs,
                          double *lse, double *gap, double *z_out)
{
    if (!h || !W || !ids || !logprobs) return -1;
    if (rows <= 0 || d <= 0 || V <= 0 || k < 1 || k > V) return -1;
    double *x = (double *)malloc((size_t)rows * d * sizeof(double));
    if (!x) return -2;
    for (size_t e = 0; e < (size_t)rows * d; ++e) x[e] = widen_bf16(h[e]);
    int st = head_from_x(x, W, w_is_f32, rows, d, V, k, ids, logprobs, lse, gap, z_out);
    free(x);
    return st;
}

/* Logits of chosen (row, id) pairs only, for checking ids a GPU run returned at
 * sizes where keeping every row's full logit vector is wasteful:
 * out[q] = z[row_idx[q]][col_idx[q]], each a plain fp64 dot product. */
int oracle_slimspec_logits_at(const uint16_t *h, const uint16_t *A, const uint16_t *B,
                              int rows, int d, int r, int V,
                              const int32_t *row_idx, const int32_t *col_idx, int n, double *out)
{
    if (!h || !A || !B || !row_idx || !col_idx || !out || n < 0) return -1;
    double *t = (double *)malloc((size_t)rows * r * sizeof(double));
    if (!t) return -2;
    int st = oracle_down_projection(h, A, rows, d, r, t);
    if (st == 0) {
        for (int q = 0; q < n; ++q) {
            int i = row_idx[q], v = col_idx[q];
            if (i < 0 || i >= rows || v < 0 || v >= V) { st = -1; break; }
            double acc = 0.0;
            for (int j = 0; j < r; ++j) acc += t[(size_t)i * r + j] * widen_bf16(B[(size_t)j * V + v]);
            out[q] = acc;
        }
    }
    free(t);
    return st;
}

int oracle_full_logits_at(const uint16_t *h, const void *W, int w_is_f32,
                          int rows, int d, int V,
                          const int32_t *row_idx, const int32_t *col_idx, int n, double *out)
{
    if (!h || !W || !row_idx || !col_idx || !out || n < 0) return -1;
    for (int q = 0; q < n; ++q) {
        int i = row_idx[q], v = col_idx[q];
        if (i < 0 || i >= rows || v < 0 || v >= V) return -1;
        double acc = 0.0;
        for (int c = 0; c < d; ++c) {
            double w = w_is_f32 ? (double)((const float *)W)[(size_t)c * V + v]
                                : widen_bf16(((const uint16_t *)W)[(size_t)c * V + v]);
            acc += widen_bf16(h[(size_t)i * d + c]) * w;
        }
        out[q] = acc;
    }
    return 0;
}

/* ======================================================================================
 * Heads around the low-rank head that the paper compares it with or proposes next.
 * Each is the plain definition, built from the functions above.
 * ====================================================================================== */

/* Truncated-vocabulary head (the static truncation of section 2, "Static vocabulary
 * truncation": a full head over a subset V_tr of the vocabulary plus a token-index map).
 * W_tr [d, V_tr] holds the kept columns; id_map[c] is the vocabulary id of column c.
 * The softmax runs over the kept columns only (the masked softmax of section 4.2 restricted
 * to V_tr); order: logit descending, equal logits by smaller COLUMN index; the emitted ids are
 * id_map[column]. */
int oracle_truncated_head_topk(const uint16_t *h, const void *W_tr, int w_is_f32, const int32_t *id_map,
                               int rows, int d, int V_tr, int k,
                               int32_t *ids, float *logprobs, double *lse, double *gap, double *z_out)
{
    if (!id_map) return -1;
    int st = oracle_full_head_topk(h, W_tr, w_is_f32, rows, d, V_tr, k, ids, logprobs, lse, gap, z_out);
    if (st != 0) return st;
    for (size_t e = 0; e < (size_t)rows * k; ++e) ids[e] = id_map[ids[e]];
    return 0;
}

/* Position-specific down-projections with a shared up-projection (the future direction named
 * in section 7): rows [pos_off[p], pos_off[p + 1]) use A_stack[p] ([d, r] each), every row the
 * same B.  pos_off has n_pos + 1 entries, pos_off[0] = 0, pos_off[n_pos] = rows. */
int oracle_slimspec_head_topk_positions(const uint16_t *h, const uint16_t *A_stack, const int32_t *pos_off, int n_pos,
                                        const uint16_t *B, int rows, int d, int r, int V, int k,
                                        int32_t *ids, float *logprobs, double *lse, double *gap, double *z_out)
{
    if (!h || !A_stack || !pos_off || !B || !ids || !logprobs || n_pos < 1) return -1;
    if (rows <= 0 || d <= 0 || r <= 0 || V <= 0 || k < 1 || k > V) return -1;
    if (pos_off[0] != 0 || pos_off[n_pos] != rows) return -1;
    double *t = (double *)malloc((size_t)rows * r * sizeof(double));
    if (!t) return -2;
    int st = 0;
    for (int p = 0; p < n_pos && st == 0; ++p) {
        int r0 = pos_off[p], n = pos_off[p + 1] - r0;
        if (n < 0) { st = -1; break; }
        if (n == 0) continue;
        st = oracle_down_projection(h + (size_t)r0 * d, A_stack + (size_t)p * d * r, n, d, r, t + (size_t)r0 * r);
    }
    if (st == 0) st = head_from_x(t, B, 0, rows, r, V, k, ids, logprobs, lse, gap, z_out);
    free(t);
    return st;
}

/* ---- sampling at temperature 1 (section 5.3 evaluates T = 1; section 3.2 counts the softmax
 * over the vocabulary among the overheads of stochastic decoding).
 * Gumbel-max: argmax_v (z_v + g_v) with independent standard Gumbel g_v is a draw from
 * softmax(z).  The noise is a pure function of (seed, row, id), so that any implementation
 * draws the same token:
 *     x = id * 0x9E3779B1 + row * 0x85EBCA77 + seed_lo                       (mod 2^32)
 *     x = mix(x);  x = x + seed_hi * 0xC2B2AE3D;  x = mix(x)
 *     mix(x): x ^= x >> 16; x *= 0x21F0AAAD; x ^= x >> 15; x *= 0x735A2D97; x ^= x >> 15
 *     n = x >> 9 (23 bits),  u = (2 n + 1) / 2^24 in (0, 1),  E = -ln(1 - u) ~ Exp(1),  g = -ln E. */
static uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x21F0AAADu; x ^= x >> 15; x *= 0x735A2D97u; x ^= x >> 15;
    return x;
}

double oracle_gumbel_noise(uint64_t seed, int32_t row, int32_t id)
{
    uint32_t x = (uint32_t)id * 0x9E3779B1u + (uint32_t)row * 0x85EBCA77u + (uint32_t)(seed & 0xffffffffu);
    x = mix32(x);
    x += (uint32_t)(seed >> 32) * 0xC2B2AE3Du;
    x = mix32(x);
    uint32_t n = x >> 9;
    double u = (2.0 * (double)n + 1.0) / 16777216.0;
    double E = -log1p(-u);
    return -log(E);
}

/* One draw from softmax(z) of one fp64 logit row: id of the largest z_v + g_v (equal sums: smaller id);
 * also that largest sum. */
int oracle_sample_row(const double *z, int V, uint64_t seed, int32_t row, int32_t *id_out, double *best_out)
{
    if (!z || !id_out || V <= 0) return -1;
    int best = 0;
    double wb = z[0] + oracle_gumbel_noise(seed, row, 0);
    for (int v = 1; v < V; ++v) {
        double w = z[v] + oracle_gumbel_noise(seed, row, v);
        if (w > wb) { wb = w; best = v; }
    }
    *id_out = best;
    if (best_out) *best_out = wb;
    return 0;
}

/* Low-rank head (full head when A == NULL: then M is W [d, V], bf16 or fp32) with the outputs of
 * stochastic decoding: top-k as before, lse [rows], and per row one sampled id with its log-probability.
 * z_out [rows, V] optional. */
int oracle_head_sample(const uint16_t *h, const uint16_t *A, const void *M, int m_is_f32,
                       int rows, int d, int r, int V, int k, uint64_t seed,
                       int32_t *ids, float *logprobs, double *lse,
                       int32_t *sample_ids, float *sample_logprobs, double *z_out)
{
    if (!h || !M || !ids || !logprobs || !lse || !sample_ids || !sample_logprobs) return -1;
    double *z = z_out ? z_out : (double *)malloc((size_t)rows * V * sizeof(double));
    if (!z) return -2;
    int st = A ? oracle_slimspec_head_topk(h, A, (const uint16_t *)M, rows, d, r, V, k, ids, logprobs, lse, NULL, z)
               : oracle_full_head_topk(h, M, m_is_f32, rows, d, V, k, ids, logprobs, lse, NULL, z);
    if (st == 0) {
#pragma omp parallel for schedule(dynamic, 1)
        for (int i = 0; i < rows; ++i) {
            int32_t id = 0;
            oracle_sample_row(z + (size_t)i * V, V, seed, i, &id, NULL);
            sample_ids[i] = id;
            sample_logprobs[i] = (float)(z[(size_t)i * V + id] - lse[i]);
        }
    }
    if (!z_out) free(z);
    return st;
}

/* Router-then-exact head (the dynamic vocabulary selection of section 2, "Dynamic vocabulary
 * selection": a low-rank router scores the whole vocabulary, the k_route best tokens are kept and
 * the full head is evaluated on those only).
 *   router logits  q = (h A) B                       over all V
 *   S = the k_route ids with the largest q (equal q: smaller id)
 *   y_v = h W[:, v] for v in S (exact full-head logits), softmax over S
 *   output: the k best of S by y (equal y: smaller id) with y_v - ln sum_{u in S} exp(y_u);
 *   route_ids [rows, k_route] optional: S in router order. */
int oracle_routed_head_topk(const uint16_t *h, const uint16_t *A, const uint16_t *B, const void *W, int w_is_f32,
                            int rows, int d, int r, int V, int k_route, int k,
                            int32_t *ids, float *logprobs, double *lse, int32_t *route_ids)
{
    if (!h || !A || !B || !W || !ids || !logprobs) return -1;
    if (k_route < 1 || k_route > V || k < 1 || k > k_route) return -1;
    int32_t *S = (int32_t *)malloc((size_t)rows * k_route * sizeof(int32_t));
    float *tmp = (float *)malloc((size_t)rows * k_route * sizeof(float));
    if (!S || !tmp) { free(S); free(tmp); return -2; }
    int st = oracle_slimspec_head_topk(h, A, B, rows, d, r, V, k_route, S, tmp, NULL, NULL, NULL);
    free(tmp);
    for (int i = 0; i < rows && st == 0; ++i) {
        const int32_t *Si = S + (size_t)i * k_route;
        double *y = (double *)malloc((size_t)k_route * sizeof(double));
        int32_t *ri = (int32_t *)malloc((size_t)k_route * sizeof(int32_t));
        if (!y || !ri) { free(y); free(ri); st = -2; break; }
        for (int q = 0; q < k_route; ++q) ri[q] = i;
        st = oracle_full_logits_at(h, W, w_is_f32, rows, d, V, ri, Si, k_route, y);
        if (st == 0) {
            /* order by (y desc, vocabulary id asc): sort pairs keyed by the vocabulary id */
            scored *order = (scored *)malloc((size_t)k_route * sizeof(scored));
            if (!order) st = -2;
            else {
                double m = y[0];
                for (int q = 1; q < k_route; ++q) if (y[q] > m) m = y[q];
                double s = 0.0;
                for (int q = 0; q < k_route; ++q) s += exp(y[q] - m);
                double l = m + log(s);
                for (int q = 0; q < k_route; ++q) { order[q].z = y[q]; order[q].id = Si[q]; }
                qsort(order, (size_t)k_route, sizeof(scored), by_logit_desc_then_id);
                for (int p = 0; p < k; ++p) {
                    ids[(size_t)i * k + p] = order[p].id;
                    logprobs[(size_t)i * k + p] = (float)(order[p].z - l);
                }
                if (lse) lse[i] = l;
                free(order);
            }
        }
        free(y); free(ri);
    }
    if (st == 0 && route_ids) memcpy(route_ids, S, (size_t)rows * k_route * sizeof(int32_t));
    free(S);
    return st;
}

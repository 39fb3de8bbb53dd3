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

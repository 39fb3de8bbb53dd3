/* Runs every entry point of the CPU checker on small seeded inputs; built with -fsanitize=address,undefined by
 * tests/test_sanitizers_cpu.py.  Prints a checksum so that the run is not optimised away. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_slimspec_head_topk(const uint16_t *, const uint16_t *, const uint16_t *, int, int, int, int, int,
                              int32_t *, float *, double *, double *, double *);
int oracle_full_head_topk(const uint16_t *, const void *, int, int, int, int, int, int32_t *, float *, double *, double *, double *);
int oracle_truncated_head_topk(const uint16_t *, const void *, int, const int32_t *, int, int, int, int,
                               int32_t *, float *, double *, double *, double *);
int oracle_slimspec_head_topk_positions(const uint16_t *, const uint16_t *, const int32_t *, int, const uint16_t *,
                                        int, int, int, int, int, int32_t *, float *, double *, double *, double *);
int oracle_head_sample(const uint16_t *, const uint16_t *, const void *, int, int, int, int, int, int, uint64_t,
                       int32_t *, float *, double *, int32_t *, float *, double *);
int oracle_routed_head_topk(const uint16_t *, const uint16_t *, const uint16_t *, const void *, int, int, int, int, int, int, int,
                            int32_t *, float *, double *, int32_t *);
int oracle_slimspec_logits_at(const uint16_t *, const uint16_t *, const uint16_t *, int, int, int, int,
                              const int32_t *, const int32_t *, int, double *);
int oracle_full_logits_at(const uint16_t *, const void *, int, int, int, int, const int32_t *, const int32_t *, int, double *);

static uint32_t rng_state = 12345u;
static uint16_t rnd_bf16(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    float f = ((float)(rng_state >> 8) / 8388608.0f - 1.0f) * 0.5f;
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}

int main(void)
{
    enum { ROWS = 5, D = 24, R = 8, V = 72, K = 6, KR = 12 };
    uint16_t *h = malloc(sizeof(uint16_t) * ROWS * D), *A = malloc(sizeof(uint16_t) * 2 * D * R);
    uint16_t *B = malloc(sizeof(uint16_t) * R * V), *W = malloc(sizeof(uint16_t) * D * V);
    float *Wf = malloc(sizeof(float) * D * V);
    for (int i = 0; i < ROWS * D; ++i) h[i] = rnd_bf16();
    for (int i = 0; i < 2 * D * R; ++i) A[i] = rnd_bf16();
    for (int i = 0; i < R * V; ++i) B[i] = rnd_bf16();
    for (int i = 0; i < D * V; ++i) { W[i] = rnd_bf16(); uint32_t u = (uint32_t)W[i] << 16; memcpy(&Wf[i], &u, 4); }
    int32_t ids[ROWS * KR], sid[ROWS], route[ROWS * KR], map[V], off[3] = {0, 2, ROWS}, ri[4] = {0, 1, 4, 4}, ci[4] = {0, 71, 3, 70};
    float lp[ROWS * KR], slp[ROWS];
    double lse[ROWS], gap[ROWS * KR], z[ROWS * V], at[4], sum = 0.0;
    for (int v = 0; v < V; ++v) map[v] = V - 1 - v;
    int st = 0;
    st |= oracle_slimspec_head_topk(h, A, B, ROWS, D, R, V, K, ids, lp, lse, gap, z);
    st |= oracle_full_head_topk(h, W, 0, ROWS, D, V, K, ids, lp, lse, gap, NULL);
    st |= oracle_full_head_topk(h, Wf, 1, 1, D, V, K, ids, lp, lse, NULL, z);
    st |= oracle_truncated_head_topk(h, W, 0, map, ROWS, D, V, K, ids, lp, lse, gap, NULL);
    st |= oracle_slimspec_head_topk_positions(h, A, off, 2, B, ROWS, D, R, V, K, ids, lp, lse, gap, z);
    st |= oracle_head_sample(h, A, B, 0, ROWS, D, R, V, K, 0x123456789abcdefULL, ids, lp, lse, sid, slp, NULL);
    st |= oracle_head_sample(h, NULL, Wf, 1, ROWS, D, 0, V, K, 7, ids, lp, lse, sid, slp, z);
    st |= oracle_routed_head_topk(h, A, B, W, 0, ROWS, D, R, V, KR, K, ids, lp, lse, route);
    st |= oracle_slimspec_logits_at(h, A, B, ROWS, D, R, V, ri, ci, 4, at);
    st |= oracle_full_logits_at(h, Wf, 1, ROWS, D, V, ri, ci, 4, at);
    for (int i = 0; i < ROWS * K; ++i) sum += lp[i] + ids[i];
    for (int i = 0; i < ROWS; ++i) sum += lse[i] + sid[i] + slp[i];
    printf("status %d checksum %.6f\n", st, sum + at[0] + at[3]);
    free(h); free(A); free(B); free(W); free(Wf);
    return st != 0;
}

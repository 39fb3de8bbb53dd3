/*
 * slimspec.h - C ABI of the MI355X (gfx950) drafter LM-head library.
 *
 * The operation (paper section 4.1, "LM-head architecture"): a speculative-decoding
 * drafter maps a hidden state h in R^d to logits over the whole target vocabulary,
 * either with the standard full head  z = W_full h  (W_full in R^{V x d}) or with the
 * low-rank head  z = W_up (W_down h)  (W_down in R^{r x d}, W_up in R^{V x r}, r < d,
 * typically d/8), which cuts the cost from O(Vd) to O(rd + Vr) while keeping all V
 * logits.  This library evaluates either head for a batch of rows and reduces every
 * logit row, in the same pass and without ever writing a rows x V tensor to memory, to
 * the k most likely token ids and their natural-log probabilities
 *     logprob_v = z_v - log sum_u exp(z_u)          (softmax over the full vocabulary,
 *                                                    section 3.2; temperature 1, no bias)
 *
 * Matrix layout (row-vector form; all row-major, all DEVICE memory):
 *     h [rows, d]  bf16     hidden states, one row per drafted position
 *     A [d, r]     bf16     A = W_down^T        t = h A
 *     B [r, V]     bf16     B = W_up^T          z = t B
 *     W [d, V]     bf16|f32 W = W_full^T        z = h W
 * bf16 values are raw 16-bit patterns (upper half of an IEEE fp32).
 *
 * Outputs (DEVICE memory, caller-owned):
 *     out_ids      [rows, k] int32   vocabulary index (column of B / W) of the p-th
 *                                    largest logit of the row, p = 0..k-1
 *     out_logprobs [rows, k] float   its log-probability
 * Order: descending logit; equal logits: smaller id first.  Logits are accumulated in
 * fp32 from exact bf16 products, and the log-probabilities are fp32 values: their
 * absolute accuracy is that of fp32 at the magnitude of the logits (about 1e-3 at logits
 * of a few thousand, 1e-1 at 1e5), whatever the path.  With few rows t = h A stays in fp32 throughout.  With
 * many rows the matrix cores take a 16-bit t (bf16, or f16 for k > 12) for the sum of
 * exponentials and for finding the candidates; every candidate whose rank or reported
 * value could depend on that rounding is then evaluated again from the fp32 t.
 *
 * Ownership / asynchrony: every pointer is caller-owned; the library allocates and
 * frees nothing, keeps no data between calls (the only state it holds is per host
 * thread: the text of the last HIP error and the two event handles of
 * slimspec_set_timing_events), and never synchronises.  All work is
 * enqueued on `stream` (a hipStream_t passed as void*, NULL = the default stream) and
 * the call returns immediately; outputs are valid once the stream has been
 * synchronised.  `workspace` is device scratch of at least
 * slimspec_workspace_bytes(...) bytes, 256-byte aligned; its contents are undefined
 * after the call and two calls that overlap in time must not share it.  `shape` is read
 * on the host during the call only.
 *
 * Errors: 0 on success, a negative slimspec_status otherwise.  Arguments are validated
 * on the host before any HIP call, and nothing is enqueued or written when validation
 * fails.  NaN/Inf inputs are not checked; results are then unspecified.
 */
#ifndef SLIMSPEC_H
#define SLIMSPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct slimspec_shape {
    int32_t rows;   /* number of hidden-state rows in the call, >= 1            */
    int32_t d;      /* drafter hidden size, multiple of 8                        */
    int32_t r;      /* rank of the low-rank head, multiple of 8 (ignored by full_head_topk) */
    int32_t V;      /* vocabulary size, multiple of 8                            */
} slimspec_shape;

typedef enum slimspec_dtype {
    SLIMSPEC_BF16 = 0,
    SLIMSPEC_F32 = 1
} slimspec_dtype;

typedef enum slimspec_status {
    SLIMSPEC_OK = 0,
    SLIMSPEC_INVALID_ARGUMENT = -1,    /* null pointer, non-positive size, k < 1, k > V, bad dtype   */
    SLIMSPEC_UNSUPPORTED = -2,         /* k > SLIMSPEC_KMAX, d/r/V not a multiple of 8, misaligned,  */
                                       /* V > 2^28, d * r >= 2^31                                    */
    SLIMSPEC_WORKSPACE_TOO_SMALL = -3,
    SLIMSPEC_HIP_ERROR = -4,           /* a launch failed; text via slimspec_last_hip_error()        */
    SLIMSPEC_SCRATCH_LIMIT = -5        /* slimspec_head_topk_static: the shape needs more scratch    */
                                       /* than SLIMSPEC_STATIC_SCRATCH_BYTES                         */
} slimspec_status;

#define SLIMSPEC_KMAX 64
#define SLIMSPEC_VERSION 1
#define SLIMSPEC_MAX_POSITIONS 16
#define SLIMSPEC_STATIC_SCRATCH_BYTES (64u << 20)   /* device scratch built into the library, per GPU */

/* Library version (SLIMSPEC_VERSION it was built with).  Host only, no HIP call. */
int slimspec_version(void);

/* Device scratch needed by slimspec_head_topk / full_head_topk for this shape and k
 * (the larger of the two).  Pure host function, no HIP call.  Returns 0 when the
 * shape or k is invalid or unsupported. */
size_t slimspec_workspace_bytes(const slimspec_shape *shape, int32_t k);

/* Low-rank head (second display of section 4.1): z = (h A) B, then per-row top-k ids
 * and log-probabilities.  h, A, B: device, bf16.  All device pointers 16-byte aligned. */
int slimspec_head_topk(const void *h, const void *A, const void *B,
                       const slimspec_shape *shape, int32_t k,
                       int32_t *out_ids, float *out_logprobs,
                       void *workspace, size_t workspace_bytes,
                       void *stream);

/* Column-major copy of a bf16 weight matrix: Mt[V, K] = transpose of M[K, V] (both device,
 * 16-byte aligned, K and V multiples of 8; Mt holds K * V elements and belongs to the
 * caller).  Made once per weight matrix, not per call.  Enqueued on `stream`. */
int slimspec_transpose_weights(const void *M, int32_t K, int32_t V, void *Mt, void *stream);

/* slimspec_head_topk (second display of section 4.1) for weights that do not change
 * between calls, as in serving: the caller also passes Bt[V, r], the column-major copy of B
 * made by slimspec_transpose_weights(B, r, V, Bt).  Same operation and outputs.  With five rows
 * or more and k <= 16 the projection runs on 16-bit operands and uncertain ranks are settled
 * by exact fp32 logits of single columns: a column is r adjacent elements of Bt but one
 * element per 128-byte line of B, so these reads shrink by the line length.  Log-probabilities
 * may differ from slimspec_head_topk's in the last bits (another summation order of the exact
 * logits).  With fewer rows Bt is not read.  Bt must match B: nothing checks it. */
int slimspec_head_topk_prepared(const void *h, const void *A, const void *B, const void *Bt,
                                const slimspec_shape *shape, int32_t k,
                                int32_t *out_ids, float *out_logprobs,
                                void *workspace, size_t workspace_bytes,
                                void *stream);

/* The low-rank head for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same operation, kernels and results as slimspec_head_topk, but the scratch
 * is a fixed array of SLIMSPEC_STATIC_SCRATCH_BYTES inside the library's device code
 * (every GPU the library runs on holds one copy until the process ends); the call
 * allocates and frees nothing.  Shapes whose scratch need
 * (slimspec_workspace_bytes' figure for the low-rank head alone) exceeds that size are
 * refused with SLIMSPEC_SCRATCH_LIMIT before anything is enqueued.  All calls on one GPU
 * share that GPU's array: calls that overlap in time on one GPU (different streams or
 * host threads) race and give undefined results; calls on one stream are ordered and
 * safe.  The array keeps the previous call's contents; no kernel relies on them. */
int slimspec_head_topk_static(const void *h, const void *A, const void *B,
                              const slimspec_shape *shape, int32_t k,
                              int32_t *out_ids, float *out_logprobs,
                              void *stream);

/* Full head (first display of section 4.1): z = h W, same reduction.  W is bf16 or
 * fp32 as named by w_dtype; shape->r is ignored. */
int full_head_topk(const void *h, const void *W, slimspec_dtype w_dtype,
                   const slimspec_shape *shape, int32_t k,
                   int32_t *out_ids, float *out_logprobs,
                   void *workspace, size_t workspace_bytes,
                   void *stream);

/* The heads with the outputs stochastic decoding needs (section 5.3 evaluates temperature 1;
 * section 3.2 counts the softmax over the whole vocabulary, which sampling and acceptance need,
 * among the per-step overheads): besides the top-k of slimspec_head_topk / full_head_topk,
 *     out_lse             [rows] float   log sum_v exp(z_v) over the whole vocabulary, so that
 *                                        log q(v) = z_v - lse can be formed for any token
 *     out_sample_ids      [rows] int32   one draw per row from softmax(z) (temperature 1)
 *     out_sample_logprobs [rows] float   its log-probability
 * all DEVICE memory.  The draw is the Gumbel-max rule argmax_v (z_v + g_v) with standard Gumbel
 * noise that is a pure function of (seed, row, id):
 *     x = id * 0x9E3779B1 + row * 0x85EBCA77 + seed_lo (mod 2^32);  x = mix(x);
 *     x = x + seed_hi * 0xC2B2AE3D;  x = mix(x);
 *     mix(x): x ^= x >> 16; x *= 0x21F0AAAD; x ^= x >> 15; x *= 0x735A2D97; x ^= x >> 15;
 *     n = x >> 9;  u = (2 n + 1) / 2^24;  E = -ln(1 - u);  g = -ln E
 * (seed_lo, seed_hi: the halves of `seed`; row: the row's index in the call), so a call with the
 * same seed draws the same tokens on any row count or launch shape; equal z_v + g_v: the
 * smaller id.  Same workspace size as the top-k calls. */
int slimspec_head_sample(const void *h, const void *A, const void *B,
                         const slimspec_shape *shape, int32_t k, uint64_t seed,
                         int32_t *out_ids, float *out_logprobs,
                         float *out_lse, int32_t *out_sample_ids, float *out_sample_logprobs,
                         void *workspace, size_t workspace_bytes,
                         void *stream);
int full_head_sample(const void *h, const void *W, slimspec_dtype w_dtype,
                     const slimspec_shape *shape, int32_t k, uint64_t seed,
                     int32_t *out_ids, float *out_logprobs,
                     float *out_lse, int32_t *out_sample_ids, float *out_sample_logprobs,
                     void *workspace, size_t workspace_bytes,
                     void *stream);

/* Low-rank head with one down-projection per drafted position and a shared up-projection
 * (the direction section 7 names as future work: "position-specific down-projections while
 * sharing a single up-projection"):  t_i = h_i A^(p(i)),  z_i = t_i B.  A_stack: device, bf16,
 * [n_pos, d, r] row-major.  The rows are ordered by position: rows [pos_offsets[p],
 * pos_offsets[p + 1]) use matrix p.  pos_offsets: HOST array of n_pos + 1 int32, read during
 * the call only; pos_offsets[0] = 0, pos_offsets[n_pos] = rows, non-decreasing (a position may
 * have no rows); 1 <= n_pos <= SLIMSPEC_MAX_POSITIONS.  Everything else, the workspace size
 * included, as slimspec_head_topk; with n_pos = 1 it is slimspec_head_topk. */
int slimspec_head_topk_positions(const void *h, const void *A_stack, int32_t n_pos, const int32_t *pos_offsets,
                                 const void *B, const slimspec_shape *shape, int32_t k,
                                 int32_t *out_ids, float *out_logprobs,
                                 void *workspace, size_t workspace_bytes,
                                 void *stream);

/* Truncated-vocabulary head (section 2, "Static vocabulary truncation": the drafter's head
 * restricted to a kept subset V_tr of the vocabulary, plus a token-index map; the baseline
 * family of Appendix C's VocabTrim / FR-Spec rows): z = h W_tr over the V_tr kept columns only,
 * W_tr [d, V_tr] row-major (shape->V = V_tr, shape->r ignored), the softmax and the top-k run
 * over those columns, and the emitted ids are id_map[column].  id_map: device, int32 [V_tr],
 * read only for the k winners of every row.  Equal logits: smaller COLUMN first.  Everything
 * else as full_head_topk (workspace: slimspec_workspace_bytes of the same shape). */
int truncated_head_topk(const void *h, const void *W_tr, slimspec_dtype w_dtype, const int32_t *id_map,
                        const slimspec_shape *shape, int32_t k,
                        int32_t *out_ids, float *out_logprobs,
                        void *workspace, size_t workspace_bytes,
                        void *stream);

/* Router-then-exact head (section 2, "Dynamic vocabulary selection": a low-rank router scores
 * the vocabulary, the best-scoring tokens are kept and the full head is evaluated on those only;
 * the shape of the SpecVocab baseline of Appendix C):
 *     q = (h A) B over all V          (the router: slimspec_head_topk with k = k_route)
 *     S = the k_route ids of the largest q of the row
 *     y_v = h W[:, v] for v in S       (exact full-head logits, fp32 accumulation)
 *     outputs: the k best of S by y (equal y: smaller id) with y_v - log sum_{u in S} exp(y_u)
 * W [d, V] bf16 or fp32; 1 <= k <= k_route <= SLIMSPEC_KMAX.  Workspace: routed_workspace_bytes.
 * (A router k above 16 takes the streaming kernels in groups of 8 rows: meant for few rows.) */
size_t routed_workspace_bytes(const slimspec_shape *shape, int32_t k_route);
int routed_head_topk(const void *h, const void *A, const void *B, const void *W, slimspec_dtype w_dtype,
                     const slimspec_shape *shape, int32_t k_route, int32_t k,
                     int32_t *out_ids, float *out_logprobs,
                     void *workspace, size_t workspace_bytes,
                     void *stream);

/* slimspec_head_sample and slimspec_head_topk_positions with the column-major copy Bt [V, r]
 * of B as well (see slimspec_head_topk_prepared): same operations and outputs; ids, draws and
 * log-probabilities as from the plain calls up to the summation order of the exact logits. */
int slimspec_head_sample_prepared(const void *h, const void *A, const void *B, const void *Bt,
                                  const slimspec_shape *shape, int32_t k, uint64_t seed,
                                  int32_t *out_ids, float *out_logprobs,
                                  float *out_lse, int32_t *out_sample_ids, float *out_sample_logprobs,
                                  void *workspace, size_t workspace_bytes,
                                  void *stream);
int slimspec_head_topk_positions_prepared(const void *h, const void *A_stack, int32_t n_pos,
                                          const int32_t *pos_offsets, const void *B, const void *Bt,
                                          const slimspec_shape *shape, int32_t k,
                                          int32_t *out_ids, float *out_logprobs,
                                          void *workspace, size_t workspace_bytes,
                                          void *stream);

/* routed_head_topk for weights in the layouts a serving stack keeps anyway: Wt [V, d] is the
 * token-major full head (the transpose of W [d, V]: the row of a token is d adjacent elements,
 * bf16 or fp32 by w_dtype, 16-byte aligned), so the exact logits of the routed ids read
 * k_route * d adjacent-element rows instead of one element per 128-byte line; Bt is null or
 * the column-major copy of B for the router (see slimspec_head_topk_prepared).  Same operation
 * and outputs (the exact logits are summed in another order: last bits).  Nothing checks that
 * Wt and Bt match W and B. */
int routed_head_topk_prepared(const void *h, const void *A, const void *B, const void *Bt,
                              const void *Wt, slimspec_dtype w_dtype,
                              const slimspec_shape *shape, int32_t k_route, int32_t k,
                              int32_t *out_ids, float *out_logprobs,
                              void *workspace, size_t workspace_bytes,
                              void *stream);

/* Human-readable name of a status code (static storage). */
const char *slimspec_status_string(int status);

/* Text of the HIP error behind the calling thread's most recent SLIMSPEC_HIP_ERROR
 * ("" if none).  Static/thread-local storage. */
const char *slimspec_last_hip_error(void);

/* Measurement aid (not part of the method).  This is per-thread state that lasts until
 * it is switched off again: when both are non-NULL, every later call
 * made by this host thread records `start_event` just before and `stop_event` just
 * after its vocabulary-projection kernel (the kernel that streams B or W; for calls
 * that run it several times, the first run) on the call's stream, so a harness can
 * read that kernel's duration with hipEventElapsedTime.  Both are hipEvent_t handles
 * owned by the caller and must outlive the calls.  NULL, NULL switches it off.
 * Returns SLIMSPEC_OK, or SLIMSPEC_INVALID_ARGUMENT if exactly one is NULL. */
int slimspec_set_timing_events(void *start_event, void *stop_event);

#ifdef __cplusplus
}
#endif
#endif /* SLIMSPEC_H */

// Per-lane stream bookkeeping shared by the matrix-core head kernels: every lane keeps, for each
// row it owns, a running max / sum of exp and the L largest "group maxima" of its share of the
// vocabulary (a group = the 16 logits of one row that one 32x32 MFMA tile gives a lane).
#pragma once
#include "device_utils.hpp"

namespace slimspec {

// plain VALU min / max / median without the canonicalising pre-ops the compiler adds for fmaxf
__device__ __forceinline__ float vmax(float a, float b) { float d; asm("v_max_f32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b)); return d; }
__device__ __forceinline__ float vmin(float a, float b) { float d; asm("v_min_f32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b)); return d; }
__device__ __forceinline__ float vmed3(float a, float b, float c) { float d; asm("v_med3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c)); return d; }

// ---------------------------------------------------------------------------
// Per-lane stream of one row.
template <int L>
struct Stream {
    float mc, s, U;          // running max (times log2 e), sum of exp relative to it, best dropped group maximum
    float x[L], y[L];        // group maxima (low 4 bits = position in the group) and second largest values
    int tag[L];              // group name: vocabulary tile * 8 + MFMA tile
};

constexpr float kNegBig = -3.0e38f;     // stands for "no value" (finite, so that tagging its low bits stays a number)

template <int L>
__device__ __forceinline__ void stream_init(Stream<L> &st) {
    st.mc = kNegBig; st.s = 0.f; st.U = kNegBig;
#pragma unroll
    for (int l = 0; l < L; ++l) { st.x[l] = kNegBig; st.y[l] = kNegBig; st.tag[l] = 0; }
}

// Fold one group (16 logits of one row) into the stream.
template <int L>
__device__ __forceinline__ void stream_group(Stream<L> &st, const float (&v)[16], int tag)
{
    float p[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) p[i] = __uint_as_float((__float_as_uint(v[i]) & 0xfffffff0u) | (uint32_t)i);
    // largest and second largest of the 16 tagged values
    float a[8], b[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) { a[q] = vmax(p[2 * q], p[2 * q + 1]); b[q] = vmin(p[2 * q], p[2 * q + 1]); }
#pragma unroll
    for (int w = 4; w >= 1; w >>= 1)
#pragma unroll
        for (int q = 0; q < w; ++q) {
            float hi = vmax(a[2 * q], a[2 * q + 1]);
            float lo = vmed3(a[2 * q], a[2 * q + 1], vmax(b[2 * q], b[2 * q + 1]));
            a[q] = hi; b[q] = lo;
        }
    float gm = a[0], g2 = b[0];

    // running log-sum-exp (base 2 inside)
    const float mc_new = vmax(st.mc, gm * kLog2e);
    float sum = st.s * __builtin_amdgcn_exp2f(st.mc - mc_new);
#pragma unroll
    for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(v[i], kLog2e, -mc_new));
    st.s = sum;
    st.mc = mc_new;

    // keep the L groups with the largest maxima
    int tg = tag;
#pragma unroll
    for (int l = 0; l < L; ++l) {
        const bool c = gm > st.x[l];
        const float nx = c ? gm : st.x[l], ny = c ? g2 : st.y[l];
        const int nt = c ? tg : st.tag[l];
        gm = c ? st.x[l] : gm; g2 = c ? st.y[l] : g2; tg = c ? st.tag[l] : tg;
        st.x[l] = nx; st.y[l] = ny; st.tag[l] = nt;
    }
    st.U = vmax(st.U, gm);
}

// Work of block g: row block rb and the vocabulary tiles col, col + gw, col + 2 gw, ...
// Blocks are dealt round-robin to the 8 XCDs, so blocks g and g + 8 share an L2: they get the same
// vocabulary tiles and different row blocks, and so read each tile of M from HBM once.
struct HeadGrid { int n_rb, gw, n_vt; };

}  // namespace slimspec

// Per-lane stream bookkeeping of the matrix-core head kernel: every lane keeps, for each
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

__device__ __forceinline__ float vmax3(float a, float b, float c) { float d; asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c)); return d; }

// Largest and second largest of 16 values in 20 instructions: five triples (max3 / med3), then
// "top two of three pairs" = (max3 of the maxima, max(med3 of the maxima, the seconds)).
__device__ __forceinline__ void top2_of_16(const float (&p)[16], float &hi, float &lo) {
    float h[5], l[5];
#pragma unroll
    for (int t = 0; t < 5; ++t) { h[t] = vmax3(p[3 * t], p[3 * t + 1], p[3 * t + 2]); l[t] = vmed3(p[3 * t], p[3 * t + 1], p[3 * t + 2]); }
    const float ha = vmax3(h[0], h[1], h[2]);
    const float la = vmax(vmax3(vmed3(h[0], h[1], h[2]), l[0], l[1]), l[2]);
    const float hb = vmax3(h[3], h[4], p[15]);
    const float lb = vmax3(vmed3(h[3], h[4], p[15]), l[3], l[4]);
    hi = vmax(ha, hb);
    lo = vmed3(ha, hb, vmax(la, lb));
}

// Fold one group into the stream when the 16 values are base-2 logits RELATIVE to `ref` (the accumulators
// were started at -ref): the sum of 2^v needs no subtraction; the group's top two go back to absolute
// values for the list.  The caller rescales st.s and moves st.mc once per tile (see tile_max).
// NAT: the values are natural-log logits (the operand was not pre-multiplied by log2 e): one multiply more.
template <int L, bool NAT>
__device__ __forceinline__ void stream_group_rel(Stream<L> &st, const float (&v)[16], float ref, float &tile_max, int tag)
{
    float p[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) p[i] = __uint_as_float((__float_as_uint(v[i]) & 0xfffffff0u) | (uint32_t)i);
    float gr, g2r;
    top2_of_16(p, gr, g2r);
    __builtin_amdgcn_sched_barrier(0);          // the tagged copies are dead before the exponentials start
    float sum = st.s;
#pragma unroll
    for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(NAT ? v[i] * kLog2e : v[i]);
    st.s = sum;
    float gm = __uint_as_float((__float_as_uint(gr + ref) & 0xfffffff0u) | (__float_as_uint(gr) & 15u));
    float g2 = g2r + ref;
    tile_max = vmax(tile_max, gm);
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

// Fold stream b into stream a (both cover different logits of the same row): log-sum-exp in base 2, the L
// largest group maxima of the union, U = the largest maximum that is not listed.
template <int L>
__device__ __forceinline__ void stream_combine(Stream<L> &a, const Stream<L> &b)
{
    const float m = fmaxf(a.mc, b.mc);
    a.s = a.s * __builtin_amdgcn_exp2f(a.mc - m) + b.s * __builtin_amdgcn_exp2f(b.mc - m);
    a.mc = m;
    a.U = fmaxf(a.U, b.U);
#pragma unroll
    for (int e = 0; e < L; ++e) {
        float gm = b.x[e], g2 = b.y[e];
        int tg = b.tag[e];
#pragma unroll
        for (int l = 0; l < L; ++l) {
            const bool c = gm > a.x[l];
            const float nx = c ? gm : a.x[l], ny = c ? g2 : a.y[l];
            const int nt = c ? tg : a.tag[l];
            gm = c ? a.x[l] : gm; g2 = c ? a.y[l] : g2; tg = c ? a.tag[l] : tg;
            a.x[l] = nx; a.y[l] = ny; a.tag[l] = nt;
        }
        a.U = fmaxf(a.U, gm);
    }
}

// ---------------------------------------------------------------------------
// Gumbel-max sampling next to a stream: the two largest z_v + g_v the lane has seen for the row (in the records'
// units) with their vocabulary ids, and the third largest (a bound for everything else the lane saw).
struct SampleTrack { float w1, w2, w3; int id1, id2; };
__device__ __forceinline__ void sample_init(SampleTrack &s) { s.w1 = kNegBig; s.w2 = kNegBig; s.w3 = kNegBig; s.id1 = 0; s.id2 = 0; }

// The 16 values of one group (relative to `ref`, as in stream_group_rel); id0: the vocabulary id of element 0, element
// i sits at id0 + 8 (i / 4) + i % 4.  Ids rise with i and from group to group, so "strictly larger" keeps the smaller
// id among equal sums.
template <bool NAT>
__device__ __forceinline__ void sample_group(SampleTrack &s, const float (&v)[16], float ref, const GumbelKey &gk, int id0)
{
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int id = id0 + 8 * (i >> 2) + (i & 3);
        const float g2 = gumbel_base2(gk, (uint32_t)id);
        const float w = (v[i] + ref) + (NAT ? g2 * kLn2 : g2);
        const bool first = w > s.w1, second = w > s.w2;
        s.w3 = second ? s.w2 : vmax(s.w3, w);
        s.w2 = first ? s.w1 : (second ? w : s.w2);
        s.id2 = first ? s.id1 : (second ? id : s.id2);
        s.id1 = first ? id : s.id1;
        s.w1 = first ? w : s.w1;
    }
}

// fold track b into a (both saw different logits of the same row)
__device__ __forceinline__ void sample_combine(SampleTrack &a, const SampleTrack &b)
{
    // merge of two sorted pairs (ties: smaller id first); the third place takes what is left
    const auto before = [](float wa, int ia, float wb, int ib) { return wa > wb || (wa == wb && ia < ib); };
    SampleTrack r;
    const bool a1 = before(a.w1, a.id1, b.w1, b.id1);
    r.w1 = a1 ? a.w1 : b.w1; r.id1 = a1 ? a.id1 : b.id1;
    // candidates for second: the loser of the heads, and the winner's own second
    const float lw = a1 ? b.w1 : a.w1, ow = a1 ? a.w2 : b.w2;
    const int li = a1 ? b.id1 : a.id1, oi = a1 ? a.id2 : b.id2;
    const bool l2 = before(lw, li, ow, oi);
    r.w2 = l2 ? lw : ow; r.id2 = l2 ? li : oi;
    // third: the larger of what was not taken (values only)
    const float rest = l2 ? fmaxf(ow, a1 ? b.w2 : a.w2) : fmaxf(lw, a1 ? a.w3 : b.w3);
    r.w3 = fmaxf(rest, fmaxf(a.w3, b.w3));
    a = r;
}

// Work of block g: row block rb and the vocabulary tiles col, col + gw, col + 2 gw, ...
// Blocks are dealt round-robin to the 8 XCDs, so blocks g and g + 8 share an L2: they get the same
// vocabulary tiles and different row blocks, and so read each tile of M from HBM once.
struct HeadGrid { int n_rb, gw, n_vt, spb; };      // spb: records a block leaves per row (4, 2 or 1)

}  // namespace slimspec

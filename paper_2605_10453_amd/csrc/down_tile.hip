// Down-projection t = h A for calls with many rows (paper section 4.1, the first of the two dense products).
//
//   down_tile_kernel     64 x 64 tiles of t over a slice of the contraction (bf16 MFMA, fp32 accumulate)
//   down_finish_kernel   fixed-order sum of the slices -> fp32 t, the 16-bit t in the k-grouped layout the
//                        up-projection kernel reads, per-row rounding statistics; further blocks of the same launch
//                        estimate the scale of B's columns per 256-column vocabulary tile
//
// A CU fills its LDS at a few tens of bytes per clock, so what a block has to load decides the time: a block owns a
// 64 x 64 tile (its four wavefronts share every stage, 32 x 32 each) and the contraction is split over as many slices
// as it takes to give every CU a block.  Stages of 32 contraction elements travel global memory -> LDS without
// passing registers (global_load_lds_dwordx4): 32 rows of A as full 128-byte lines, the 64 rows of h as 16-byte
// vectors of 8 consecutive contraction elements.  The A operand of the transposed product t^T = A^T h^T comes from
// LDS through the transposing read (4 consecutive contraction elements of one column per lane).
//
// Waits: the compiler does not see the direct-to-LDS loads (inline asm), so the kernel counts them itself: every
// wavefront issues exactly two per stage, vector memory returns in order, hence s_waitcnt vmcnt(2 (NB - 2)) =
// "my part of the stage needed next has landed", and the barrier that follows publishes the stage.
#include "device_utils.hpp"
#include "launch.hpp"

namespace slimspec {

namespace {

constexpr int kDT = 64;                     // rows and columns of t per block
constexpr int kDKB = 32;                    // contraction elements per stage
constexpr int kDStageBytes = 8192;          // 4 KB of A (32 rows x 128 B), 4 KB of h (64 rows x 64 B)
constexpr int kDNB = 8;                     // stage buffers
constexpr int kDLoads = 2;                  // loads per wavefront and stage
constexpr int kDLds = kDNB * kDStageBytes;  // 64 KB
constexpr int kColSamples = 32;             // entries sampled per column of B for its scale (see column_scale_block)
constexpr float kTileMaxBias = 1.35f;      // expected largest / true of 256 column rms estimates from 32 samples each
constexpr float kTileNoiseRatio = 2.8f;    // largest column mean square / tile mean square that sampling noise alone explains (1.8 in a typical tile, 2.2 in the
                                           // most extreme of the 500 tiles of a Gaussian B; a column of 1.6 times the rms of its tile and more stands out)

typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define LDS_PTR(T, byte_addr) ((__attribute__((address_space(3))) T *)(uintptr_t)(byte_addr))

// 16 bytes per lane, global memory -> LDS at buf + 16 * lane (buf uniform)
__device__ __forceinline__ void dma16(uint32_t buf, uint32_t voff, const void *base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(buf), "v"(voff), "s"(base) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_loads() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }

}  // namespace

// Scale of B's columns, for the bound on what rounding t to 16 bits does to a logit (the error of column v is
// sum_j dt_j B[j, v], about |dt| times the column's rms).  Block b covers columns [512 b, 512 b + 512): thread
// (8 adjacent columns, row phase tid / 64) squares every col_stride-th row of its columns, 16 loads in flight at a
// time (full 128-byte lines per wavefront); the four phases meet in shared memory in a fixed order; the block writes,
// for each of its two 256-column vocabulary tiles, (the largest column rms, the mean square of the tile's entries).  The sample covers every column and a
// subset of rows (all rows up to r = kColSamples, at least kColSamples rows beyond), 1 / col_stride of B's bytes: sample i of a group
// of 64 columns (one 128-byte line per row) is row i col_stride + (c + 5 i) mod col_stride with c depending on the
// group, so that a periodic pattern over the rows of B is sampled in proportion and cannot hide from a column's sum.
__device__ __forceinline__ void column_scale_block(const uint16_t *__restrict__ B, int r, int V, float2 *__restrict__ tilescale,
                                                   int b, float *sh, int tid)
{
    const int col_stride = max(1, r / kColSamples), n_s = (r + col_stride - 1) / col_stride;
    const int oct = tid & 63, phase = tid >> 6;
    const int col = b * 512 + oct * 8;
    const int g64 = col >> 6;
    const int row_off = 13 * (g64 >> 2) + 3 * (g64 & 3);
    const auto sample_row = [&](int i) { return i * col_stride + (row_off + 5 * i) % col_stride; };
    float ss[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) ss[e] = 0.f;
    if (col < V) {
        const uint16_t *src = B + col;
        constexpr int NL = 8;                                  // loads in flight per thread
        for (int i0 = phase; i0 < n_s; i0 += 4 * NL) {
            uint4 w[NL];
#pragma unroll
            for (int u = 0; u < NL; ++u)
                w[u] = *reinterpret_cast<const uint4 *>(src + (size_t)min(sample_row(min(i0 + 4 * u, n_s - 1)), r - 1) * V);
#pragma unroll
            for (int u = 0; u < NL; ++u) {
                if (i0 + 4 * u >= n_s || sample_row(i0 + 4 * u) >= r) continue;
                const float f[8] = {bf16_lo(w[u].x), bf16_hi(w[u].x), bf16_lo(w[u].y), bf16_hi(w[u].y),
                                    bf16_lo(w[u].z), bf16_hi(w[u].z), bf16_lo(w[u].w), bf16_hi(w[u].w)};
#pragma unroll
                for (int e = 0; e < 8; ++e) ss[e] = fmaf(f[e], f[e], ss[e]);
            }
        }
    }
    float m = 0.f;                                             // largest sum of squares among this thread's columns
    if (phase != 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sh[((phase - 1) * 64 + oct) * 8 + e] = ss[e];
    }
    __syncthreads();
    if (phase == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float v = ((ss[e] + sh[oct * 8 + e]) + sh[(64 + oct) * 8 + e]) + sh[(128 + oct) * 8 + e];
            m = fmaxf(m, v);
        }
        // lanes 0..31: the block's first vocabulary tile, lanes 32..63: its second
        m = fmaxf(m, dpp_f32<0xB1>(m));
        m = fmaxf(m, dpp_f32<0x4E>(m));
        m = fmaxf(m, dpp_f32<0x141>(m));
        m = fmaxf(m, dpp_f32<0x140>(m));
        uint32_t x, y;
        swap_pair<16>(__float_as_uint(m), x, y);
        m = fmaxf(__uint_as_float(x), __uint_as_float(y));
        // ... and the tile's mean square (its columns' sums added in lane order)
        float sum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) sum += ((ss[e] + sh[oct * 8 + e]) + sh[(64 + oct) * 8 + e]) + sh[(128 + oct) * 8 + e];
        sum += dpp_f32<0xB1>(sum);
        sum += dpp_f32<0x4E>(sum);
        sum += dpp_f32<0x141>(sum);
        sum += dpp_f32<0x140>(sum);
        swap_pair<16>(__float_as_uint(sum), x, y);
        sum = __uint_as_float(x) + __uint_as_float(y);
        const int vt = 2 * b + (oct >> 5);
        const int tile_cols = min(256, V - vt * 256);
        if ((oct & 31) == 0 && tile_cols > 0) {
            // The largest of 256 rms estimates from 32 samples each overshoots the true rms of equal columns by about
            // a third (1.35); where it stands further above the tile's own mean square than that noise explains, the
            // tile holds a column that really is larger: then the estimate stands (its own noise is 12 %: 1.1 on top).
            const float max_ms = m / (float)n_s, tile_ms = sum / ((float)n_s * (float)tile_cols);
            const float scale = (max_ms <= kTileNoiseRatio * tile_ms) ? sqrtf(max_ms) * (1.f / kTileMaxBias) : sqrtf(max_ms) * 1.1f;
            tilescale[vt] = make_float2(scale, tile_ms);
        }
    }
}

// part [slices][n_rt][n_ct][4 wavefronts][16][64] fp32: the accumulators as the wavefronts hold them; wavefront
// (wr, wc) of tile (rt, ct) owns rows 64 rt + 32 wr + lane % 32 and, for element i, column
// 64 ct + 32 wc + 8 (i / 4) + 4 (lane / 32) + i % 4.
// Block g works on XCD g % 8 (each XCD has its own L2): slices are dealt to the XCDs first, so that an XCD reads
// only its slices' rows of A and columns of h.
__global__ __launch_bounds__(256) void down_tile_kernel(
    const uint16_t *__restrict__ h, const uint16_t *__restrict__ A, float *__restrict__ part,
    int d, int r, DownGrid g)
{
    extern __shared__ __align__(1024) unsigned char lds_raw[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) unsigned char *)lds_raw);
    const int tid = threadIdx.x, lane = tid & 63;

    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, wc = wave & 1;

    int slice, tile;
    {
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        if (g.slices >= 8) { slice = xcd + 8 * (slot % (g.slices >> 3)); tile = slot / (g.slices >> 3); }
        else { slice = xcd % g.slices; tile = xcd / g.slices + (8 / g.slices) * slot; }
    }
    if (tile >= g.n_rt * g.n_ct) return;
    const int rt = tile % g.n_rt, ct = tile / g.n_rt;
    int grp = 0;                                               // the group of rows (one down-projection matrix) this row tile belongs to
    while (grp + 1 < g.n_groups && rt >= g.g_tile0[grp + 1]) ++grp;
    const int row0 = g.g_row0[grp] + (rt - g.g_tile0[grp]) * kDT, n0 = ct * kDT;
    const int rows = g.g_row0[grp + 1];                        // rows beyond the group's last are not this tile's
    A += (size_t)g.g_mat[grp] * d * r;
    const int half = lane >> 5, l32 = lane & 31, g1 = (lane >> 4) & 1, j16 = lane & 15;

    f32x16 acc0, acc1;
#pragma unroll
    for (int i = 0; i < 16; ++i) { acc0[i] = 0.f; acc1[i] = 0.f; }

    // stages [s_beg, s_end) of the d / 32 full ones; what is left of d (8, 16 or 24 elements) is added by the finish kernel
    const int n_full = d / kDKB;
    const int per = (n_full + g.slices - 1) / g.slices;
    const int s_beg = min(n_full, slice * per), s_end = min(n_full, s_beg + per);
    const int nst = (n0 < r) ? s_end - s_beg : 0;                         // columns of padding load nothing
    if (nst > 0) {
        // The two loads of this wavefront per stage:
        //   A: stage rows 8 wave + lane / 8, 16-byte piece lane % 8 of the tile's 128 bytes; the piece is stored at
        //      position piece ^ 4 in rows with (row & 2) set, so that the four rows a transposing read touches fall
        //      into different banks; columns >= r are clamped to the last piece that exists (never used)
        //   h: rows 16 wave + lane % 16, 8-element group lane / 16 of the stage (rows beyond the last: the last)
        const int a_row = 8 * wave + (lane >> 3);
        const int a_piece = (lane & 7) ^ ((a_row & 2) << 1);
        const uint32_t a_off = (uint32_t)a_row * (uint32_t)r * 2u + (uint32_t)min(n0 + 8 * a_piece, r - 8) * 2u;
        const uint32_t h_off = (uint32_t)min(row0 + 16 * wave + (lane & 15), rows - 1) * (uint32_t)d * 2u + (uint32_t)(lane >> 4) * 16u;
        // (Blocks of one XCD walk the same slice in step.  Starting them at different points of it, so that they
        // prefetch for each other, measured slower: 10.0 against 8.9 us at 512 rows.)
        const unsigned char *a_ptr = reinterpret_cast<const unsigned char *>(A) + (size_t)s_beg * kDKB * r * 2;
        const unsigned char *h_ptr = reinterpret_cast<const unsigned char *>(h) + (size_t)s_beg * kDKB * 2;
        const size_t a_step = (size_t)kDKB * r * 2, h_step = (size_t)kDKB * 2;
        int issued = 0;
        uint32_t buf_ahead = lds0;
        const uint32_t a_lds = (uint32_t)(wave * 1024), h_lds = (uint32_t)(4096 + wave * 1024);
        const auto issue_stage = [&]() {
            dma16(buf_ahead + a_lds, a_off, a_ptr);
            dma16(buf_ahead + h_lds, h_off, h_ptr);
            // past the end the last stage is loaded once more (into a buffer nobody reads): the count stays uniform
            if (++issued < nst) { a_ptr += a_step; h_ptr += h_step; }
            buf_ahead = (buf_ahead + kDStageBytes == lds0 + kDLds) ? lds0 : buf_ahead + kDStageBytes;
        };
#pragma unroll
        for (int pre = 0; pre < kDNB - 1; ++pre) issue_stage();

        // operand addresses inside a stage (k-step ks: rows 16 ks .. of A, groups 2 ks, 2 ks + 1 of h)
        const uint32_t xa = (uint32_t)(4096 + (2 * wr + (l32 >> 4)) * 1024 + half * 256 + (l32 & 15) * 16);      // + 512 per k-step
        const int m_row = 8 * half + (j16 >> 2);                                                              // + 4 for the second read, + 16 per k-step
        const int m_piece = (4 * wc + 2 * g1 + ((j16 & 3) >> 1)) ^ ((m_row & 2) << 1);
        const uint32_t ma = (uint32_t)(m_row * 128 + m_piece * 16 + (j16 & 1) * 8);                           // + 2048 per k-step
        uint32_t buf = lds0;
        for (int q = 0; q < nst; ++q) {
            wait_loads<(kDNB - 2) * kDLoads>();               // this wavefront's part of stage q has landed
            __builtin_amdgcn_s_barrier();                     // ... everybody's; and everybody has read stage q - 1
            u32x4 xf[2], mf[2];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                xf[ks] = *LDS_PTR(u32x4, buf + xa + ks * 512);
                const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4i16, buf + ma + ks * 2048));
                const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4i16, buf + ma + ks * 2048 + 512));
                mf[ks] = __builtin_bit_cast(u32x4, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            }
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, mf[0]), __builtin_bit_cast(bf16x8, xf[0]), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, mf[1]), __builtin_bit_cast(bf16x8, xf[1]), acc1, 0, 0, 0);
            // the next loads go to the buffer of stage q - 1, which every wavefront finished reading before the barrier above
            issue_stage();
            buf = (buf + kDStageBytes == lds0 + kDLds) ? lds0 : buf + kDStageBytes;
        }
        wait_loads<0>();                                      // the surplus loads of the last stages
    }
    float *dst = part + ((((size_t)slice * g.n_rt + rt) * g.n_ct + ct) * 4 + wave) * (16 * 64) + lane;
#pragma unroll
    for (int i = 0; i < 16; ++i) dst[i * 64] = acc0[i] + acc1[i];
}

// Fixed-order sum of the slices and everything that follows from t.  One block of 256 threads per 32 x 32 piece of
// t (a wavefront's share of a tile of down_tile_kernel); grid = 4 n_rt n_ct.
//   t32   [rows_pad, r]            fp32 t (zero for padding rows)
//   t16   [8 ceil(r / 64), rows_pad]   16-byte vectors of 8 values t log2(e) in bf16 or f16 (round to nearest even),
//                                      zero for k >= r and for padding rows
//   stat  [2 ceil(r / 64), rows_pad]   per 32-column piece: (sum of (t - its 16-bit value)^2, sum of t^2) of its entries
__global__ __launch_bounds__(256) void down_finish_kernel(
    const float *__restrict__ part, const uint16_t *__restrict__ h, const uint16_t *__restrict__ A,
    int rows_pad, int d, int r,
    float *__restrict__ t32, uint4 *__restrict__ t16, float2 *__restrict__ stat,
    const uint16_t *__restrict__ B, int V, float2 *__restrict__ tilescale, int as_f16, DownGrid g)
{
    __shared__ float tile[32 * 33];
    __shared__ float red_a[4 * 32], red_b[4 * 32];
    __shared__ float colsh[3 * 64 * 8];
    const int tid = threadIdx.x;
    if ((int)blockIdx.x >= 4 * g.n_rt_all * g.n_ct) {
        // (next to the tile kernel's blocks instead, these blocks cost 6.7 us at 512 rows; here 2-3)
        column_scale_block(B, r, V, tilescale, (int)blockIdx.x - 4 * g.n_rt_all * g.n_ct, colsh, tid);
        return;
    }
    const int piece = blockIdx.x;                              // ((rt * n_ct + ct) * 4 + wave of the tile kernel)
    const int w = piece & 3, ct = (piece >> 2) % g.n_ct, rt = (piece >> 2) / g.n_ct;      // rt < n_rt_all; no partial sums exist for rt >= n_rt
    int grp = 0;                                               // group n_groups: the rows of padding, zero-filled
    while (grp < g.n_groups && rt >= g.g_tile0[grp + 1]) ++grp;
    const int row0 = g.g_row0[grp] + (rt - g.g_tile0[grp]) * kDT + 32 * (w >> 1), n0 = ct * kDT + 32 * (w & 1);
    const int row_end = g.g_row0[grp + 1];                     // this piece's rows end with its group
    const int rows = (grp < g.n_groups) ? row_end : 0;         // rows that carry values
    A += (size_t)g.g_mat[grp < g.n_groups ? grp : 0] * d * r;

    // the slices, in order: several loads of a thread are in flight together (they come from other CUs' writes)
    const size_t slice_stride = (size_t)g.n_rt * g.n_ct * 4 * (16 * 64);
    const float *src = part + (((size_t)rt * g.n_ct + ct) * 4 + w) * (16 * 64);
    const int k_tail0 = (d / kDKB) * kDKB;
    // a thread owns four (i, lane) pairs of the accumulator layout; the loads of SB slices of all four are in flight together
    constexpr int SB = 8;
    float v4[4] = {0.f, 0.f, 0.f, 0.f};
    const int n_slices = grp < g.n_groups ? g.slices : 0;
    for (int s0 = 0; s0 < n_slices; s0 += SB) {
        float x[SB][4];
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            const float *sp = src + (size_t)min(s0 + u, n_slices - 1) * slice_stride + tid;
#pragma unroll
            for (int e = 0; e < 4; ++e) x[u][e] = sp[256 * e];
        }
#pragma unroll
        for (int u = 0; u < SB; ++u)
            if (s0 + u < n_slices) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v4[e] += x[u][e];
            }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int qq = tid + 256 * e;                          // (i, lane) pair
        const int i = qq >> 6, ln = qq & 63;
        float v = v4[e];
        const int row = ln & 31, n = 8 * (i >> 2) + 4 * (ln >> 5) + (i & 3);
        if (k_tail0 < d && row0 + row < rows && n0 + n < r) {
            const uint16_t *hr = h + (size_t)(row0 + row) * d;
            for (int kk = k_tail0; kk < d; ++kk)
                v = fmaf(bf16_to_float(hr[kk]), bf16_to_float(A[(size_t)kk * r + n0 + n]), v);
        }
        tile[row * 33 + n] = v;
    }
    __syncthreads();

    // thread (row, group of 8 columns)
    if (tid < 128) {
        const int row = tid & 31, cg = tid >> 5;
        const int kg = (n0 >> 3) + cg;
        const bool valid = row0 + row < rows && kg < (r >> 3);
        const bool mine = row0 + row < row_end;                 // rows beyond belong to the next group's tiles
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = valid ? tile[row * 33 + cg * 8 + e] : 0.f;
        float a = 0.f, b = 0.f;
        if (mine && kg < (r >> 3)) {
            float4 *o = reinterpret_cast<float4 *>(t32 + (size_t)(row0 + row) * r + kg * 8);
            o[0] = make_float4(v[0], v[1], v[2], v[3]);
            o[1] = make_float4(v[4], v[5], v[6], v[7]);
        }
        uint4 packed;
        if (!as_f16) {
            uint32_t hb[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                // bf16 operand of the head kernel, in base-2 units: t log2(e)
                hb[e] = operand_bf16_bits(v[e]);                            // round to nearest even
                const float dlt = v[e] - __uint_as_float(hb[e] << 16) * kLn2;
                a += dlt * dlt;
                b += v[e] * dlt;
            }
            packed = make_uint4(hb[0] | (hb[1] << 16), hb[2] | (hb[3] << 16), hb[4] | (hb[5] << 16), hb[6] | (hb[7] << 16));
        } else {
            f16x8 hv;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                hv[e] = operand_f16(v[e]);
                const float dlt = v[e] - (float)hv[e] * kLn2;
                a += dlt * dlt;
                b += v[e] * dlt;
            }
            packed = __builtin_bit_cast(uint4, hv);
        }
        if (mine) t16[(size_t)kg * rows_pad + row0 + row] = packed;     // kg < 8 ceil(r / 64): the tile grid covers exactly that
        red_a[cg * 32 + row] = a;
        red_b[cg * 32 + row] = b;
    }
    __syncthreads();
    if (tid < 32 && row0 + tid < row_end)
        stat[(size_t)(n0 >> 5) * rows_pad + row0 + tid] =
            make_float2(((red_a[tid] + red_a[32 + tid]) + red_a[64 + tid]) + red_a[96 + tid],
                        ((red_b[tid] + red_b[32 + tid]) + red_b[64 + tid]) + red_b[96 + tid]);
}

hipError_t launch_down_projection_tiles(const uint16_t *h, const uint16_t *A, float *part, const DownGrid &g,
                                        int rows_pad, int d, int r,
                                        float *t32, void *t16, float2 *stat, const uint16_t *B, int V, float2 *tilescale,
                                        bool as_f16, hipStream_t st)
{
    static LdsLimit lds_limit;
    hipError_t e = lds_limit.raise(reinterpret_cast<const void *>(down_tile_kernel), kDLds);
    if (e != hipSuccess) return e;
    const int tiles = g.n_rt * g.n_ct;
    // slices >= 8: every XCD has slices / 8 slices of every tile; fewer: 8 / slices XCDs share a slice and split the tiles
    const int blocks = g.slices >= 8 ? tiles * g.slices : 8 * ((tiles + 8 / g.slices - 1) / (8 / g.slices));
    down_tile_kernel<<<blocks, 256, kDLds, st>>>(h, A, part, d, r, g);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    down_finish_kernel<<<4 * g.n_rt_all * g.n_ct + (V + 511) / 512, 256, 0, st>>>(
        part, h, A, rows_pad, d, r, t32, static_cast<uint4 *>(t16), stat, B, V, tilescale, as_f16 ? 1 : 0, g);
    return hipGetLastError();
}

}  // namespace slimspec

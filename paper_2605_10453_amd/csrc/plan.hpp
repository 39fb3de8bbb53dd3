// Host-side launch plan: which kernels a call runs and where each scratch
// array sits in the caller's workspace.  Pure arithmetic, no HIP calls, so the
// argument checks and the workspace query work on a machine without a GPU.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace slimspec {

constexpr int kChunkCols = 512;      // vocabulary columns per partial at most: one wavefront x 8 columns per lane
constexpr int kGemvMaxRows = 8;      // rows handled by one pass of the streaming (lane-owns-columns) path
constexpr int kMergeThreads = 512;    // threads of the stream-merge block of one row
constexpr int SLIMSPEC_KMAX_INTERNAL = 64;
constexpr size_t kAlign = 256;

enum class HeadKind { LowRank, Full };

// How the few-row down-projection is shared out: n_cb column blocks of 64 columns of A x nds slices of d.
struct DownPlan { int n_items = 0, n_cb = 0, nds = 0, slice = 0; };
inline DownPlan make_down_plan(bool low_rank, int d, int r) {
    DownPlan p;
    if (low_rank) {
        p.n_cb = (r + 63) / 64;
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

// Geometry of the streaming kernel: a block owns one chunk of 8 * lanes adjacent columns (lanes <= 64 lanes of every
// wavefront hold columns) and its nw wavefronts split the contraction.  One block of 16 wavefronts fills a CU, so
// up to 256 chunks run as one round.  A vocabulary with more 512-column chunks than that (151936 columns: 297)
// would leave 41 CUs with two chunks and the others waiting: for a single row the chunks are instead made narrower
// and the blocks smaller (8 wavefronts: two blocks share a CU, 512 at once; 4 wavefronts: 1024 at once) so that all
// of them are resident together and every CU gets the same number of columns within a few per cent.
struct ChunkGeom { int lanes = 64, nw1 = 16, chunks = 0; };
inline ChunkGeom make_chunk_geom(int rows, int V) {
    ChunkGeom g;
    g.chunks = (V + kChunkCols - 1) / kChunkCols;
    if (rows == 1 && g.chunks > 256) {
        const int n16 = (V + 7) / 8;                         // 16-byte column groups
        const int slots = g.chunks <= 512 ? 512 : 1024;
        g.nw1 = g.chunks <= 512 ? 8 : 4;
        if (g.chunks <= slots) {
            g.lanes = (n16 + slots - 1) / slots;
            g.chunks = (n16 + g.lanes - 1) / g.lanes;
        }
    }
    return g;
}

struct Plan {
    bool ok = false;
    int rows = 0, d = 0, r = 0, V = 0, k = 0;
    int K = 0;                 // contraction length of the vocabulary projection (r or d)
    int chunks = 0;            // partials per row
    int lanes = 64, nw1 = 16;  // see ChunkGeom
    // byte offsets into the workspace
    size_t off_x = 0;          // fp32 [kGemvMaxRows, K]: t (low-rank) or widened h (full)
    size_t off_tpart = 0;      // fp32 [nds, kGemvMaxRows, r]  slices of t
    size_t off_part_ms = 0;    // float2 [rows, chunks]      running max, sum of exp
    size_t off_part_val = 0;   // float  [rows, chunks, k]   per-chunk top-k logits
    size_t off_part_id = 0;    // int32  [rows, chunks, k]   per-chunk top-k ids
    size_t off_part_smp = 0;   // float4 [rows, chunks]      per-chunk Gumbel-max winners (sampling calls)
    size_t bytes = 0;
};

inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

inline Plan make_plan(HeadKind kind, int rows, int d, int r, int V, int k) {
    Plan p;
    p.rows = rows; p.d = d; p.r = r; p.V = V; p.k = k;
    p.K = (kind == HeadKind::LowRank) ? r : d;
    const ChunkGeom cg = make_chunk_geom(rows, V);
    p.chunks = cg.chunks; p.lanes = cg.lanes; p.nw1 = cg.nw1;
    size_t off = 0;
    p.off_x = off;          off = align_up(off + sizeof(float) * kGemvMaxRows * (size_t)p.K);
    {
        const DownPlan dp = make_down_plan(kind == HeadKind::LowRank, d, r);
        p.off_tpart = off;  off = align_up(off + sizeof(float) * (size_t)dp.nds * kGemvMaxRows * (size_t)r);
    }
    p.off_part_ms = off;    off = align_up(off + 2 * sizeof(float) * (size_t)rows * p.chunks);
    p.off_part_val = off;   off = align_up(off + sizeof(float) * (size_t)rows * p.chunks * k);
    p.off_part_id = off;    off = align_up(off + sizeof(int32_t) * (size_t)rows * p.chunks * k);
    p.off_part_smp = off;   off = align_up(off + 16 * (size_t)rows * p.chunks);
    p.bytes = off;
    p.ok = true;
    return p;
}

// Dynamic shared memory of the merge kernel: the head key of every list, the gathered
// candidates (at most k lists of k entries), every list's k logits and, optionally, its k ids.
inline size_t merge_lds_bytes(int chunks, int k, bool with_ids = false) {
    return sizeof(uint64_t) * ((size_t)chunks + (size_t)k * k) + (with_ids ? 2 : 1) * sizeof(float) * (size_t)chunks * k;
}
constexpr size_t kMergeLdsLimit = 160 * 1024 - 1024;

// ---- matrix-core path -------------------------------------------------------------------
constexpr int kPlanSlotsPerXcd = 32;     // blocks per XCD of the persistent kernel (256 CUs / 8 XCDs)
constexpr int kStreamsPerBlock = 4;      // lane streams of a row in one block of the head kernel: two half-wavefronts x two column halves
// Records a block of the head kernel leaves per row: all four lane streams while a row then has at most 512 records
// (many rows: few column blocks, where three listed groups per folded record would often be too few), two or one
// where there are more column blocks (the merge's time grows with the number of records).
inline int streams_per_block(int gw) { return gw <= 128 ? kStreamsPerBlock : gw <= 256 ? 2 : 1; }
constexpr int kStreamListPlan = 3;       // must equal kStreamList (launch.hpp)
constexpr int kStreamRecPlan = 3 + 3 * kStreamListPlan + 8;      // sized for sampling calls (kStreamRecSample, launch.hpp)

int head_tile_rows_per_block(int rows);
size_t merge_defer_bytes(int rows);
// Rows whose exact re-evaluations are parked for exact_cols_kernel: worth two more launches when a few rows with long
// column gathers would otherwise hold the merge up.  Always from K = 2048 (the full head: 127 -> 35 us at 512 rows);
// from K = 1024 when the kernel ran on f16 operands, where few rows need any re-evaluation (C5: 42.7 -> 34.3 us).
// With bf16 operands most rows re-evaluate something and the gathers are bound by the memory side's bandwidth, not by
// one CU's latency: parked or not measures the same at K = 1024 (58 us) and worse at K = 512 (32 -> 43 us).
constexpr int kDeferMinK = 2048, kDeferMinKFine = 1024;
inline bool merge_parks_rows(int K, bool fine_operand) { return K >= kDeferMinK || (fine_operand && K >= kDeferMinKFine); }

// Many-row down-projection: tiles of 64 x 64 of t, the contraction in `slices` slices (a power of two): enough
// blocks for every CU, at least two stages of 32 contraction elements per block.  The rows come in groups that share
// a down-projection matrix (one group unless the call names one matrix per drafted position); a row tile never
// crosses a group, and the rows of padding [rows, rows_pad) form one more group that is only zero-filled.
constexpr int kMaxPositions = 16;
struct DownGrid {
    int n_rt = 0;                        // row tiles that hold rows, over all groups
    int n_rt_all = 0;                    // ... with the tiles of the padding group
    int n_ct = 0, slices = 1;
    int n_groups = 0;                    // groups with rows; group n_groups is the padding
    int g_row0[kMaxPositions + 2] = {};  // first row of group g; g_row0[n_groups] = rows, g_row0[n_groups + 1] = rows_pad
    int g_tile0[kMaxPositions + 2] = {}; // first row tile of group g; g_tile0[n_groups + 1] = n_rt_all
    int g_mat[kMaxPositions + 1] = {};   // which matrix of the stack the group uses
};
// group g covers rows [g_first[g], g_first[g + 1]) of the launch (g_first[n_groups] = rows), all groups non-empty
inline DownGrid make_down_grid(int rows, int rows_pad, int d, int r, int n_groups = 1, const int *g_first = nullptr,
                               const int *g_mat = nullptr) {
    DownGrid g;
    g.n_groups = n_groups;
    int tile = 0;
    for (int q = 0; q < n_groups; ++q) {
        const int lo = g_first ? g_first[q] : 0, hi = g_first ? g_first[q + 1] : rows;
        g.g_row0[q] = lo; g.g_tile0[q] = tile; g.g_mat[q] = g_mat ? g_mat[q] : 0;
        tile += (hi - lo + 63) / 64;
    }
    g.n_rt = tile;
    g.g_row0[n_groups] = rows; g.g_tile0[n_groups] = tile;
    tile += (rows_pad - rows + 63) / 64;
    g.g_row0[n_groups + 1] = rows_pad; g.g_tile0[n_groups + 1] = tile;
    g.n_rt_all = tile;
    g.n_ct = (r + 63) / 64;
    const int tiles = g.n_rt * g.n_ct, n_full = d / 32;
    // (two blocks per CU, i.e. twice the slices, measured slower: 10.7 + 4.6 against 8.9 + 4.5 us at 512 rows)
    // (at most 16 slices: with 32, at 16 and 64 rows, the tile kernel measures the same and the sum of the slices 1.1 us more)
    while (g.slices < 16 && tiles * g.slices < 256 && n_full / (2 * g.slices) >= 2) g.slices *= 2;
    return g;
}
// Partial tiles of t, in 64 x 64 tiles of floats, for any grouping of `rows` rows into at most kMaxPositions groups:
// slices * tiles stays below 512 while the contraction is split, and is the tile count itself when it is not.
inline size_t down_part_tiles_bound(int rows, int r) {
    const size_t tiles = ((size_t)(rows + 63) / 64 + kMaxPositions - 1) * (size_t)((r + 63) / 64);
    return tiles > 512 ? tiles : 512;
}

struct MfmaPlan {
    int rows = 0, rows_pad = 0, rt = 0, n_rb = 0, gw = 0, nsr = 0, n_vt = 0;
    DownGrid down;
    size_t off_down_part = 0;            // fp32 [slices][n_rt][n_ct][4][16][64]: partial tiles of t (sized for any grouping of the rows)
    size_t off_t32 = 0;                  // fp32 [rows_pad, r]
    size_t off_t16 = 0;                  // 16-byte vectors [8 ceil(K / 64), rows_pad]: the head kernel's row operand
    size_t off_stat = 0;                 // float2 [2 ceil(r / 64), rows_pad]: per row and 32 columns of t, (sum of dt^2, sum of t dt), dt = t - rounded t
    size_t off_tilescale = 0;            // float2 [n_vt]: (column scale, mean square) of B per vocabulary tile
    size_t off_streams = 0;              // fp32 [rows, nsr, kStreamRec]
    size_t off_defer = 0;                // parked rows of the merge (long contractions only; bytes 0 otherwise)
    bool defer = false;
    size_t bytes = 0;
};

// rows here is the number of rows of ONE launch (at most kPlanSlotsPerXcd row blocks)
inline MfmaPlan make_mfma_plan(HeadKind kind, int rows, int d, int r, int V) {
    MfmaPlan p;
    p.rows = rows;
    p.rt = head_tile_rows_per_block(rows);
    p.n_rb = (rows + p.rt - 1) / p.rt;
    p.rows_pad = p.n_rb * p.rt;
    p.n_vt = (V + 255) / 256;
    int colgroups = (p.rt == 128 ? 2 : 1) * kPlanSlotsPerXcd / p.n_rb;      // 128-row blocks: two per CU
    if (colgroups < 1) colgroups = 1;
    const int need = (p.n_vt + 7) / 8;
    if (colgroups > need) colgroups = need;
    p.gw = 8 * colgroups;
    p.nsr = streams_per_block(p.gw) * p.gw;
    size_t off = 0;
    if (kind == HeadKind::LowRank) {
        p.off_t32 = off;       off = align_up(off + sizeof(float) * (size_t)p.rows_pad * r);
        p.off_t16 = off;       off = align_up(off + 2 * (size_t)p.rows_pad * ((r + 63) / 64 * 64));
        p.off_stat = off;      off = align_up(off + 2 * sizeof(float) * (size_t)p.rows_pad * 2 * ((r + 63) / 64));
        p.down = make_down_grid(rows, p.rows_pad, d, r);
        p.off_down_part = off; off = align_up(off + sizeof(float) * 4096 * down_part_tiles_bound(rows, r));
        p.off_tilescale = off; off = align_up(off + 2 * sizeof(float) * (size_t)p.n_vt);
    } else {
        p.off_t16 = off;       off = align_up(off + 2 * (size_t)p.rows_pad * ((d + 63) / 64 * 64));      // h regrouped for the kernel
    }
    p.off_streams = off;       off = align_up(off + sizeof(float) * (size_t)rows * p.nsr * kStreamRecPlan);
    p.defer = (kind == HeadKind::Full ? d : r) >= kDeferMinKFine;      // room for it; the call decides (merge_parks_rows)
    if (p.defer) { p.off_defer = off; off = align_up(off + merge_defer_bytes(rows)); }
    p.bytes = off;
    return p;
}
// Rows of one launch of the matrix-core kernels.  More rows per launch would leave fewer column blocks (gw), hence
// fewer stream records per row, and a row whose top-k crowd into one record pays an exact rescan of that record's
// columns: at 512 rows a row still has 128 column blocks, with four records each.
inline int mfma_max_rows_per_launch(int rows) { return rows > 512 ? 512 : rows; }
size_t merge_streams_lds_bytes(int nsr, int k, int n_vt);

}  // namespace slimspec

// Internal structures shared by the host scheduler and the device kernels of libbspmm.
// Not part of the public ABI (see include/bspmm.h for that).
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define BSPMM_HD __host__ __device__
#else
#define BSPMM_HD
#endif

namespace bspmm {

constexpr int kThreads = 256;      // lanes per workgroup (4 wavefronts of 64)
constexpr int kRanges = 5;         // launch ranges: 256 lanes, fused 256, then 64, 32, 16 lanes
constexpr int kMaxMembers = 8;     // operations one fused task may add up
constexpr int kMaxLdsBytes = 160 * 1024;    // LDS one workgroup can have on gfx950 (the whole CU's)
constexpr int kBuildLdsBytes = 64 * 1024;   // most the transpose / conversion kernels take
// The transpose / conversion kernels run one workgroup per operation: 256 lanes, or 1024 when
// the batch has an operation of more than a thousand entries (the launch lasts as long as its
// largest operation).  Operations of up to build_entries_per_lane(T) * T entries keep their
// entries in registers.
constexpr int kBuildThreadsLarge = 1024;
BSPMM_HD constexpr int build_entries_per_lane(int threads) { return threads == kThreads ? 4 : 5; }
constexpr int kHalfLdsBytes = 80 * 1024;    // half a CU's LDS (two workgroups per CU): default of the fused front

// Slot size (lanes) of launch range r, and its log2.
BSPMM_HD constexpr int range_log2_slot(int r) { return r <= 1 ? 8 : (r == 2 ? 6 : (r == 3 ? 5 : 4)); }

// One unit of work: the rows [row0, row0+nrows) of one operation restricted to the feature
// columns [f0, f0+fw).  64 bytes so one item is a single 64-byte fetch.
struct alignas(16) WorkItem {
    int64_t rpt_off;      // element offset of the operation's row pointers
    int64_t nz_off;       // element offset of the operation's entries
    int64_t in_row_off;   // first row of the dense input block
    int64_t out_row_off;  // first row of the dense output block
    int32_t m;            // output rows of the operation
    int32_t k;            // dense-input rows of the operation (columns of the sparse matrix)
    int32_t nnz;          // stored entries of the operation
    int32_t row0;         // first output row of this item
    int32_t nrows;        // output rows of this item (0 = empty item)
    int32_t f0;           // first feature column
    int32_t fw;           // feature columns
    int32_t staged;       // bit 0: operation and dense tile staged in LDS (0 = generic bin);
                          // bit 1: no other item reads this dense tile (stream it);
                          // bit 2: the item stands in for a set of summed operations and reads
                          // the set's merged CSR; bit 3 (fused front): dense tile in 32 x 32 blocks;
                          // fused tasks: bits 8-15 of the first member = number of members,
                          // bits 16-23 of member j = the member whose dense tile j shares
};
static_assert(sizeof(WorkItem) == 64, "WorkItem must be 64 bytes");

// The same unit of work for the lean kernel (launches made only of whole-workgroup items with a
// power-of-two tile): 32-bit offsets, and everything the host can derive - LDS placement, tile
// shape - already derived, so that a workgroup's scalar preamble is a handful of instructions.
// Two kinds: staged items (the operation and its dense tile in LDS) and row blocks of the
// generic bin (operations too large for LDS: the dense rows are gathered from L2).  For a row
// block the position of its entries is filled in on the device, once per plan, so that a run
// requests row pointers, entries and dense rows in ONE round trip instead of three.
struct alignas(16) LeanItem {
    uint32_t rpt_off;     // element offset of the operation's row pointers
    uint32_t nz_off;      // element offset of the operation's entries
    uint32_t in_row;      // first row of the dense input block
    uint32_t out_row;     // first row of the dense output block
    int32_t m, k, nnz;    // as WorkItem
    int32_t row0, nrows;  // output rows of this item
    int32_t f0;           // first feature column
    int32_t sh;           // log2 of the float4 per tile row (tile width = 4 << sh floats)
    int32_t flags;        // bit 0: no other item reads this dense tile; bit 1: row block of the
                          // generic bin
    int32_t cv_byte;      // staged: LDS byte offset of the (row offset, value) pairs
    int32_t b_byte;       // staged: LDS byte offset of the dense tile
    int32_t tile_vecs;    // staged: float4 in the tile, k << sh
                          // row block: its first entry, rpt[row0] (filled on the device)
    int32_t count;        // row block: its entries, rpt[row0 + nrows] - rpt[row0] (filled on the
                          // device)
};
static_assert(sizeof(LeanItem) == 64, "LeanItem must be 64 bytes");

// Kernel argument block, passed by value.  Task t belongs to range r when
// wg_end[r-1] <= t < wg_end[r]; its first item is item_base[r] + (t - wg_end[r-1]) * n(r) with
// n = 1 (range 0), fused_stride (range 1: operations summed into one output block), 4, 8, 16.
// The launch has min(n_tasks, resident workgroups) workgroups; workgroup w runs tasks
// w, w + gridDim.x, ...
struct LaunchParams {
    const WorkItem* items;
    const int32_t* rpt;
    const int32_t* colids;
    const float* values;
    const float* in;
    float* out;
    int64_t ld_in;
    int64_t ld_out;
    int32_t wg_end[kRanges];
    int32_t item_base[kRanges];
    int32_t n_tasks;      // == wg_end[kRanges-1]
    int32_t fused_stride; // item slots per fused task (fused-front launches: floats between the
                          // bias rows of the channels)
    int32_t lds_floats;   // LDS per workgroup, in 4-byte words
    int32_t pad;          // words added to every staged dense row
    // fused front of the graph-convolution layer (bspmm_run_gcn): `in` is then the layer input
    // X with n_front columns, and the dense tile is X_i . W + bias computed on chip
    const float* w;       // n_front x F weights; launches without a front: the merged CSR arrays
                          // of the summed sets of this direction (32-bit words)
    const float* bias;    // F floats
    int64_t ld_w;
    int32_t n_front;
    int32_t accumulate;   // add to the output instead of overwriting it
};

// Whole layers in launches of many rounds (bspmm_run_gcn, plans with front_features and
// BSPMM_ACCUMULATE): resident workgroups that keep their weight tile in registers and stream
// the graphs of their list through LDS.  One record per graph (a set of M channel operations
// with one merged CSR):
struct alignas(16) StreamSet {
    int64_t in_row;       // first row of X_i
    int64_t out_row;      // first row of Y_i
    uint32_t csr_off;     // word offset, from the base of the merged arrays, of the set's block:
                          // row pointers (m + 1, padded to 4), columns (nnz, padded to 4), values
    int32_t m;            // rows of Y_i (rows of every channel matrix)
    int32_t kx;           // rows of X_i (columns of every channel matrix)
    int32_t nnz;          // entries of the merged CSR
};
static_assert(sizeof(StreamSet) == 32, "StreamSet must be 32 bytes");

constexpr int kStreamPasses = 4;   // row passes of the gather a streamed graph may take: the
                                   // results of a graph wait in registers for one loop trip

// Arguments of the streaming kernel.  Every list l < lists has one workgroup per feature tile
// (columns [fw * tile, fw * tile + fw)), which takes the graphs list[l] .. list[l + 1]; the
// workgroups of a list sit on one XCD (see the kernel for the mapping; the grid is
// round_up(lists, 8) * tiles).
// LDS, in words: the dense tile (tile_words), two buffers for rows of X (x_words each), two
// for merged CSR blocks (csr_words each), 64 words that take the tile rows past a graph's end.
// (The pointers are kernel arguments of their own, qualified so that the graph records are
// fetched with scalar loads.)
struct StreamShape {
    int64_t ld_x, ld_w, ld_y, bias_stride;
    int32_t tiles, fw, channels, accumulate;
    int32_t tile_words, x_words, csr_words, big_csr_words;
    int32_t lists, compact, real_channels, reserved_;   // (channels >= real_channels are empty: see the host)
};
struct StreamParams {
    const StreamSet* sets;
    const int32_t* list;
    const int32_t* merged;
    const float* x;
    const float* w;
    const float* bias;
    float* y;
    StreamShape shape;
};

// One unit of work of the direct COO kernel: the output rows [row0, row0+nrows) x feature
// columns [f0, f0+fw) of one operation, computed from ALL of the operation's entries.
// LDS, in words, with stride = round_up(fw, 4): output tile nrows*stride, then (mode bit 0)
// the dense tile k*stride, then (mode bit 1) 2*nnz words of (output offset, input offset)
// pairs and nnz values.  Mode bit 2 (with bit 1): the entries of the item's rows are sorted by
// output row into LDS as (input offset, value) pairs (2*nnz words) and the rows summed in
// registers - no output tile; behind the pairs sit the row counts and the row pointers
// (nrows + 1 words each).
struct alignas(16) CooItem {
    int64_t nz_off;       // entry offset of the operation (its index pairs start at 2*nz_off)
    int64_t in_row_off;   // first row of the dense input block
    int64_t out_row_off;  // first row of the dense output block
    int32_t nnz;          // stored entries of the operation
    int32_t k;            // rows of the dense input block (bound of the gathered index)
    int32_t row0;
    int32_t nrows;
    int32_t f0;
    int32_t fw;
    int32_t op;
    int32_t mode;         // bit 0: the dense tile (k rows) is staged in LDS behind the output
                          // tile; bit 1: the entries are staged in LDS behind that; bit 2: the
                          // entries are sorted by row into LDS, no output tile
    int32_t pad_[2];
};
static_assert(sizeof(CooItem) == 64, "CooItem must be 64 bytes");

struct CooLaunchParams {
    const CooItem* items;
    const int32_t* ids;   // (row, column) pairs
    const float* values;
    const float* in;
    float* out;
    int64_t ld_in;
    int64_t ld_out;
    int32_t transposed;   // 0: output row = pair[0], gathered row = pair[1]; 1: swapped
};

// Per-operation record of the transposed-CSR build and of the validation kernel.
struct alignas(8) OpRecord {
    int64_t rpt_off;
    int64_t nz_off;
    int64_t rpt_t_off;     // element offset of the transposed row pointers
    int64_t nz_t_off;      // element offset of the transposed entries
    int64_t scratch_off;   // element offset into the global scratch, or -1 to use LDS
    int32_t m;
    int32_t k;
    int32_t nnz;
    int32_t small;         // 1: the build kernel may take its register path (see there)
};

BSPMM_HD inline int round_up(int x, int a) { return (x + a - 1) / a * a; }

// LDS words of a direct COO item (see CooItem).
BSPMM_HD inline int64_t coo_lds_words(int nrows, int k, int nnz, int fw, int mode)
{
    const int64_t stride = round_up(fw, 4);
    if (mode & 4)   // entries sorted by row in LDS, sums in registers: no output tile
        return ((mode & 1) ? (int64_t)k * stride : 0) + 2 * (int64_t)nnz + 2 * (int64_t)nrows + 4;
    return (int64_t)nrows * stride + ((mode & 1) ? (int64_t)k * stride : 0) +
           ((mode & 2) ? 3 * (int64_t)nnz + 1 : 0);
}

BSPMM_HD inline int pow2_ceil(int x)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return x <= 1 ? 1 : 1 << (32 - __builtin_clz((unsigned)(x - 1)));     // no loop on the device
#else
    int p = 1;
    while (p < x) p <<= 1;
    return p;
#endif
}

// LDS layout of a staged item, in 4-byte words from the start of its slot:
//   [0, m+1)                      row pointers (clamped to nnz)
//   [cv_off, cv_off + 2*nnz)      (column * stride, value) pairs: the word offset of the entry's
//                                 dense row inside the tile, and its value
//   [b_off, b_off + k*stride)     dense tile, row stride `stride`
//   [hub_off, total)              workgroup items only: hub-row list and reduction scratch
struct StagedLayout {
    int cv_off;
    int b_off;
    int stride;
    int hub_off;
    int total;
};

// A row is a hub when it has at least kHubMin entries and at least kHubRatio times the
// average of its operation; its entries are then split across all lane groups.
constexpr int kHubMin = 64;
constexpr int kHubRatio = 4;

// Words of the hub area: a counter, one slot per possible hub row, and one tile row per
// wavefront for the cross-wavefront sum (16-byte aligned).
BSPMM_HD inline int hub_words(int max_hubs, int fw)
{
    return round_up(1 + max_hubs, 4) + (kThreads / 64) * round_up(fw, 4);
}

BSPMM_HD inline StagedLayout staged_layout(int m, int k, int nnz, int fw, int pad, bool hub)
{
    StagedLayout L;
    L.cv_off = round_up(m + 1, 2);
    L.b_off = round_up(L.cv_off + 2 * nnz, 4);
    L.stride = round_up(fw, 4) + pad;
    L.hub_off = L.b_off + k * L.stride;
    L.total = L.hub_off + (hub ? hub_words(nnz / kHubMin, fw) : 0);
    return L;
}

// Operations that are summed into one output block ("a set") run from a merged CSR that a device
// kernel builds once per plan and direction: row r of the set is row r of every member, one
// after the other in member order, and an entry names a row of the members' dense tiles laid
// end to end (members that read the same dense block share one tile).  Per set, in the
// workspace: round_up(m+1, 4) row pointers, then round_up(sum nnz, 2) entries of two words
// (tile row, value); 2*round_up(sum nnz, 4) words are reserved for them.
//
// LDS layout of a fused task, in words:
//   [0, rs)                            merged row pointers, rs = round_up(m+1, 4)
//   [rs, rs + 2*round_up(sum nnz, 2))  merged entries
//   then per distinct dense input      its tile, k rows of round_up(fw, 4) words
struct FusedLayout {
    int rs;
    int entry_words;
    int tile_off;
};

BSPMM_HD inline FusedLayout fused_layout(int m, int nnz_sum)
{
    FusedLayout L;
    L.rs = round_up(m + 1, 4);
    L.entry_words = 2 * round_up(nnz_sum, 2);
    L.tile_off = L.rs + L.entry_words;
    return L;
}

// What the kernel that merges a set needs (one record per set and direction).
struct alignas(8) SetRecord {
    int64_t rpt_off[kMaxMembers];   // the members' row pointers and entries in the CSR arrays
    int64_t nz_off[kMaxMembers];
    int64_t merged_rpt_off;         // word offsets of the set's merged arrays
    int64_t merged_nz_off;
    int32_t nnz[kMaxMembers];
    int32_t k[kMaxMembers];         // dense-input rows of the members (bound of their columns)
    int32_t tile_row[kMaxMembers];  // first row of member j's dense tile in the concatenation
    int32_t row_off[kMaxMembers];   // the set's row that is member j's row 0, and member j's rows
    int32_t rows[kMaxMembers];      // (summed sets: 0 and m for every member; groups of graphs in
                                    // the streaming launch: each graph's members have their own)
    int32_t members;
    int32_t m;
    int32_t plain;                  // 1: the members read one dense block; the merged arrays are
                                    // then an ordinary CSR (row pointers, round_up(sum nnz, 4)
                                    // columns, as many values) that a plain item reads
    int32_t compact;                // 0, or channels | rows of the group's layer input << 8: the
                                    // rows of each channel's dense tile that are in use are
                                    // listed behind the values and the columns renumbered
};

// Words behind the values of a compacted set: counts and first tile rows of the channels
// (padded to four each), then a list of kxt words per channel.
BSPMM_HD inline int compact_words(int chans, int kxt)
{
    return chans > 0 ? round_up(2 * round_up(chans, 4) + chans * kxt, 4) : 0;
}
constexpr int kCompactRows = 1024;   // tile rows (channels x rows of X) of a set that is compacted, at most

// Lanes that share one output row: enough 4-float vectors to cover the tile, a power of two.
BSPMM_HD inline int lanes_per_row(int fw, int vec)
{
    int g = pow2_ceil((fw + vec - 1) / vec);
    return g > 64 ? 64 : g;
}

}  // namespace bspmm

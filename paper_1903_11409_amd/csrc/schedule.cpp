// Batch scheduler (host only).
//
// The paper's Batched SpMM for CSR (Sec. IV-C) sizes one launch from the batch maximum:
// max m_A * subWarp * batch [* p] threads, column blocking for all operations if any needs it,
// surplus threads exit.  Here every operation is scheduled from its own size instead:
//   * the feature dimension is cut into tiles (the column blocking of Fig. 5(d)); the
//     batch-wide tile is the widest one that still yields enough workgroups to fill the chip,
//     and an operation whose dense tile does not fit its LDS share gets narrower tiles;
//   * an (operation, tile) item runs on a 16/32-lane slice, a wavefront or a workgroup,
//     whichever is the smallest that finishes its rows in a few passes and holds its operands
//     in the slot's share of LDS; operations too large for LDS at the narrowest tile fall to
//     the generic bin, cut into row blocks that read global memory;
//   * work is ordered largest-first; items that read the same dense tile (row blocks of a
//     large operation, channels of one graph) are kept on one XCD, i.e. on workgroup indices
//     that are equal modulo 8, so the tile is fetched into one L2 only.
#include "schedule.hpp"

#include <algorithm>
#include <cstdint>
#include <map>
#include <numeric>
#include <utility>

namespace bspmm {

namespace {

constexpr int kXcds = 8;
constexpr int kFrontBlocks = 8;   // matrix-core blocks one workgroup of the fused front should make

struct Draft {           // one item before placement
    int op;
    int bin;
    int row0, nrows, f0, fw;
    int staged;
    int64_t cost;
    int group;           // items with one group read the same dense tile
    int fused;           // >= 0: index of the set of operations this task adds up
};

int bin_slot_lanes(int bin)
{
    switch (bin) {
        case BSPMM_BIN_WAVE: return 64;
        case BSPMM_BIN_SLICE32: return 32;
        case BSPMM_BIN_SLICE16: return 16;
        default: return kThreads;
    }
}

int bin_range(int bin)
{
    switch (bin) {
        case BSPMM_BIN_WAVE: return 2;
        case BSPMM_BIN_SLICE32: return 3;
        case BSPMM_BIN_SLICE16: return 4;
        default: return 0;
    }
}

int draft_range(const Draft& x) { return x.fused >= 0 ? 1 : bin_range(x.bin); }

// Candidate tile widths, widest first.
std::vector<int> tile_candidates(int F, const Knobs& kn)
{
    std::vector<int> c;
    int t = std::min(F, kn.max_tile);
    c.push_back(t);
    int p = 1;
    while (p * 2 < t) p *= 2;        // largest power of two below t
    if (p == t) p /= 2;
    for (; p >= kn.min_tile && p >= 4; p /= 2) c.push_back(p);
    return c;
}

struct Choice {
    int bin;
    int tile;
};

bool fits_slot(const DirOps& o, int i, int tile, int F, int vec, int lanes, int max_passes,
               const Knobs& kn)
{
    const int fw = std::min(tile, F);
    const int g = lanes_per_row(fw, vec);
    if (g > lanes) return false;
    const int64_t lanes_wanted = (int64_t)o.m[i] * g;
    if (max_passes > 0 && (lanes_wanted + lanes - 1) / lanes > max_passes) return false;
    const int64_t head = (int64_t)round_up(o.m[i] + 1, 2) + 2 * (int64_t)o.nnz[i];
    int64_t need = (head + 3) / 4 * 4 + (int64_t)o.k[i] * (round_up(fw, 4) + kn.pad);
    if (kn.hubs && lanes == kThreads) need += hub_words(o.nnz[i] / kHubMin, fw);   // as staged_layout()
    if (kn.front > 0)   // a weight tile and a bias tile per channel and at least 16 rows of X_i ride along
        need += 16 * (int64_t)kn.front +
                o.channels(i) * ((int64_t)kn.front * round_up(fw, 4) + round_up(fw, 4));
    return need <= (int64_t)kn.lds_words * lanes / kThreads;
}

// Decide bin and tile of operation i given the batch-wide tile candidates from `first` on.
// `widest_fit` (optional): per operation, the index of the widest candidate whose whole-workgroup
// item fits LDS (cand.size() when none does).  Fitting is monotone in the tile width, so with it
// the plain case - no forced bin, no sub-workgroup slots - is answered without looking at the
// operation again, however often the search over tiles and row cuts asks.
Choice choose(const DirOps& o, int i, int F, int vec, const std::vector<int>& cand, size_t first,
              const Knobs& kn, bool allow_small, const std::vector<uint8_t>* widest_fit = nullptr)
{
    const int forced = kn.front > 0 ? BSPMM_BIN_WORKGROUP : kn.force_bin;   // the fused front runs on whole workgroups
    if (widest_fit && forced < 0 && !allow_small) {
        const size_t c = std::max<size_t>(first, (*widest_fit)[i]);
        return c < cand.size() ? Choice{BSPMM_BIN_WORKGROUP, cand[c]} : Choice{BSPMM_BIN_GENERIC, cand[0]};
    }
    if (forced == BSPMM_BIN_GENERIC) return {BSPMM_BIN_GENERIC, cand[0]};
    if (forced >= 0) {
        for (size_t c = first; c < cand.size(); ++c) {
            // fused front: a workgroup makes its whole dense tile on the matrix cores before it
            // can gather, and the launch lasts as long as its slowest workgroup, so a larger
            // operation takes a narrower tile (at most kFrontBlocks 16 x 16 blocks each)
            if (kn.front > 0 && c + 1 < cand.size() &&
                ((o.k[i] + 15) / 16) * ((std::min(cand[c], F) + 15) / 16) > kFrontBlocks)
                continue;
            if (fits_slot(o, i, cand[c], F, vec, bin_slot_lanes(forced), 0, kn))
                return {forced, cand[c]};
        }
    }
    const int tile = cand[first];
    static const int small_bins[3] = {BSPMM_BIN_SLICE16, BSPMM_BIN_SLICE32, BSPMM_BIN_WAVE};
    for (int b : small_bins)
        if (allow_small && fits_slot(o, i, tile, F, vec, bin_slot_lanes(b), kn.max_passes, kn))
            return {b, tile};
    for (size_t c = first; c < cand.size(); ++c)
        if (fits_slot(o, i, cand[c], F, vec, kThreads, 0, kn))
            return {BSPMM_BIN_WORKGROUP, cand[c]};
    return {BSPMM_BIN_GENERIC, cand[0]};
}

int64_t item_cost(const DirOps& o, int i, int nrows, int fw, bool staged)
{
    const int64_t dense_in = staged ? o.k[i] : std::min<int64_t>(o.k[i], (int64_t)nrows * 4);
    return 4 * (int64_t)fw * (dense_in + nrows) + 8 * (int64_t)o.nnz[i] * nrows / std::max(o.m[i], 1) +
           4 * (int64_t)nrows + 512;
}

// Where drafted items go.  Sizing the launch only needs to know how many items each launch
// range would get, so the search over tiles and row cuts runs on a sink that counts; the one
// draft that is kept is built with a sink that stores the items.
struct Sink {
    std::vector<Draft>* out = nullptr;     // null: count only
    int per_range[kRanges] = {0, 0, 0, 0, 0};
    int generic = 0;                       // items that read their operands from global memory
    int64_t tile_words = 0;                // counting only: dense-tile words the staged items copy
    const std::vector<int>* block_of_op = nullptr;   // dense-input block index of every operation
    int tiles_per_block = 1;               // group id = block * tiles_per_block + f0 / tile_unit
    int tile_unit = 4;
    void add(const DirOps& o, int i, int bin, int row0, int nrows, int f0, int fw, int staged,
             int fused)
    {
        per_range[fused >= 0 ? 1 : bin_range(bin)]++;
        generic += bin == BSPMM_BIN_GENERIC;
        if (!out) return;
        const int gid = fused >= 0 ? -1 : (*block_of_op)[i] * tiles_per_block + f0 / tile_unit;
        out->push_back({i, bin, row0, nrows, f0, fw, staged,
                        fused >= 0 ? 0 : item_cost(o, i, nrows, fw, staged != 0), gid, fused});
    }
    int workgroups() const
    {
        int wgs = per_range[0] + per_range[1];
        for (int r = 2; r < kRanges; ++r) {
            const int slots = kThreads >> range_log2_slot(r);
            wgs += (per_range[r] + slots - 1) / slots;
        }
        return wgs;
    }
};

// `cap` > 0 cuts a workgroup item into row ranges of at most `cap` passes each (every range
// stages the whole operation, so the cut costs on-chip traffic and buys parallelism).
void draft_op(const DirOps& o, int i, int F, int vec, const Choice& ch, const Knobs& kn, int cap,
              Sink& sink)
{
    if (o.m[i] <= 0) return;
    const int tile = ch.tile;
    if (!sink.out) {    // counting: the same items in closed form
        auto per_tile = [&](int fw) {
            if (ch.bin == BSPMM_BIN_WORKGROUP && cap > 0) {
                const int chunk = cap * (kThreads / lanes_per_row(fw, vec));
                return (o.m[i] + chunk - 1) / chunk;
            }
            if (ch.bin != BSPMM_BIN_GENERIC) return 1;
            return (o.m[i] + kn.generic_rows - 1) / kn.generic_rows;
        };
        const int full = F / tile, tail = F % tile;
        const int n_full = full ? per_tile(tile) : 0, n_tail = tail ? per_tile(tail) : 0;
        const int n = full * n_full + n_tail;
        sink.per_range[bin_range(ch.bin)] += n;
        sink.generic += ch.bin == BSPMM_BIN_GENERIC ? n : 0;
        if (ch.bin != BSPMM_BIN_GENERIC)   // every piece of a cut item copies the whole tile
            sink.tile_words += (int64_t)o.k[i] * ((int64_t)full * n_full * tile + (int64_t)n_tail * tail);
        return;
    }
    for (int f0 = 0; f0 < F; f0 += tile) {
        const int fw = std::min(tile, F - f0);
        if (ch.bin == BSPMM_BIN_WORKGROUP && cap > 0) {
            const int rows_per_pass = kThreads / lanes_per_row(fw, vec);
            const int chunk = cap * rows_per_pass;
            for (int r0 = 0; r0 < o.m[i]; r0 += chunk)
                sink.add(o, i, ch.bin, r0, std::min(chunk, o.m[i] - r0), f0, fw, 1, -1);
        } else if (ch.bin != BSPMM_BIN_GENERIC) {
            sink.add(o, i, ch.bin, 0, o.m[i], f0, fw, 1, -1);
        } else {
            for (int r0 = 0; r0 < o.m[i]; r0 += kn.generic_rows)
                sink.add(o, i, ch.bin, r0, std::min(kn.generic_rows, o.m[i] - r0), f0, fw, 0, -1);
        }
    }
}

// LDS words a fused task needs: mirrors run_fused() in kernels.hip.
int64_t fused_words(const DirOps& o, const std::vector<int>& members, int fw)
{
    int64_t nnz_sum = 0;
    for (int i : members) nnz_sum += o.nnz[i];
    int64_t words = round_up(o.m[members[0]] + 1, 4) + 2 * ((nnz_sum + 1) / 2 * 2);
    for (size_t j = 0; j < members.size(); ++j) {
        bool owns = true;
        for (size_t e = 0; e < j; ++e)   // (the same block: same first row AND same row count)
            owns = owns && !(o.in_off[members[e]] == o.in_off[members[j]] && o.k[members[e]] == o.k[members[j]]);
        if (owns) words += (int64_t)o.k[members[j]] * round_up(fw, 4);
    }
    return words;
}

// Tasks of one set of operations that are summed into one output block.  The tile is the
// widest candidate (from `first` on, then 16, 8 and 4 floats) whose task fits LDS; returns false
// when none does.
bool draft_fused(const DirOps& o, const std::vector<int>& members, int fused_index, int F, int vec,
                 const std::vector<int>& cand, size_t first, const Knobs& kn, int cap,
                 Sink& sink)
{
    std::vector<int> tiles(cand.begin() + first, cand.end());
    for (int t : {16, 8, 4})
        if (t < tiles.back()) tiles.push_back(t);
    int tile = 0;
    for (int t : tiles)
        if (fused_words(o, members, std::min(t, F)) <= kn.lds_words) {
            tile = t;
            break;
        }
    if (!tile) return false;
    const int m = o.m[members[0]];
    for (int f0 = 0; f0 < F; f0 += tile) {
        const int fw = std::min(tile, F - f0);
        const int rows_per_pass = kThreads / lanes_per_row(fw, vec);
        const int chunk = cap > 0 ? cap * rows_per_pass : m;
        for (int r0 = 0; r0 < m; r0 += chunk) {
            const int nr = std::min(chunk, m - r0);
            sink.add(o, members[0], BSPMM_BIN_WORKGROUP, r0, nr, f0, fw, 1, fused_index);
            if (sink.out) {
                int64_t cost = 0;
                for (int i : members) cost += item_cost(o, i, nr, fw, true);
                sink.out->back().cost = cost;
            }
        }
    }
    return true;
}

// Operations grouped by the output block they name: a group of more than one is summed.
// Groups are listed in the order of their first operation, members in operation order; group g
// is member[start[g]] .. member[start[g + 1] - 1].
struct Groups {
    std::vector<int> start, member;
    int size() const { return (int)start.size() - 1; }
    int count(int g) const { return start[g + 1] - start[g]; }
    const int* begin(int g) const { return member.data() + start[g]; }
    std::vector<int> members(int g) const { return std::vector<int>(begin(g), begin(g) + count(g)); }
};

Groups output_groups(const DirOps& o)
{
    Groups out;
    const int n = o.size();
    out.member.reserve(n);
    out.start.reserve(n + 1);
    // the usual case: every operation has an output block of its own, later operations at
    // higher rows - nothing to sort
    bool separate = true;
    int64_t end = -1;
    for (int i = 0; i < n && separate; ++i) {
        if (o.m[i] <= 0) continue;
        separate = o.out_off[i] >= end;
        end = o.out_off[i] + o.m[i];
    }
    if (separate) {
        for (int i = 0; i < n; ++i)
            if (o.m[i] > 0) {
                out.start.push_back((int)out.member.size());
                out.member.push_back(i);
            }
        out.start.push_back((int)out.member.size());
        return out;
    }
    std::vector<int> idx;
    idx.reserve(n);
    for (int i = 0; i < n; ++i)
        if (o.m[i] > 0) idx.push_back(i);
    std::vector<int> sorted = idx;
    std::sort(sorted.begin(), sorted.end(), [&](int a, int b) {
        if (o.out_off[a] != o.out_off[b]) return o.out_off[a] < o.out_off[b];
        if (o.m[a] != o.m[b]) return o.m[a] < o.m[b];
        return a < b;
    });
    // leader[i] = first operation (lowest index) naming the same block as i; size[l] = members
    std::vector<int> leader(n, -1), size(n, 0);
    for (size_t a = 0; a < sorted.size();) {
        size_t b = a;
        while (b < sorted.size() && o.out_off[sorted[b]] == o.out_off[sorted[a]] &&
               o.m[sorted[b]] == o.m[sorted[a]])
            leader[sorted[b++]] = sorted[a];
        size[sorted[a]] = (int)(b - a);
        a = b;
    }
    // groups in the order of their leaders; a group's slots are filled in operation order
    std::vector<int> at(n, -1);
    int total = 0;
    for (int i : idx)
        if (leader[i] == i) {
            out.start.push_back(total);
            at[i] = total;
            total += size[i];
        }
    out.start.push_back(total);
    out.member.resize(total);
    for (int i : idx) out.member[at[leader[i]]++] = i;
    return out;
}

// Index of the dense-input block of every operation (operations reading the same first row
// share an index).
std::vector<int> input_blocks(const DirOps& o)
{
    std::vector<int> order(o.size());
    std::iota(order.begin(), order.end(), 0);
    std::sort(order.begin(), order.end(),
              [&](int a, int b) { return o.in_off[a] != o.in_off[b] ? o.in_off[a] < o.in_off[b] : a < b; });
    std::vector<int> block(o.size(), 0);
    int nb = -1;
    for (size_t t = 0; t < order.size(); ++t) {
        if (t == 0 || o.in_off[order[t]] != o.in_off[order[t - 1]]) ++nb;
        block[order[t]] = nb;
    }
    return block;
}

// Narrowest tile a stand-in may take: the narrowest batch-wide candidate, or half of it when
// only that fits (the members' tiles side by side are several times an operation's tile; 0 when
// neither fits).
int stand_in_tile(const DirOps& o, int v, int F, int vec, const std::vector<int>& cand, const Knobs& kn)
{
    if (fits_slot(o, v, cand.back(), F, vec, kThreads, 0, kn)) return cand.back();
    const int half = cand.back() / 2;
    if (half >= 16 && half % 4 == 0 && fits_slot(o, v, half, F, vec, kThreads, 0, kn)) return half;
    return 0;
}

// `stand_in[g]` >= 0: the operations of group g all read one dense block, so their sum is the
// product with the sum of their matrices: one operation (appended to `o` at that index, its CSR
// the set's merged one) stands in for them and is drafted as a workgroup item like any other.
void draft_all(const DirOps& o, int F, int vec, const std::vector<int>& cand, size_t first,
               const Knobs& kn, int cap, bool allow_small,
               const Groups& outs, const std::vector<int>& stand_in, bool* fits, Sink& sink,
               const std::vector<uint8_t>* widest_fit = nullptr)
{
    int nfused = 0;
    for (int g = 0; g < outs.size(); ++g) {
        if (outs.count(g) == 1) {
            const int i = *outs.begin(g);
            draft_op(o, i, F, vec, choose(o, i, F, vec, cand, first, kn, allow_small, widest_fit), kn, cap, sink);
        } else if (stand_in[g] >= 0) {
            const int v = stand_in[g];
            Choice ch = {BSPMM_BIN_WORKGROUP, stand_in_tile(o, v, F, vec, cand, kn)};
            for (size_t c = first; c < cand.size(); ++c)
                if (fits_slot(o, v, cand[c], F, vec, kThreads, 0, kn)) {
                    ch.tile = cand[c];
                    break;
                }
            draft_op(o, v, F, vec, ch, kn, cap, sink);
        } else if (!draft_fused(o, outs.members(g), nfused++, F, vec, cand, first, kn, cap, sink)) {
            *fits = false;
        }
    }
}

WorkItem to_item(const DirOps& o, const Draft& x)
{
    WorkItem w;
    w.rpt_off = o.rpt_off[x.op];
    w.nz_off = o.nz_off[x.op];
    w.in_row_off = o.in_off[x.op];
    w.out_row_off = o.out_off[x.op];
    w.m = o.m[x.op];
    w.k = o.k[x.op];
    w.nnz = o.nnz[x.op];
    w.row0 = x.row0;
    w.nrows = x.nrows;
    w.f0 = x.f0;
    w.fw = x.fw;
    w.staged = x.staged;
    return w;
}

WorkItem empty_item()
{
    WorkItem w;
    w.rpt_off = w.nz_off = w.in_row_off = w.out_row_off = 0;
    w.m = w.k = w.nnz = w.row0 = w.nrows = w.f0 = w.fw = 0;
    w.staged = 1;
    return w;
}

}  // namespace

// Workgroups per CU a launch aims for.  Plain products: four (their time is latency).  The
// fused front stages X_i again for every feature tile, so it wants fewer, wider tiles the
// wider the layer input is: two per CU measured best up to 64 input columns, one from 128 on.
int workgroups_per_cu(int front)
{
    return front <= 0 ? 4 : (front < 128 ? 2 : 1);
}

Knobs resolve_knobs(const bspmm_options* o)
{
    Knobs k;
    if (!o) return k;
    if (o->force_bin > 0 && o->force_bin <= BSPMM_NUM_BINS) k.force_bin = o->force_bin - 1;
    if (o->lds_bytes > 0) k.lds_words = std::min(o->lds_bytes, kMaxLdsBytes) / 256 * 64;
    if (k.lds_words < 256) k.lds_words = 256;
    if (o->max_tile > 0) k.max_tile = std::min(std::max(o->max_tile, 4), 256) / 4 * 4;
    if (o->min_tile > 0) k.min_tile = std::min(std::max(o->min_tile, 4), k.max_tile);
    if (o->compute_units > 0) k.compute_units = o->compute_units;
    k.target_given = o->target_workgroups > 0;
    k.target_wgs = o->target_workgroups > 0 ? o->target_workgroups
                                            : workgroups_per_cu(o->front_features) * k.compute_units;
    if (o->lds_pad > 0) k.pad = std::min(o->lds_pad, 64) / 4 * 4;
    if (o->lds_pad < 0) k.pad = 0;
    if (o->max_passes > 0) k.max_passes = o->max_passes;
    if (o->generic_rows > 0) k.generic_rows = o->generic_rows;
    k.wg_passes = o->wg_passes;
    if (o->resident_workgroups > 0) k.persistent_wgs = o->resident_workgroups;
    k.hubs = (o->flags & BSPMM_SPLIT_HUB_ROWS) != 0;
    k.accumulate = (o->flags & BSPMM_ACCUMULATE) != 0;
    k.coo_direct = (o->flags & BSPMM_COO_DIRECT) != 0;
    k.symmetric = (o->flags & BSPMM_SYMMETRIC) != 0;
    k.one_front_launch = (o->flags & BSPMM_ONE_FRONT_LAUNCH) != 0;
    k.lds_given = o->lds_bytes > 0;
    if (o->front_features > 0) {   // the matrix-core blocks of the fused front are 16 columns wide
        k.front = o->front_features;
        // an item also holds X_i and a weight tile: take half the CU's LDS unless told otherwise
        // (the launch asks only for what its largest item needs)
        if (o->lds_bytes <= 0) k.lds_words = kHalfLdsBytes / 4;
        k.max_tile = std::max(16, k.max_tile / 16 * 16);
        k.min_tile = o->min_tile > 0 ? std::min(std::max(16, (k.min_tile + 15) / 16 * 16), k.max_tile) : 16;
    }
    return k;
}

Schedule make_schedule(const DirOps& ops_in, int F, const Knobs& kn_in)
{
    Schedule s;
    Knobs kn = kn_in;
    if (!kn_in.target_wgs) kn.target_wgs = 4 * kn.compute_units;
    const int vec = (F % 4 == 0) ? 4 : 1;
    const std::vector<int> cand = tile_candidates(F, kn);
    const Groups outs = output_groups(ops_in);

    // Sets of summed operations whose dense blocks are one block (the same one, or blocks that
    // lie back to back in the packed input): an operation with the members' matrices side by
    // side stands in for the set when it fits a staged workgroup item at the narrowest tile.
    DirOps ext;
    std::vector<int> stand_in(outs.size(), -1);
    {
        bool copied = false;
        for (int g = 0; g < outs.size(); ++g) {
            const int cnt = outs.count(g);
            if (cnt < 2 || cnt > kMaxMembers || kn.force_bin == BSPMM_BIN_GENERIC) continue;
            const int* mem = outs.begin(g);
            // the members' dense blocks, each counted once in member order, must lie back to
            // back: laid end to end they are then one block of the packed input as it stands
            bool one_block = true;
            int64_t nnz = 0, rows = 0;
            for (int j = 0; j < cnt; ++j) {
                nnz += ops_in.nnz[mem[j]];
                bool seen = false;
                for (int e = 0; e < j && !seen; ++e)
                    seen = ops_in.in_off[mem[e]] == ops_in.in_off[mem[j]] && ops_in.k[mem[e]] == ops_in.k[mem[j]];
                if (kn.front > 0) {
                    // fused front: the channels of a set share the layer input X_i, and each
                    // makes a dense tile of its own from it (X_i W[ch] + bias[ch]) on chip:
                    // the tiles are side by side by construction
                    one_block = one_block && (j == 0 || seen);
                    rows += ops_in.k[mem[j]];
                    continue;
                }
                if (seen) continue;
                one_block = one_block && ops_in.in_off[mem[j]] == ops_in.in_off[mem[0]] + rows;
                rows += ops_in.k[mem[j]];
            }
            if (!one_block || nnz > INT32_MAX || rows > INT32_MAX) continue;
            if (!copied) {
                ext = ops_in;
                copied = true;
            }
            const int v = ext.size();
            ext.m.push_back(ops_in.m[mem[0]]);
            ext.k.push_back((int32_t)rows);
            ext.nnz.push_back((int32_t)nnz);
            ext.rpt_off.push_back(0);       // the merged arrays are placed by the caller
            ext.nz_off.push_back(0);
            ext.in_off.push_back(ops_in.in_off[mem[0]]);
            ext.out_off.push_back(ops_in.out_off[mem[0]]);
            if (kn.front > 0) {
                ext.chan.resize(ext.size(), 1);
                ext.chan.back() = cnt;
            }
            if (stand_in_tile(ext, v, F, vec, cand, kn) > 0) {
                stand_in[g] = v;
                s.merged_sets.push_back(outs.members(g));
            } else {   // take it back: the set runs as a fused task (or does not fit at all)
                ext.m.pop_back(), ext.k.pop_back(), ext.nnz.pop_back(), ext.rpt_off.pop_back();
                ext.nz_off.pop_back(), ext.in_off.pop_back(), ext.out_off.pop_back();
                if (!ext.chan.empty()) ext.chan.pop_back();
            }
        }
    }
    s.first_stand_in = ops_in.size();
    // the whole layer per item: M channels make M times the matrix-core work of a plain front
    // item, so the launch wants M times the workgroups (128 graphs of 4 channels, n_X = 64:
    // 15.5 us at 512 workgroups, 11.7 us at 1024)
    if (kn.front > 0 && !s.merged_sets.empty() && !kn.target_given)
        kn.target_wgs *= (int)s.merged_sets[0].size();
    const DirOps& ops = s.merged_sets.empty() ? ops_in : ext;

    // widest batch-wide tile that still gives the launch enough workgroups
    std::vector<Draft> d;
    size_t chosen = cand.size() - 1;
    // Sub-workgroup slots pack several small items into one workgroup.  Measured on MI355X
    // that only pays when the launch is over-subscribed (more workgroups than the chip holds
    // at once); a launch that fits is latency-bound and every item is fastest with a whole
    // workgroup staging it.  A forced bin overrides this.
    const int fixed_cap = kn.wg_passes > 0 ? kn.wg_passes : 0;
    bool allow_small = kn.force_bin >= 0 && kn.front == 0;
    size_t most_members = 1;
    for (int g = 0; g < outs.size(); ++g) most_members = std::max<size_t>(most_members, outs.count(g));
    if (most_members > (size_t)kMaxMembers) {
        s.error = BSPMM_ETOOBIG;
        return s;
    }
    bool fits = true;
    int64_t counted_tile_words = 0;
    std::vector<uint8_t> widest_fit(ops.size(), (uint8_t)std::min<size_t>(cand.size(), 255));
    if (kn.front == 0 && kn.force_bin < 0 && cand.size() < 255)
        for (int i = 0; i < ops.size(); ++i)
            for (size_t c = 0; c < cand.size(); ++c)
                if (fits_slot(ops, i, cand[c], F, vec, kThreads, 0, kn)) {
                    widest_fit[i] = (uint8_t)c;
                    break;
                }
    const std::vector<uint8_t>* fit_table = kn.front == 0 && kn.force_bin < 0 && cand.size() < 255 ? &widest_fit : nullptr;
    auto workgroups_of = [&](size_t first, int cap, bool small) {
        Sink counter;
        draft_all(ops, F, vec, cand, first, kn, cap, small, outs, stand_in, &fits, counter, fit_table);
        counted_tile_words = counter.tile_words;
        return counter.workgroups();
    };
    int wgs = 0;
    for (int attempt = 0; attempt < 2; ++attempt) {
        for (size_t c = 0; c < cand.size(); ++c) {
            wgs = workgroups_of(c, fixed_cap, allow_small);
            if (wgs >= kn.target_wgs || c + 1 == cand.size()) {
                chosen = c;
                break;
            }
        }
        if (allow_small || wgs <= kn.capacity_wgs || kn.front > 0) break;
        allow_small = true;
    }
    s.tile = cand[chosen];
    // still too few workgroups at the narrowest tile: the batch is small, its time is set by
    // the slowest workgroup, so cut multi-pass workgroup items into row ranges
    // Likewise while the launch still fits the chip at once: the workgroups with several passes
    // are its critical path, and cutting them pays as long as no workgroup has to wait for a
    // free slot and the pieces, each of which copies the whole dense tile again, do not add
    // more than 60 % to the tile traffic (measured: 256 molecule graphs 4.9 -> 4.3 us, 512
    // graphs 5.9 -> 4.8 us; cut beyond what the chip holds, 384 graphs go from 4.9 to 5.9 us;
    // wide tiles of 100-row graphs cut to four rows each, 8.2 -> 9.2 us).
    int cap = fixed_cap;
    if (kn.wg_passes == 0 && kn.front == 0) {
        const int uncut = wgs;                         // (the tile search ended on this very count)
        const int64_t uncut_words = counted_tile_words;
        bool done = false;
        // (a launch that moves more than about 28 MB is bound by bandwidth, not by its slowest
        // workgroup: there the extra copies only cost)
        const bool latency_bound = uncut_words <= 3500000;
        for (int c = 1; c <= 4 && uncut <= kn.capacity_wgs && latency_bound; c *= 2) {
            const int w = workgroups_of(chosen, c, allow_small);
            if (w <= kn.capacity_wgs && 5 * (counted_tile_words - uncut_words) <= 3 * uncut_words) {
                cap = c;
                wgs = w;
                done = true;
                break;
            }
        }
        if (!done && uncut < kn.target_wgs) {
            for (cap = 4; cap >= 1; cap /= 2) {
                wgs = workgroups_of(chosen, cap, allow_small);
                if (wgs >= kn.target_wgs || cap == 1) break;
            }
        }
    }
    if (!fits) {   // a set of summed operations does not fit LDS together even at 4 columns
        s.error = BSPMM_ETOOBIG;
        return s;
    }
    if (kn.front > 0) {   // every operation must hold its layer input on chip
        Sink probe;
        draft_all(ops, F, vec, cand, chosen, kn, cap, allow_small, outs, stand_in, &fits, probe, fit_table);
        if (probe.per_range[1] || probe.generic) {
            s.error = BSPMM_ETOOBIG;
            return s;
        }
    }
    // the draft that is kept
    const std::vector<int> block_of_op = input_blocks(ops);
    Sink keep;
    keep.out = &d;
    keep.block_of_op = &block_of_op;
    keep.tile_unit = std::max(4, std::min(cand.back(), F));
    keep.tiles_per_block = (F + keep.tile_unit - 1) / keep.tile_unit;
    if (kn.front > 0) {   // every feature tile of an operation reads the whole of X_i: one group
        keep.tile_unit = std::max(4, F);
        keep.tiles_per_block = 1;
    }
    d.reserve((size_t)wgs * 4 + 16);
    draft_all(ops, F, vec, cand, chosen, kn, cap, allow_small, outs, stand_in, &fits, keep, fit_table);

    // group costs, for ordering and XCD placement
    int ngroups = 0;
    for (int bi : block_of_op) ngroups = std::max(ngroups, (bi + 1) * keep.tiles_per_block);
    for (Draft& x : d)
        if (x.fused >= 0) x.group = ngroups++;                // fused tasks stand alone
    std::vector<int64_t> gcost(ngroups, 0);
    std::vector<int> gsize(ngroups, 0);
    for (const Draft& x : d) {
        gcost[x.group] = std::max(gcost[x.group], x.cost);
        ++gsize[x.group];
    }
    for (Draft& x : d)
        if (x.fused < 0 && x.staged && gsize[x.group] == 1) x.staged |= 2;   // tile read once

    // Largest group first, members of a group together, larger items first inside a group,
    // equal keys in draft order.  The order only steers the greedy placement below, so costs
    // are compared in 15 and 16 bits (scaled to the largest): the three keys then pack into one
    // 55-bit word and a stable radix sort (11-bit digits: the counters stay in L1; digits that
    // are equal in every key are skipped) replaces the comparison sort, which was the most
    // expensive step of planning a large batch.
    std::vector<std::vector<int>> by_range(kRanges);
    {
        int64_t top = 1;
        for (int64_t c : gcost) top = std::max(top, c);
        int shift = 0;
        while ((top >> shift) > 0x7fff) ++shift;
        size_t n_in[kRanges] = {0, 0, 0, 0, 0};
        for (const Draft& x : d) n_in[draft_range(x)]++;
        std::vector<uint64_t> key[kRanges], key_tmp;
        std::vector<int> idx_tmp;
        for (int r = 0; r < kRanges; ++r) {
            key[r].reserve(n_in[r]);
            by_range[r].reserve(n_in[r]);
        }
        const bool packable = ngroups < (1 << 24);
        for (int idx = 0; idx < (int)d.size(); ++idx) {
            const Draft& x = d[idx];
            const int r = draft_range(x);
            const uint64_t g15 = 0x7fff - (uint64_t)(gcost[x.group] >> shift);
            const uint64_t c16 = 0xffff - (uint64_t)(std::min(x.cost, gcost[x.group]) >> shift << 1);
            key[r].push_back(g15 << 40 | (uint64_t)x.group << 16 | c16);
            by_range[r].push_back(idx);
        }
        uint32_t count[1 << 11];
        for (int r = 0; r < kRanges; ++r) {
            std::vector<uint64_t>& k = key[r];
            std::vector<int>& v = by_range[r];
            const size_t n = k.size();
            if (n < 2) continue;
            if (packable && n < 4096) {   // few items: the counters of a radix pass would outweigh them
                std::vector<std::pair<uint64_t, int>> kv(n);
                for (size_t t = 0; t < n; ++t) kv[t] = {k[t], v[t]};
                std::sort(kv.begin(), kv.end());     // (equal keys: by draft index, as the stable sort)
                for (size_t t = 0; t < n; ++t) v[t] = kv[t].second;
                continue;
            }
            if (!packable) {   // more groups than the key holds: compare
                std::vector<int> order(n);
                std::iota(order.begin(), order.end(), 0);
                std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
                    const Draft &x = d[v[a]], &y = d[v[b]];
                    if ((k[a] >> 40) != (k[b] >> 40)) return k[a] < k[b];
                    if (x.group != y.group) return x.group < y.group;
                    return (k[a] & 0xffff) < (k[b] & 0xffff);
                });
                std::vector<int> sorted(n);
                for (size_t t = 0; t < n; ++t) sorted[t] = v[order[t]];
                v.swap(sorted);
                continue;
            }
            key_tmp.resize(n);
            idx_tmp.resize(n);
            for (int pass = 0; pass < 5; ++pass) {
                const int sh = 11 * pass;
                std::fill(count, count + (1 << 11), 0u);
                for (size_t t = 0; t < n; ++t) ++count[(k[t] >> sh) & 0x7ff];
                if (count[(k[0] >> sh) & 0x7ff] == n) continue;   // one digit everywhere
                uint32_t run = 0;
                for (uint32_t& c : count) {
                    const uint32_t here = c;
                    c = run;
                    run += here;
                }
                for (size_t t = 0; t < n; ++t) {
                    const uint32_t at = count[(k[t] >> sh) & 0x7ff]++;
                    key_tmp[at] = k[t];
                    idx_tmp[at] = v[t];
                }
                k.swap(key_tmp);
                v.swap(idx_tmp);
            }
        }
    }

    // range 0: one item per workgroup; groups dealt to the XCD with the least cost so far,
    // then the eight lists interleaved so that list x occupies workgroups x, x+8, x+16, ...
    std::vector<std::vector<int>> xcd(kXcds);
    {
        int64_t load[kXcds] = {0};
        const std::vector<int>& v = by_range[0];
        for (auto& l : xcd) l.reserve(v.size() / kXcds + 64);
        size_t a = 0;
        while (a < v.size()) {
            size_t b = a;
            int64_t total = 0;
            while (b < v.size() && d[v[b]].group == d[v[a]].group) total += d[v[b++]].cost;
            const int x = (int)(std::min_element(load, load + kXcds) - load);
            for (size_t t = a; t < b; ++t) xcd[x].push_back(v[t]);
            load[x] += total;
            a = b;
        }
    }
    size_t longest = 0;
    for (auto& l : xcd) longest = std::max(longest, l.size());
    const int grid0 = (int)(longest * kXcds);

    // Optional persistent launch (off by default: the hardware dispatcher balances uneven
    // tasks better than a static stride): W workgroups take tasks w, w+W, ...  With the lists
    // sorted largest-first, every second round of W tasks is laid out backwards (in whole
    // groups of eight, so a task keeps its XCD) and the workgroup that drew the largest task
    // of one round draws the smallest of the next.
    bool slices = false;
    for (const Draft& x : d) slices = slices || x.bin == BSPMM_BIN_SLICE32 || x.bin == BSPMM_BIN_SLICE16;
    s.has_slices = slices;
    const int capacity = slices ? kn.capacity_wgs_slices : kn.capacity_wgs;
    const int W = std::max(kXcds, (kn.persistent_wgs > 0 ? kn.persistent_wgs : capacity) / kXcds * kXcds);
    const size_t per_round = (size_t)W / kXcds;
    for (auto& l : xcd) {
        l.resize(longest, -1);
        for (size_t a = per_round; kn.persistent_wgs > 0 && a < longest; a += 2 * per_round) {
            const size_t b = std::min(longest, a + per_round);
            std::reverse(l.begin() + a, l.begin() + b);
        }
    }

    // Whole layers in a launch of several rounds of workgroups, up to 64 input features: the
    // dense tiles are made in 32 x 32 blocks (half the LDS reads per flop, a quarter of the
    // blocks).  Measured on MI355X, four channels, F = 128: 2048 graphs 88 -> 79 us at
    // n_X = 32 and 130 -> 122 us at 64, 512 graphs 27.6 -> 25.6 and 35.8 -> 34.6 us; at
    // n_X = 128 it is 4 % slower, and a launch of one round (128 graphs) gains nothing.
    const bool wide_blocks = kn.front > 0 && kn.front <= 64 && wgs > 6 * kn.compute_units;
    auto emit = [&](int draft_idx, int wg, int slot) {
        const Draft& x = d[draft_idx];
        s.item_op.resize(s.items.size(), -1);      // empty items before this one
        s.items.push_back(to_item(ops, x));
        s.item_op.push_back(x.op);
        s.items_in_bin[x.bin]++;
        if (x.op < s.first_stand_in) {
            s.view.push_back({x.op, x.bin, x.row0, x.nrows, x.f0, x.fw, wg, slot});
        } else {   // a stand-in: the view lists the operations it stands for
            s.items.back().staged |= 4 | (kn.front > 0 ? ops.channels(x.op) << 8 : 0) | (wide_blocks ? 8 : 0);
            const std::vector<int>& mem = s.merged_sets[x.op - s.first_stand_in];
            for (size_t j = 0; j < mem.size(); ++j)
                s.view.push_back({mem[j], x.bin, x.row0, x.nrows, x.f0, x.fw, wg, (int)j});
        }
    };

    s.items.reserve(longest * kXcds + d.size() * (most_members > 1 ? most_members : 1) + 64);
    s.view.reserve(d.size() * (most_members > 1 ? most_members : 1));
    s.item_base[0] = 0;
    for (size_t pos = 0; pos < longest; ++pos)
        for (int x = 0; x < kXcds; ++x) {
            if (xcd[x][pos] >= 0)
                emit(xcd[x][pos], (int)(pos * kXcds + x), 0);
            else
                s.items.push_back(empty_item());
        }
    s.wg_end[0] = grid0;

    // range 1: fused tasks, `fused_stride` item slots each (the members, then empty items)
    int wg = grid0;
    {
        std::vector<std::vector<int>>& fused_sets = s.fused_sets;
        for (int g = 0; g < outs.size(); ++g)
            if (outs.count(g) > 1 && stand_in[g] < 0) fused_sets.push_back(outs.members(g));
        s.fused_stride = (int)most_members;
        s.item_base[1] = (int)s.items.size();
        for (int idx : by_range[1]) {
            const Draft& x = d[idx];
            const std::vector<int>& mem = fused_sets[x.fused];
            for (size_t j = 0; j < mem.size(); ++j) {
                Draft y = x;
                y.op = mem[j];
                WorkItem w = to_item(ops, y);
                size_t owner = j;
                for (size_t e = 0; e < j; ++e)
                    if (ops.in_off[mem[e]] == ops.in_off[mem[j]] && ops.k[mem[e]] == ops.k[mem[j]]) {
                        owner = e;
                        break;
                    }
                w.staged = 1 | (j == 0 ? (int)mem.size() << 8 : 0) | ((int)owner << 16);
                s.item_op.resize(s.items.size(), -1);
                s.items.push_back(w);
                s.item_op.push_back(y.op);
                s.view.push_back({y.op, BSPMM_BIN_WORKGROUP, x.row0, x.nrows, x.f0, x.fw, wg, (int)j});
                s.items_in_bin[BSPMM_BIN_WORKGROUP]++;
            }
            for (size_t j = mem.size(); j < most_members; ++j) s.items.push_back(empty_item());
            s.task_set.push_back(x.fused);
            ++wg;
            ++s.fused_tasks;
        }
        s.wg_end[1] = wg;
    }
    for (int r = 2; r < kRanges; ++r) {
        const int slots = kThreads >> range_log2_slot(r);
        s.item_base[r] = (int)s.items.size();
        const std::vector<int>& v = by_range[r];
        for (size_t t = 0; t < v.size(); ++t) emit(v[t], wg + (int)(t / slots), (int)(t % slots));
        const int nwg = (int)((v.size() + slots - 1) / slots);
        while ((int)s.items.size() < s.item_base[r] + nwg * slots) s.items.push_back(empty_item());
        wg += nwg;
        s.wg_end[r] = wg;
    }
    s.item_op.resize(s.items.size(), -1);
    s.grid = wg;
    s.launch_grid = kn.persistent_wgs > 0 ? std::min(wg, W) : wg;
    // The lean kernel serves launches made only of whole-workgroup items (staged operations and
    // row blocks of the generic bin) on the float4 path whose tile rows are a power-of-two number
    // of float4.
    s.lean = vec == 4 && kn.pad == 0 && !kn.hubs && kn.front == 0 && kn.persistent_wgs == 0 &&
             s.merged_sets.empty() && s.wg_end[0] == wg && wg > 0;
    for (const WorkItem& w : s.items) {
        if (!s.lean) break;
        if (w.nrows <= 0) continue;
        const int nvec = w.fw >> 2;
        s.lean = (w.fw & 3) == 0 && nvec > 0 && (nvec & (nvec - 1)) == 0 && nvec <= 64;
    }
    if (kn.front > 0) {
        int64_t most = 0;
        for (const WorkItem& w : s.items) {
            if (w.nrows <= 0) continue;
            const StagedLayout L = staged_layout(w.m, w.k, w.nnz, w.fw, 0, false);
            const int ch = std::max(1, (w.staged >> 8) & 0xff);     // channels of a stand-in
            most = std::max<int64_t>(most, (int64_t)L.total + (int64_t)(w.k / ch) * kn.front +
                                               ch * ((int64_t)kn.front * w.fw + w.fw));
        }
        s.front_lds_words = (int)std::min<int64_t>(kn.lds_words, round_up((int)most, 64));
    }
    return s;
}

// Direct COO kernel (the resource assignment of Sec. IV-C for SparseTensor operands, cases 1-3):
// an item keeps its whole output tile in LDS.  Where they fit beside it, the operation's dense
// tile and its entries are staged in LDS too (one bulk copy instead of one round trip to
// memory per entry); an operation that is too large for that at the batch-wide tile takes a
// narrower tile of its own, and one that fits at no width keeps only the output tile (and
// the entries, if they fit) on chip and is cut into row ranges, each of which scans all of the
// operation's entries and keeps its own (the paper falls back to atomics on global memory
// there).  As for CSR, the batch-wide tile is the widest one that still gives the launch
// enough workgroups.
namespace {

constexpr int kCooSortedRows = 128;   // rows of an item that sorts its entries and reads dense rows from memory

struct CooChoice {
    int fw;      // tile width of this operation
    int nr;      // rows per item
    int mode;
};

CooChoice coo_choice(const DirOps& o, int i, int F, size_t first, const std::vector<int>& cand,
                     const Knobs& kn)
{
    const int64_t W = kn.lds_words;
    // entries sorted by row on chip and the rows summed in registers (no output tile, no
    // atomics): with the dense tile beside them at the widest tile that fits, else with the
    // dense rows read from memory at the batch-wide tile
    for (size_t c = first; c < cand.size(); ++c) {
        const int fw = std::min(cand[c], F);
        if (coo_lds_words(o.m[i], o.k[i], o.nnz[i], fw, 7) <= W) return {fw, o.m[i], 7};
    }
    {
        // the dense rows come from memory entry by entry: narrow tiles and short row ranges, so
        // that a workgroup has many rows in flight and few to go through one after another
        const int fw = std::min(cand.back(), F);
        const int nr = std::min(o.m[i], kCooSortedRows);
        if (coo_lds_words(nr, o.k[i], o.nnz[i], fw, 6) <= W) return {fw, nr, 6};
    }
    for (size_t c = first; c < cand.size(); ++c) {
        const int fw = std::min(cand[c], F);
        if (coo_lds_words(o.m[i], o.k[i], o.nnz[i], fw, 3) <= W) return {fw, o.m[i], 3};
    }
    const int fw = std::min(cand[first], F);
    const int64_t stride = round_up(fw, 4);
    const int64_t ent = 3 * (int64_t)o.nnz[i] + 1;
    if (ent + 16 * stride <= W)
        return {fw, (int)std::min<int64_t>(o.m[i], (W - ent) / stride), 2};
    return {fw, (int)std::min<int64_t>(o.m[i], std::max<int64_t>(1, W / stride)), 0};
}

}  // namespace

namespace {
CooSchedule coo_schedule_at(const DirOps& ops, int F, const Knobs& kn_in);
}

// Without a budget from the caller the launch gets the smallest of a few LDS sizes at which
// every operation is sorted on chip (or has its entries and both tiles there): an operation that
// falls through to the row-range forms goes over all of its entries once per range and holds the
// whole launch up.
CooSchedule make_coo_schedule(const DirOps& ops, int F, const Knobs& kn)
{
    if (kn.lds_given) return coo_schedule_at(ops, F, kn);
    CooSchedule s;
    for (int words : {6144, 8192, 12288, 16384}) {
        Knobs k2 = kn;
        k2.lds_words = words;
        s = coo_schedule_at(ops, F, k2);
        bool ranges = false;
        for (const CooItem& it : s.items) ranges = ranges || (!(it.mode & 4) && it.mode != 3);
        if (!ranges) break;
    }
    return s;
}

namespace {

CooSchedule coo_schedule_at(const DirOps& ops, int F, const Knobs& kn_in)
{
    CooSchedule s;
    Knobs kn = kn_in;
    if (!kn.target_wgs) kn.target_wgs = 4 * kn.compute_units;
    const std::vector<int> cand = tile_candidates(F, kn);
    auto count = [&](size_t first) {
        int64_t n = 0;
        for (int i = 0; i < ops.size(); ++i)
            if (ops.m[i] > 0) {
                const CooChoice ch = coo_choice(ops, i, F, first, cand, kn);
                n += (int64_t)((F + ch.fw - 1) / ch.fw) * ((ops.m[i] + ch.nr - 1) / ch.nr);
            }
        return n;
    };
    size_t first = cand.size() - 1;
    for (size_t c = 0; c < cand.size(); ++c)
        if (count(c) >= kn.target_wgs) {
            first = c;
            break;
        }
    s.tile = std::min(cand[first], F);
    struct Key { int64_t work; int idx; };
    std::vector<CooItem> raw;
    for (int i = 0; i < ops.size(); ++i) {
        if (ops.m[i] <= 0) continue;
        const CooChoice ch = coo_choice(ops, i, F, first, cand, kn);
        const int parts = (ops.m[i] + ch.nr - 1) / ch.nr;
        const int per = (ops.m[i] + parts - 1) / parts;
        for (int f0 = 0; f0 < F; f0 += ch.fw)
            for (int r0 = 0; r0 < ops.m[i]; r0 += per) {
                CooItem it{};
                it.nz_off = ops.nz_off[i];
                it.in_row_off = ops.in_off[i];
                it.out_row_off = ops.out_off[i];
                it.nnz = ops.nnz[i];
                it.k = ops.k[i];
                it.row0 = r0;
                it.nrows = std::min(per, ops.m[i] - r0);
                it.f0 = f0;
                it.fw = std::min(ch.fw, F - f0);
                it.op = i;
                it.mode = ch.mode;
                raw.push_back(it);
            }
    }
    std::vector<Key> order(raw.size());
    for (size_t j = 0; j < raw.size(); ++j)
        order[j] = {(int64_t)raw[j].fw * ((int64_t)raw[j].nnz * ((raw[j].mode & 1) ? 1 : 4) +
                                          2 * raw[j].nrows + raw[j].k), (int)j};
    std::stable_sort(order.begin(), order.end(),
                     [](const Key& a, const Key& b) { return a.work > b.work; });
    s.items.reserve(raw.size());
    s.view.reserve(raw.size());
    for (const Key& kx : order) {
        const CooItem& it = raw[kx.idx];
        bspmm_item v;
        v.op = it.op;
        v.bin = BSPMM_BIN_COO;
        v.row0 = it.row0;
        v.nrows = it.nrows;
        v.f0 = it.f0;
        v.fw = it.fw;
        v.workgroup = (int32_t)s.items.size();
        v.slot = it.mode;
        s.items.push_back(it);
        s.view.push_back(v);
        s.lds_words = (int)std::max<int64_t>(s.lds_words, coo_lds_words(it.nrows, it.k, it.nnz, it.fw, it.mode));
    }
    s.lds_words = std::min(kn.lds_words, round_up(s.lds_words, 64));
    return s;
}

}  // namespace

}  // namespace bspmm

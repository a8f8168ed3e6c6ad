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
#include <map>
#include <numeric>
#include <utility>

namespace bspmm {

namespace {

constexpr int kXcds = 8;

struct Draft {           // one item before placement
    int op;
    int bin;
    int row0, nrows, f0, fw;
    int staged;
    int64_t cost;
    int group;           // items with one group read the same dense tile
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
        case BSPMM_BIN_WAVE: return 1;
        case BSPMM_BIN_SLICE32: return 2;
        case BSPMM_BIN_SLICE16: return 3;
        default: return 0;
    }
}

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
    return need <= (int64_t)kn.lds_words * lanes / kThreads;
}

// Decide bin and tile of operation i given the batch-wide tile candidates from `first` on.
Choice choose(const DirOps& o, int i, int F, int vec, const std::vector<int>& cand, size_t first,
              const Knobs& kn, bool allow_small)
{
    const int forced = kn.force_bin;
    if (forced == BSPMM_BIN_GENERIC) return {BSPMM_BIN_GENERIC, cand[0]};
    if (forced >= 0) {
        for (size_t c = first; c < cand.size(); ++c)
            if (fits_slot(o, i, cand[c], F, vec, bin_slot_lanes(forced), 0, kn))
                return {forced, cand[c]};
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

// `cap` > 0 cuts a workgroup item into row ranges of at most `cap` passes each (every range
// stages the whole operation, so the cut costs on-chip traffic and buys parallelism).
void draft_op(const DirOps& o, int i, int F, int vec, const Choice& ch, const Knobs& kn, int cap,
              std::map<std::pair<int64_t, int>, int>& groups, std::vector<Draft>& out)
{
    if (o.m[i] <= 0) return;
    const int tile = ch.tile;
    for (int f0 = 0; f0 < F; f0 += tile) {
        const int fw = std::min(tile, F - f0);
        auto key = std::make_pair(o.in_off[i], f0);
        auto it = groups.find(key);
        int gid;
        if (it == groups.end()) {
            gid = (int)groups.size();
            groups.emplace(key, gid);
        } else {
            gid = it->second;
        }
        if (ch.bin == BSPMM_BIN_WORKGROUP && cap > 0) {
            const int rows_per_pass = kThreads / lanes_per_row(fw, vec);
            const int chunk = cap * rows_per_pass;
            for (int r0 = 0; r0 < o.m[i]; r0 += chunk) {
                const int nr = std::min(chunk, o.m[i] - r0);
                out.push_back({i, ch.bin, r0, nr, f0, fw, 1, item_cost(o, i, nr, fw, true), gid});
            }
        } else if (ch.bin != BSPMM_BIN_GENERIC) {
            out.push_back({i, ch.bin, 0, o.m[i], f0, fw, 1, item_cost(o, i, o.m[i], fw, true), gid});
        } else {
            for (int r0 = 0; r0 < o.m[i]; r0 += kn.generic_rows) {
                const int nr = std::min(kn.generic_rows, o.m[i] - r0);
                out.push_back({i, ch.bin, r0, nr, f0, fw, 0, item_cost(o, i, nr, fw, false), gid});
            }
        }
    }
}

std::vector<Draft> draft_all(const DirOps& o, int F, int vec, const std::vector<int>& cand,
                             size_t first, const Knobs& kn, int cap, bool allow_small)
{
    std::vector<Draft> d;
    std::map<std::pair<int64_t, int>, int> groups;
    for (int i = 0; i < o.size(); ++i)
        draft_op(o, i, F, vec, choose(o, i, F, vec, cand, first, kn, allow_small), kn, cap, groups,
                 d);
    return d;
}

int count_workgroups(const std::vector<Draft>& d)
{
    int per_range[kRanges] = {0, 0, 0, 0};
    for (const Draft& x : d) per_range[bin_range(x.bin)]++;
    int wgs = per_range[0];
    for (int r = 1; r < kRanges; ++r) {
        const int slots = kThreads >> range_log2_slot(r);
        wgs += (per_range[r] + slots - 1) / slots;
    }
    return wgs;
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
    k.target_wgs = o->target_workgroups > 0 ? o->target_workgroups : 4 * k.compute_units;
    if (o->lds_pad > 0) k.pad = std::min(o->lds_pad, 64) / 4 * 4;
    if (o->lds_pad < 0) k.pad = 0;
    if (o->max_passes > 0) k.max_passes = o->max_passes;
    if (o->generic_rows > 0) k.generic_rows = o->generic_rows;
    k.wg_passes = o->wg_passes;
    if (o->resident_workgroups > 0) k.persistent_wgs = o->resident_workgroups;
    k.hubs = (o->flags & BSPMM_SPLIT_HUB_ROWS) != 0;
    return k;
}

Schedule make_schedule(const DirOps& ops, int F, const Knobs& kn_in)
{
    Schedule s;
    Knobs kn = kn_in;
    if (!kn_in.target_wgs) kn.target_wgs = 4 * kn.compute_units;
    const int vec = (F % 4 == 0) ? 4 : 1;
    const std::vector<int> cand = tile_candidates(F, kn);

    // widest batch-wide tile that still gives the launch enough workgroups
    std::vector<Draft> d;
    size_t chosen = cand.size() - 1;
    // Sub-workgroup slots pack several small items into one workgroup.  Measured on MI355X
    // that only pays when the launch is over-subscribed (more workgroups than the chip holds
    // at once); a launch that fits is latency-bound and every item is fastest with a whole
    // workgroup staging it.  A forced bin overrides this.
    const int fixed_cap = kn.wg_passes > 0 ? kn.wg_passes : 0;
    bool allow_small = kn.force_bin >= 0;
    for (int attempt = 0; attempt < 2; ++attempt) {
        for (size_t c = 0; c < cand.size(); ++c) {
            d = draft_all(ops, F, vec, cand, c, kn, fixed_cap, allow_small);
            if (count_workgroups(d) >= kn.target_wgs || c + 1 == cand.size()) {
                chosen = c;
                break;
            }
        }
        if (allow_small || count_workgroups(d) <= kn.capacity_wgs) break;
        allow_small = true;
    }
    s.tile = cand[chosen];
    // still too few workgroups at the narrowest tile: the batch is small, its time is set by
    // the slowest workgroup, so cut multi-pass workgroup items into row ranges
    if (kn.wg_passes == 0 && count_workgroups(d) < kn.target_wgs) {
        for (int cap = 4; cap >= 1; cap /= 2) {
            d = draft_all(ops, F, vec, cand, chosen, kn, cap, allow_small);
            if (count_workgroups(d) >= kn.target_wgs) break;
        }
    }

    // group costs, for ordering and XCD placement
    int ngroups = 0;
    for (const Draft& x : d) ngroups = std::max(ngroups, x.group + 1);
    std::vector<int64_t> gcost(ngroups, 0);
    std::vector<int> gsize(ngroups, 0);
    for (const Draft& x : d) {
        gcost[x.group] = std::max(gcost[x.group], x.cost);
        ++gsize[x.group];
    }
    for (Draft& x : d)
        if (x.staged && gsize[x.group] == 1) x.staged |= 2;   // nobody else reads this tile

    std::vector<std::vector<int>> by_range(kRanges);
    for (int idx = 0; idx < (int)d.size(); ++idx) by_range[bin_range(d[idx].bin)].push_back(idx);
    auto big_first = [&](int a, int b) {
        const Draft &x = d[a], &y = d[b];
        if (gcost[x.group] != gcost[y.group]) return gcost[x.group] > gcost[y.group];
        if (x.group != y.group) return x.group < y.group;
        if (x.cost != y.cost) return x.cost > y.cost;
        return a < b;
    };
    for (auto& v : by_range) std::sort(v.begin(), v.end(), big_first);

    // range 0: one item per workgroup; groups dealt to the XCD with the least cost so far,
    // then the eight lists interleaved so that list x occupies workgroups x, x+8, x+16, ...
    std::vector<std::vector<int>> xcd(kXcds);
    {
        int64_t load[kXcds] = {0};
        const std::vector<int>& v = by_range[0];
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

    auto emit = [&](int draft_idx, int wg, int slot) {
        const Draft& x = d[draft_idx];
        s.items.push_back(to_item(ops, x));
        s.view.push_back({x.op, x.bin, x.row0, x.nrows, x.f0, x.fw, wg, slot});
        s.items_in_bin[x.bin]++;
    };

    s.item_base[0] = 0;
    for (size_t pos = 0; pos < longest; ++pos)
        for (int x = 0; x < kXcds; ++x) {
            if (xcd[x][pos] >= 0)
                emit(xcd[x][pos], (int)(pos * kXcds + x), 0);
            else
                s.items.push_back(empty_item());
        }
    s.wg_end[0] = grid0;

    int wg = grid0;
    for (int r = 1; r < kRanges; ++r) {
        const int slots = kThreads >> range_log2_slot(r);
        s.item_base[r] = (int)s.items.size();
        const std::vector<int>& v = by_range[r];
        for (size_t t = 0; t < v.size(); ++t) emit(v[t], wg + (int)(t / slots), (int)(t % slots));
        const int nwg = (int)((v.size() + slots - 1) / slots);
        while ((int)s.items.size() < s.item_base[r] + nwg * slots) s.items.push_back(empty_item());
        wg += nwg;
        s.wg_end[r] = wg;
    }
    s.grid = wg;
    s.launch_grid = kn.persistent_wgs > 0 ? std::min(wg, W) : wg;
    return s;
}

}  // namespace bspmm

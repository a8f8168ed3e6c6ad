// C ABI of libbspmm (see include/bspmm.h for the contract of every entry point).
#include <hip/hip_runtime.h>
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <atomic>
#include <cstring>
#include <mutex>
#include <new>
#include <set>
#include <memory>
#include <utility>
#include <vector>

#include "../../include/bspmm.h"
#include "plan.hpp"
#include "schedule.hpp"

namespace bspmm {
hipError_t launch_bspmm(const LaunchParams& P, int grid, int lds_bytes, bool vec4, bool slices,
                        bool hubs, bool merged, hipStream_t stream);
hipError_t launch_bspmm_lean(const LeanItem* items, const LaunchParams& P, int grid, int lds_bytes,
                             hipStream_t stream);
hipError_t launch_lean_hints(LeanItem* items, int n, const int32_t* rpt, hipStream_t stream);
hipError_t launch_bspmm_gcn(const LaunchParams& P, int grid, int lds_bytes, bool accumulate,
                            bool sets, bool wide, hipStream_t stream);
int front_workgroups_per_cu(bool sets, bool wide, int lds_bytes);
hipError_t launch_bspmm_gcn_stream(const StreamParams& S, int nx16, int units, int waves, int grid,
                                   int lds_bytes, hipStream_t stream);
bool stream_supported(int nx16, int units, int waves);
int stream_workgroups_per_cu(int nx16, int units, int waves, int lds_bytes);
hipError_t launch_build_transpose(const OpRecord* ops, int batch, int threads, int lds_bytes,
                                  const int32_t* rpt, const int32_t* colids,
                                  const float* values, int32_t* rpt_t, int32_t* colids_t,
                                  float* values_t, int32_t* gscratch, const int32_t* order,
                                  hipStream_t stream);
hipError_t launch_build_from_coo(const OpRecord* ops, int batch, int threads, int lds_bytes, const int32_t* ids,
                                 const float* values, int32_t* rpt, int32_t* colids,
                                 float* csr_values, int32_t* gscratch, const int32_t* order,
                                 hipStream_t stream);
hipError_t launch_bspmm_coo(const CooLaunchParams& P, int grid, int lds_bytes, bool vec4,
                            hipStream_t stream);
hipError_t launch_merge_sets(const SetRecord* sets, int count, const int32_t* rpt,
                             const int32_t* colids, const float* values, int32_t* merged,
                             hipStream_t stream);
hipError_t launch_validate_coo(const OpRecord* ops, int batch, const int32_t* ids, int32_t* flag,
                               hipStream_t stream);
int bspmm_max_resident_workgroups(int lds_bytes, bool slices, bool hubs);
hipError_t kernel_resources(int which, int lds_bytes, int out[7]);
hipError_t launch_validate(const OpRecord* ops, int batch, const int32_t* rpt,
                           const int32_t* colids, int32_t* flag, hipStream_t stream);
}  // namespace bspmm

using namespace bspmm;


// Workspace of plans made by bspmm_create_static: device memory that belongs to the library's
// code object, so no allocation is needed to get it.  Every GPU the library runs on holds its own
// copy at its own address until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress (see static_workspace below); it is never passed to a kernel or a copy.
static __device__ __align__(256) unsigned char scratch[BSPMM_STATIC_WORKSPACE_BYTES];

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return BSPMM_EHIP;
}

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Where each table sits inside the workspace (byte offsets).
struct Layout {
    size_t items[2] = {0, 0};
    size_t lean[2] = {0, 0};     // item tables of the lean kernel (empty when a direction is not lean)
    size_t op_records = 0;
    size_t build_order = 0;
    size_t rpt_t = 0, colids_t = 0, values_t = 0;
    size_t scratch = 0;
    size_t flag = 0;
    // summed sets (BSPMM_ACCUMULATE), per direction: their records and their merged CSR arrays
    size_t sets[2] = {0, 0};
    size_t merged[2] = {0, 0};
    // whole layers run by streaming workgroups: graph records, list bounds, and the items of the
    // graphs that stay with the one-launch kernel
    size_t stream_records = 0, stream_merged = 0, stream_sets = 0, stream_list = 0, stream_rest = 0;
    // plans made from COO operands: the CSR arrays built on the device and what the build needs
    size_t coo_records = 0;
    size_t csr_rpt = 0, csr_colids = 0, csr_values = 0;
    size_t coo_scratch = 0;
    size_t total = 0;
};

}  // namespace

struct bspmm_plan {
    int static_device = -1;         // >= 0: the workspace is that device's static array ...
    uint64_t static_generation = 0; // ... as handed out by this call of bspmm_create_static
    int32_t batch = 0;
    int32_t F = 0;
    bool dry = false;
    int front_wide = 0;             // the one-launch layer kernel runs with workgroups of eight wavefronts
    Knobs knobs;
    DirOps dir[2];
    Schedule sched[2];
    std::vector<OpRecord> records;
    std::vector<int32_t> build_order;      // operations, most entries first: the order the build
                                           // kernels take them in
    std::vector<LeanItem> lean_items[2];   // per direction: the items again, for the lean kernel
    int32_t lean_rows[2] = {0, 0};         // most input rows / output rows of an operation: bounds
    int32_t lean_out_rows[2] = {0, 0};     // of the 32-bit offsets the lean kernel forms per call
    bool lean_blocks[2] = {false, false};  // the lean table has row blocks of the generic bin ...
    bool lean_hints_built[2] = {false, false};   // ... and the device has filled in their entry ranges
    std::vector<char> tables;   // host image of the workspace's front: item tables and records
    Layout lay;
    int build_lds_bytes = 0;
    int build_threads = kThreads;          // lanes per workgroup of the build kernels
    int64_t scratch_words = 0;
    bool transposed_supported = true;
    bool transposed_built = false;
    std::vector<SetRecord> set_records[2];   // summed sets of the forward / transposed schedule
    int64_t merged_words[2] = {0, 0};
    bool merged_built[2] = {false, false};
    int front_channels = 1;   // fused front with BSPMM_ACCUMULATE: channels per output block
    // Whole layers in launches of many rounds: the graphs that fit the LDS budget of the
    // streaming launch, in list order; list l is sets[list[l]] .. sets[list[l + 1]]; the items of
    // the other graphs, for a launch of bspmm_gcn_kernel of their own.
    struct Stream {
        std::vector<StreamSet> sets;
        std::vector<int32_t> list;
        std::vector<WorkItem> rest;
        int nx16 = 0, units = 0, waves = 4, fw = 0, tiles = 0, lists = 0;
        bool compact = false;            // the groups bring lists of the tile rows in use
        int channels = 1;                // channels the kernel runs with (the layer's, or the next of 4 and 8)
        std::vector<SetRecord> records;   // one per group of graphs, for the kernel that merges CSR arrays
        int64_t merged_words = 0;  // words of the groups' merged CSR blocks
        bool merged_built = false;
        int graphs = 0;            // graphs in the lists (a list entry is a group of one or more)
        int tile_words = 0, x_words = 0, csr_words = 0;
        int big_csr_words = 0;     // room for the merged CSR block of a graph taken one at a time
        int big = 0;               // graphs taken one at a time
        int lds_bytes() const { return 4 * (tile_words + 2 * x_words + 2 * csr_words + 64); }
        bool on() const { return !sets.empty(); }
    } stream;
    int64_t effective_bytes[2] = {0, 0};
    int64_t flops = 0;
    bool reads_dense = false;   // some operation has rows and columns: the runs read the dense input
    // borrowed device pointers
    const int32_t* rpt = nullptr;
    const int32_t* colids = nullptr;
    const float* values = nullptr;
    char* ws = nullptr;
    // COO / SparseTensor input: borrowed pair array and values, records of the conversion
    bool from_coo = false;
    const int32_t* ids = nullptr;
    const float* coo_values = nullptr;
    std::vector<OpRecord> coo_records;
    int coo_build_lds_bytes = 0;
    int64_t csr_rpt_words = 0, csr_nz = 0, coo_scratch_words = 0;
    // BSPMM_COO_DIRECT: no CSR at all, the runs launch the direct COO kernel
    bool coo_direct = false;
    CooSchedule coo_sched[2];
};

namespace {

int check_batch(const bspmm_batch* b, int32_t F, bool need_device)
{
    if (!b || F <= 0 || b->batch < 0) return BSPMM_EINVAL;
    if (b->batch == 0) return BSPMM_OK;
    if (!b->rows || !b->cols || !b->nnz || !b->rpt_off || !b->nz_off || !b->b_row_off ||
        !b->c_row_off)
        return BSPMM_EINVAL;
    int64_t total_nnz = 0;
    for (int i = 0; i < b->batch; ++i) {
        if (b->rows[i] < 0 || b->cols[i] < 0 || b->nnz[i] < 0) return BSPMM_EINVAL;
        if (b->rpt_off[i] < 0 || b->nz_off[i] < 0 || b->b_row_off[i] < 0 || b->c_row_off[i] < 0)
            return BSPMM_EINVAL;
        if ((b->rows[i] == 0 || b->cols[i] == 0) && b->nnz[i] != 0) return BSPMM_EINVAL;
        total_nnz += b->nnz[i];
    }
    if (need_device) {
        if (!b->rpt) return BSPMM_EINVAL;
        if (total_nnz > 0 && (!b->colids || !b->values)) return BSPMM_EINVAL;
    }
    return BSPMM_OK;
}

// How the half-open row intervals [off, off+len) with len > 0 relate:
// 0 = pairwise disjoint, 1 = some are identical but none overlaps otherwise, 2 = real overlap.
int overlap_kind(const int64_t* off, const int32_t* len, int n)
{
    bool in_order = true;   // the usual case: blocks back to back in operation order
    int64_t end = 0;
    for (int i = 0; i < n && in_order; ++i) {
        if (len[i] <= 0) continue;
        in_order = off[i] >= end;
        end = off[i] + len[i];
    }
    if (in_order) return 0;
    std::vector<std::pair<int64_t, int64_t>> v;
    v.reserve(n);
    for (int i = 0; i < n; ++i)
        if (len[i] > 0) v.emplace_back(off[i], off[i] + len[i]);
    std::sort(v.begin(), v.end());
    int kind = 0;
    for (size_t i = 1; i < v.size(); ++i) {
        if (v[i] == v[i - 1])
            kind = std::max(kind, 1);
        else if (v[i].first < v[i - 1].second)
            return 2;
    }
    return kind;
}

// The sets of summed operations of direction d: one record per set for the kernel that merges
// their CSR arrays, room for the merged arrays, and the location of those in the first item of
// every task of the set (its rpt_off, nz_off and nnz then describe the merged CSR).
void describe_sets(bspmm_plan& p, int d)
{
    Schedule& sc = p.sched[d];
    const DirOps& o = p.dir[d];
    std::vector<SetRecord>& recs = p.set_records[d];
    recs.clear();
    int64_t words = 0;
    auto describe = [&](const std::vector<int>& mem, bool plain) {
        SetRecord r;
        std::memset(&r, 0, sizeof r);
        r.members = (int32_t)mem.size();
        r.m = o.m[mem[0]];
        r.plain = plain ? 1 : 0;
        int32_t rows = 0;
        int64_t nnz_sum = 0;
        for (size_t j = 0; j < mem.size(); ++j) {
            r.rpt_off[j] = o.rpt_off[mem[j]];
            r.nz_off[j] = o.nz_off[mem[j]];
            r.nnz[j] = o.nnz[mem[j]];
            r.k[j] = o.k[mem[j]];
            r.row_off[j] = 0;
            r.rows[j] = o.m[mem[0]];
            size_t owner = j;
            for (size_t e = 0; e < j; ++e)
                if (o.in_off[mem[e]] == o.in_off[mem[j]] && o.k[mem[e]] == o.k[mem[j]]) {
                    owner = e;
                    break;
                }
            if (owner == j || (plain && d == 0 && p.knobs.front > 0)) {   // (front: a tile per channel)
                r.tile_row[j] = rows;
                rows += o.k[mem[j]];
            } else {
                r.tile_row[j] = r.tile_row[owner];
            }
            nnz_sum += o.nnz[mem[j]];
        }
        r.merged_rpt_off = words;
        words += round_up(r.m + 1, 4);
        r.merged_nz_off = words;
        words += 2 * (int64_t)round_up((int)nnz_sum, 4);
        recs.push_back(r);
        return (int32_t)nnz_sum;
    };
    // sets run as fused tasks, then sets an operation with the summed matrix stands in for
    std::vector<int32_t> nnz_sum;
    for (const std::vector<int>& mem : sc.fused_sets) nnz_sum.push_back(describe(mem, false));
    const size_t first_plain = recs.size();
    for (const std::vector<int>& mem : sc.merged_sets) describe(mem, true);
    p.merged_words[d] = words;
    for (size_t t = 0; t < sc.task_set.size(); ++t) {
        const int si = sc.task_set[t];
        WorkItem& w = sc.items[(size_t)sc.item_base[1] + t * sc.fused_stride];
        w.rpt_off = recs[si].merged_rpt_off;
        w.nz_off = recs[si].merged_nz_off;
        w.nnz = nnz_sum[si];
    }
    if (!sc.merged_sets.empty())
        for (size_t j = 0; j < sc.items.size(); ++j) {
            const int op = j < sc.item_op.size() ? sc.item_op[j] : -1;
            if (op < sc.first_stand_in) continue;
            const SetRecord& r = recs[first_plain + (size_t)(op - sc.first_stand_in)];
            sc.items[j].rpt_off = r.merged_rpt_off;
            sc.items[j].nz_off = r.merged_nz_off;
        }
}

// Layers (bspmm_run_gcn) of two and more workgroups per CU: the plan of the streaming launch.
// A workgroup of the streaming kernel holds the weights of its feature tile in registers
// (M * fw / 16 blocks of 16 columns over four wavefronts: one or two per wavefront) and takes
// the graphs of its list one after the other; what it takes per trip is a *group*: one graph, or
// several small graphs that lie back to back in X and in Y, which are to the kernel one graph
// with a block-diagonal matrix (fewer trips, fuller 16-row blocks for the matrix instructions).
// Every group gets one merged CSR block (row pointers, columns, values back to back), built once
// per plan by the kernel that merges summed sets: its members are the channel operations of the
// group's graphs, each with its rows' place in the group and its tile's place in the group's
// dense tile.  The launch's LDS is sized for the groups that fit the budget (three workgroups per
// CU unless the caller fixed lds_bytes), smallest first; larger graphs are taken one at a time
// by the same workgroups where the kernel can, and otherwise keep their items of the one-launch
// schedule and run in a launch of their own.  Lists are balanced by
// longest-processing-time-first on an estimate of a trip's cycles.
void make_stream_plan(bspmm_plan& p)
{
    bspmm_plan::Stream& st = p.stream;
    st = bspmm_plan::Stream();
    const Schedule& sc = p.sched[0];
    const Knobs& kn = p.knobs;
    const int nx = kn.front, F = p.F;
    if (nx <= 0 || kn.one_front_launch || !sc.fused_sets.empty() || sc.fused_tasks > 0) return;
    // (plans of single channels - no operations summed - take the same kernel with one channel)
    const bool single = sc.merged_sets.empty();
    // Layers of 3, 5, 6 or 7 channels run as layers of 4 or 8 whose last channels are empty: no
    // entry names a row of their tiles, their weights read as zero, and with the lists of rows in
    // use their wavefronts have no matrix work at all.
    const int channels = single ? 1 : p.front_channels;
    if (!single && !kn.accumulate) return;
    if (nx % 16 != 0 || channels < 1 || channels > 8) return;
    const int M = channels <= 2 ? channels : (channels <= 4 ? 4 : 8);
    const int nx16 = nx / 16;
    int units = 0, fw = 0, waves = 4;
    // (two blocks per wavefront first, except for two channels: one block per wavefront makes
    // their tiles 32 columns wide like those of four channels - eight lanes per output row, 32
    // rows per gather pass, larger graphs taken in the same launch - and measured 2048 graphs at
    // n_X = 64 38 against 51 us, 512 graphs 12 against 23 us.  Eight channels: workgroups of
    // eight wavefronts, one per channel, for the same reason.)
    const int shapes[4][2] = {{M == 2 ? 1 : 2, M == 8 ? 8 : 4}, {M == 2 ? 2 : 1, M == 8 ? 8 : 4}, {2, 4}, {1, 4}};
    for (const auto& sh : shapes) {
        const int u = sh[0], wv = sh[1];
        const int w = 16 * wv * u / M;
        // (tiles of up to 64 columns: 16 lanes per output row, 64 rows in the gather's passes)
        if (w >= 16 && w <= 64 && F % w == 0 && stream_supported(nx16, u, wv)) {
            units = u;
            waves = wv;
            fw = w;
            break;
        }
    }
    if (!units) return;
    const int threads = 64 * waves;
    const int tiles = F / fw;
    const DirOps& o = p.dir[0];
    // the graphs: sets of channel operations, or the operations themselves
    std::vector<std::vector<int>> single_sets;
    if (single)
        for (int i = 0; i < o.size(); ++i) single_sets.push_back(std::vector<int>(1, i));
    const std::vector<std::vector<int>>& graphs = single ? single_sets : sc.merged_sets;
    const size_t n_graphs = graphs.size();
    // a launch of less than two workgroups per CU gains nothing from resident workgroups
    // (measured, four channels, F = 128, n_X = 64 / 32: 64 graphs 9.5 against 9.4 us for the
    // one-launch kernel; 128 graphs 10.5 / 8.2 against 11.9 / 8.2; 256 graphs 14.6 / 10.4
    // against 24.4 / 15.8)
    // Kernels with one block per wavefront and several channels (tiles of 16 columns): 128
    // graphs at n_X = 128 take 22.9 against 18.1 us, 512 graphs 51 against 63.
    if ((int64_t)n_graphs * tiles < (units == 2 || single ? 2 : 8) * (int64_t)kn.compute_units) return;
    // One channel: a trip holds a quarter of a four-channel trip's matrix work for the same
    // bookkeeping, and the one-launch kernel stays ahead for longer - measured on molecule
    // graphs of 25 nodes on 256 CUs, streamed against one launch: n_X = 32: 512 graphs 9.5
    // against 8.5 us, 1024 graphs 13.6 against 14.4; n_X = 64: 384 graphs 10.5 against 9.2, 448
    // graphs 10.9 against 11.9; n_X = 128: 256 graphs 15.4 against 15.2, 512 graphs 16.7 against
    // 19.7.  The crossing sits near 700,000 elements of layer input.
    if (single) {
        int64_t x_rows = 0;
        for (size_t g = 0; g < n_graphs; ++g) x_rows += o.k[graphs[g][0]];
        if (x_rows * nx * 256 < (int64_t)700000 * kn.compute_units) return;
    }

    // ---- groups: graphs back to back in X and in Y, while the members fit a record, the rows of
    // X three 16-row blocks (four for single channels) and the rows of Y the gather's passes
    // (three workgroups per CU: a third of the CU's 160 KiB less what the allocation granule
    // takes; 53920 bytes were measured to leave room for two only)
    // (workgroups of eight wavefronts: two per CU, half of a CU's LDS each)
    const int64_t budget_words = (kn.lds_given ? kn.lds_words * 4 : (waves == 8 ? 81920 : 53248)) / 4;
    const int rows_most = kStreamPasses * (threads / (fw / 4));
    // (a group must still go through the buffers: its tile, two buffers of X rows and two of CSR
    // blocks - about ten words a row each, and one per channel for the lists of rows in use -
    // inside the budget)
    const int group_rows = (int)std::min<int64_t>(single ? 64 : 48, (budget_words - 64) / ((int64_t)M * fw + 2 * nx + 20 + (single ? 0 : 2 * M)));
    const int group_graphs = kMaxMembers / channels;
    std::vector<int> by_input;
    for (size_t g = 0; g < n_graphs; ++g) {
        const int op0 = graphs[g][0];
        if (o.m[op0] > 0 && o.k[op0] > 0) by_input.push_back((int)g);
    }
    std::stable_sort(by_input.begin(), by_input.end(),
                     [&](int a, int b) { return o.in_off[graphs[a][0]] < o.in_off[graphs[b][0]]; });
    // How many graphs a group may hold is chosen for the launch: larger groups mean fewer and
    // longer trips, and a list of two long trips beside lists of one is a launch twice as long as
    // it need be (1024 single-channel graphs at n_X = 128: 28.6 us in groups of up to eight,
    // 21.8 us ungrouped; 2048 graphs: 33 against 43 us).  Each size is tried and the one with the
    // smallest estimate - the larger of "work per list" and "trips of the fullest list x work per
    // trip", a trip counted as two units plus three per 16-row block - is kept.
    auto form_groups = [&](int most) {
        std::vector<std::vector<int>> out;
        int64_t kx_sum = 0, m_sum = 0;
        for (int g : by_input) {
            const int op0 = graphs[g][0];
            bool joins = false;
            if (!out.empty() && (int)out.back().size() < most) {
                const int last = graphs[out.back().back()][0];
                joins = o.in_off[op0] == o.in_off[last] + o.k[last] && o.out_off[op0] == o.out_off[last] + o.m[last] &&
                        kx_sum + o.k[op0] <= group_rows && m_sum + o.m[op0] <= rows_most;
            }
            if (!joins) {
                out.push_back(std::vector<int>());
                kx_sum = m_sum = 0;
            }
            out.back().push_back(g);
            kx_sum += o.k[op0];
            m_sum += o.m[op0];
        }
        return out;
    };
    std::vector<std::vector<int>> groups;
    {
        const int64_t cap_lists = std::max<int64_t>(1, (waves == 8 ? 2 : 3) * (int64_t)kn.compute_units / tiles);
        double best = 0;
        for (int most = 1; most <= group_graphs; ++most) {
            std::vector<std::vector<int>> cand = form_groups(most);
            int64_t total = 0;
            for (const std::vector<int>& grp : cand) {
                int64_t kx = 0;
                for (int g : grp) kx += o.k[graphs[g][0]];
                total += 3 * ((kx + 15) / 16) + 2;
            }
            const int64_t lists = std::max<int64_t>(1, std::min<int64_t>((int64_t)cand.size(), cap_lists));
            const double per_trip = cand.empty() ? 0.0 : (double)total / (double)cand.size();
            const double estimate = std::max((double)total / (double)lists,
                                             (double)(((int64_t)cand.size() + lists - 1) / lists) * per_trip);
            if (most == 1 || estimate <= best) {
                best = estimate;
                groups.swap(cand);
            }
        }
    }
    const size_t n_sets = groups.size();
    if (n_sets == 0) return;
    // Layers of several channels in which a wavefront's blocks belong to one channel: the rows of
    // a channel's dense tile that none of its entries names are not made (see merge_sets_kernel).
    const bool compact_on = M >= 2 && (units == 1 || fw >= 32);
    // one record per group for the merging kernel; what the rest of this function needs of a group
    std::vector<SetRecord>& recs = st.records;
    std::vector<int64_t> nnz_sum(n_sets, 0);
    {
        int64_t words = 0;
        for (size_t s = 0; s < n_sets; ++s) {
            SetRecord r;
            std::memset(&r, 0, sizeof r);
            int64_t kxt = 0, mt = 0;
            for (int g : groups[s]) {
                kxt += o.k[graphs[g][0]];
                mt += o.m[graphs[g][0]];
            }
            int j = 0;
            int64_t x_at = 0, m_at = 0;
            for (int g : groups[s]) {
                const int op0 = graphs[g][0];
                for (int c = 0; c < channels; ++c, ++j) {
                    const int op = graphs[g][c];
                    r.rpt_off[j] = o.rpt_off[op];
                    r.nz_off[j] = o.nz_off[op];
                    r.nnz[j] = o.nnz[op];
                    r.k[j] = o.k[op0];
                    r.tile_row[j] = (int32_t)(c * kxt + x_at);     // channel c's tile, this graph's rows of it
                    r.row_off[j] = (int32_t)m_at;
                    r.rows[j] = o.m[op0];
                    nnz_sum[s] += o.nnz[op];
                }
                x_at += o.k[op0];
                m_at += o.m[op0];
            }
            r.members = j;
            r.m = (int32_t)mt;
            r.plain = 1;
            r.merged_rpt_off = words;
            words += round_up((int)mt + 1, 4);
            r.merged_nz_off = words;
            words += 2 * (int64_t)round_up((int)nnz_sum[s], 4) + (compact_on ? compact_words(M, (int)kxt) : 0);
            recs.push_back(r);
        }
        st.merged_words = words;
        if (words >= (int64_t(1) << 32)) {
            st = bspmm_plan::Stream();
            return;
        }
    }
    auto kx_of = [&](int s) {
        int64_t k = 0;
        for (int g : groups[s]) k += o.k[graphs[g][0]];
        return k;
    };

    // the groups by size; take them while the launch's LDS stays inside the budget
    std::vector<int> order(n_sets);
    for (size_t i = 0; i < n_sets; ++i) order[i] = (int)i;
    // (X has kx rows; Y has m)
    auto words_of = [&](int64_t kx, int64_t csr) { return (int64_t)M * kx * fw + 2 * kx * nx + 2 * csr + 64; };
    auto csr_of = [&](int i) {
        return (int64_t)round_up(recs[i].m + 1, 4) + 2 * (int64_t)round_up((int)nnz_sum[i], 4);
    };
    std::vector<int64_t> kxs(n_sets);
    for (size_t i = 0; i < n_sets; ++i) kxs[i] = kx_of((int)i);
    // (a group that goes through the buffers brings its lists of rows in use)
    auto csr_piped = [&](int i) {
        return csr_of(i) + (compact_on && (int64_t)M * kxs[i] <= kCompactRows ? compact_words(M, (int)kxs[i]) : 0);
    };
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
        return words_of(kxs[a], csr_piped(a)) < words_of(kxs[b], csr_piped(b));
    });
    int64_t kx_cap = 0, csr_cap = 0;
    std::vector<int> mine;
    for (int i : order) {
        const SetRecord& r = recs[i];
        // (more output rows than the gather's passes hold: not through the buffers)
        if (r.m > rows_most || (compact_on && (int64_t)M * kxs[i] > kCompactRows)) continue;
        const int64_t kx = std::max<int64_t>(kx_cap, kxs[i]);
        const int64_t cw = std::max(csr_cap, csr_piped(i));
        if (words_of(kx, cw) > budget_words) continue;    // (a later one may still fit the caps)
        kx_cap = kx;
        csr_cap = cw;
        mine.push_back(i);
    }
    if (mine.empty()) {
        st = bspmm_plan::Stream();
        return;
    }
    st.nx16 = nx16, st.units = units, st.waves = waves, st.fw = fw, st.tiles = tiles;
    st.channels = M;
    st.compact = compact_on;
    if (compact_on)
        for (int i : mine) recs[i].compact = M | ((int32_t)kxs[i] << 8);
    st.tile_words = (int)(M * kx_cap * fw);
    st.x_words = (int)(kx_cap * nx);
    st.csr_words = (int)csr_cap;
    // Larger graphs: taken one at a time, their tile at the start of the same LDS (kernels with
    // two blocks per wavefront: two half tiles of 16 columns, one after the other), the CSR block
    // at its end and at least one 16-row block of X between them; the X buffers are made larger
    // than the listed groups need where that is what it takes, up to the budget.
    std::vector<int> halves;
    if ((units == 2 && fw == 32) || units == 1) {
        const int piece = units == 2 ? 16 : fw;
        const int64_t total = budget_words - 64;
        std::vector<char> is_mine(n_sets, 0);
        for (int i : mine) is_mine[i] = 1;
        auto fits_halves = [&](int i, int64_t csr_room) {
            return csr_of(i) <= csr_room && (int64_t)M * kxs[i] * piece + 16 * nx + csr_room <= total;
        };
        int64_t room = 0;
        for (size_t i = 0; i < n_sets; ++i)
            if (!is_mine[i] && fits_halves((int)i, csr_of((int)i))) room = std::max(room, csr_of((int)i));
        for (size_t i = 0; i < n_sets; ++i)
            if (!is_mine[i] && fits_halves((int)i, room)) halves.push_back((int)i);
        st.big_csr_words = halves.empty() ? 0 : (int)room;
        st.big = (int)halves.size();
        int64_t need = 0;
        for (int i : halves) need = std::max(need, (int64_t)M * kxs[i] * piece + 16 * nx + room);
        const int64_t have = (int64_t)st.tile_words + 2 * st.x_words + 2 * st.csr_words;
        if (need > have) st.x_words += (int)round_up((int)((need - have + 1) / 2), 4);
    }

    // lists: as many workgroups as the chip holds at once, the same lists for every tile
    int per_cu = kn.device_ok ? stream_workgroups_per_cu(nx16, units, waves, st.lds_bytes()) : 0;
    if (per_cu <= 0) per_cu = std::max(1, std::min(3, kMaxLdsBytes / std::max(1, st.lds_bytes())));
    // (a graph taken one at a time stages its X twice and overlaps nothing)
    std::vector<char> in_halves(n_sets, 0);
    for (int i : halves) in_halves[i] = 1;
    // What a trip costs, in units of about a hundred cycles, fitted to per-trip clocks of three
    // launches of 2048 graphs with three workgroups per CU (four channels at n_X = 64: trips of
    // one, two and three 16-row blocks took 5200, 7400 and 15000 cycles; one channel at
    // n_X = 32: 3500 to 11500 for one to four blocks; at n_X = 128: 4900 to 18600 for one to
    // three): a fixed part, the matrix instructions of the wavefront (16-row blocks x n_X / 16
    // x blocks per wavefront), and every pass of the gather after the first, which starts from
    // the row pointers in LDS instead of from registers and costs the more the longer the
    // matrix phases of the workgroups beside it hold the SIMDs.
    const int rows_per_pass_c = threads / (fw / 4);
    const int64_t sw = (int64_t)nx16 * units;      // matrix instructions per 16-row block, in fours
    auto trip_cost = [&](int64_t blocks, int64_t m) {
        const int64_t passes = std::max<int64_t>(1, (m + rows_per_pass_c - 1) / rows_per_pass_c);
        return 20 + 3 * blocks * sw + (20 + 25 * sw / 8) * (passes - 1);
    };
    // (a graph taken one at a time pays for its chunks and pieces without overlap: in the same
    // launches four to eight blocks took 23000 to 41000 cycles with four channels, five to nine
    // blocks 16000 to 36000 with one channel at n_X = 32, three to nine 19000 to 51000 at 128)
    auto cost = [&](int i) {
        const int64_t blocks = (kxs[i] + 15) / 16;
        return in_halves[i] ? std::max<int64_t>(20, 45 * blocks + 10 * sw - 25) : trip_cost(blocks, recs[i].m);
    };
    mine.insert(mine.end(), halves.begin(), halves.end());
    const int lists = (int)std::max<size_t>(1, std::min<size_t>(mine.size(), (size_t)per_cu * kn.compute_units / tiles));
    st.lists = lists;
    std::stable_sort(mine.begin(), mine.end(), [&](int a, int b) { return cost(a) > cost(b); });
    std::vector<std::vector<int>> of_list(lists);
    {
        std::set<std::pair<int64_t, int>> load;      // (cost so far, list)
        for (int l = 0; l < lists; ++l) load.insert({0, l});
        for (int i : mine) {
            auto least = *load.begin();
            load.erase(load.begin());
            of_list[least.second].push_back(i);
            least.first += cost(i);
            load.insert(least);
        }
    }
    st.list.push_back(0);
    std::vector<char> streamed(n_graphs, 0);
    for (int l = 0; l < lists; ++l) {
        // the graphs taken one at a time first: the kernel takes them before it starts its pipeline
        std::stable_partition(of_list[l].begin(), of_list[l].end(), [&](int i) { return in_halves[i] != 0; });
        for (int i : of_list[l]) {
            const SetRecord& r = recs[i];
            const int op0 = graphs[groups[i][0]][0];
            StreamSet e;
            e.in_row = o.in_off[op0];
            e.out_row = o.out_off[op0];
            e.csr_off = (uint32_t)r.merged_rpt_off;
            e.m = r.m;
            e.kx = (int32_t)kxs[i];
            e.nnz = (int32_t)nnz_sum[i];
            st.sets.push_back(e);
            for (int g : groups[i]) streamed[g] = 1;
            st.graphs += (int)groups[i].size();
        }
        st.list.push_back((int32_t)st.sets.size());
    }
    // Every list as the kernel will read it: the graphs it takes one at a time first and
    // inside the room of that mode, every other graph inside the buffers (the kernel's own
    // tests, which decide where its loads and stores go).  A table that fails is not used.
    {
        const int rows_per_pass = threads / (fw / 4);
        const int64_t total = (int64_t)st.tile_words + 2 * st.x_words + 2 * st.csr_words;
        const int piece = units == 2 ? 16 : fw;
        bool ok = true;
        for (int l = 0; l < lists && ok; ++l) {
            bool piped = false;
            for (int j = st.list[l]; j < st.list[l + 1] && ok; ++j) {
                const StreamSet& e = st.sets[j];
                const int64_t csr = (int64_t)round_up(e.m + 1, 4) + 2 * (int64_t)round_up(e.nnz, 4);
                const int64_t lists_words = st.compact ? compact_words(M, e.kx) : 0;
                const bool big = (int64_t)M * e.kx * fw > st.tile_words || (int64_t)e.kx * nx > st.x_words ||
                                 csr + lists_words > st.csr_words || e.m > kStreamPasses * rows_per_pass ||
                                 (st.compact && (int64_t)M * e.kx > kCompactRows);
                ok = e.kx > 0 && e.m > 0;
                if (big) {
                    const int64_t chunk = ((total - st.big_csr_words - (int64_t)M * e.kx * piece) / nx) & ~int64_t(15);
                    ok = ok && !piped && ((units == 2 && fw == 32) || units == 1) && csr <= st.big_csr_words && chunk >= 16;
                } else {
                    piped = true;
                }
            }
        }
        if (!ok) {
            st = bspmm_plan::Stream();
            return;
        }
    }
    // the other graphs: their items of the one-launch schedule, in its order
    for (size_t j = 0; j < sc.items.size(); ++j) {
        const int op = j < sc.item_op.size() ? sc.item_op[j] : -1;
        if (op < (single ? 0 : sc.first_stand_in) || sc.items[j].nrows <= 0) continue;
        if (!streamed[(size_t)(op - (single ? 0 : sc.first_stand_in))]) st.rest.push_back(sc.items[j]);
    }
}

// The item table of the lean kernel for direction d, when the schedule is lean and every offset
// fits the table's 32-bit fields (else the direction keeps the general kernel).
void make_lean_items(bspmm_plan& p, int d)
{
    const Schedule& sc = p.sched[d];
    std::vector<LeanItem>& out = p.lean_items[d];
    out.clear();
    p.lean_blocks[d] = false;
    if (!sc.lean) return;
    out.reserve(sc.items.size());
    constexpr int64_t kLimit = (int64_t)1 << 31;
    int32_t most_k = 0, most_m = 0;
    for (const WorkItem& w : sc.items) {
        LeanItem t;
        std::memset(&t, 0, sizeof t);
        if (w.nrows > 0) {
            if (w.rpt_off >= kLimit || w.nz_off >= kLimit || w.in_row_off >= kLimit ||
                w.out_row_off >= kLimit) {
                out.clear();
                return;
            }
            int sh = 0;
            while ((4 << sh) < w.fw) ++sh;
            t.rpt_off = (uint32_t)w.rpt_off;
            t.nz_off = (uint32_t)w.nz_off;
            t.in_row = (uint32_t)w.in_row_off;
            t.out_row = (uint32_t)w.out_row_off;
            t.m = w.m, t.k = w.k, t.nnz = w.nnz, t.row0 = w.row0, t.nrows = w.nrows, t.f0 = w.f0;
            t.sh = sh;
            if (w.staged & 1) {
                const StagedLayout L = staged_layout(w.m, w.k, w.nnz, w.fw, 0, false);
                t.flags = (w.staged & 2) ? 1 : 0;
                t.cv_byte = 4 * L.cv_off;
                t.b_byte = 4 * L.b_off;
                t.tile_vecs = w.k << sh;
            } else {
                t.flags = 2;    // a row block: its entry range is filled in on the device
                p.lean_blocks[d] = true;
            }
            most_k = std::max(most_k, w.k);
            most_m = std::max(most_m, w.m);
        }
        out.push_back(t);
    }
    p.lean_rows[d] = most_k;
    p.lean_out_rows[d] = most_m;
}

// How the build kernel sorts an operation of `keys` key values, `nnz` entries and payloads below
// `payloads` (rows of a CSR operand, columns of a COO one); `with_rpt` when the input's row
// pointers come along.  Sets r.small and r.scratch_off and returns the LDS words it needs
// (0 when the operation works in global scratch, whose words are added to *scratch_words).
int64_t classify_build(OpRecord& r, int64_t keys, int64_t payloads, int64_t nnz, bool with_rpt,
                       int threads, int64_t* scratch_words)
{
    const int64_t budget = (kBuildLdsBytes - 2048) / 4;
    const int64_t base = keys + 1 + nnz;                     // counters and positions
    const int64_t reg_path = base + (with_rpt ? payloads + 1 : 0);
    auto bits = [](int64_t v) { int b = 0; while (v > 0) { ++b; v >>= 1; } return b; };
    r.scratch_off = -1;
    if (nnz <= (int64_t)build_entries_per_lane(threads) * threads && reg_path <= budget) {
        r.small = 1;     // register path: a few entries per lane, row pointers in LDS too
        return reg_path;
    }
    if (base + nnz <= budget && bits(keys) + bits(std::max<int64_t>(payloads - 1, 0)) <= 32) {
        r.small = 2;     // key and payload of every entry packed into one more LDS word
        return base + nnz;
    }
    r.small = 0;
    if (base <= budget) return base;
    r.scratch_off = *scratch_words;
    *scratch_words += base;
    return 0;
}

// Fill everything of the plan that needs no device.
int plan_host(bspmm_plan& p, const bspmm_batch* b, int32_t F, const Knobs& kn)
{
    const int n = b->batch;
    p.batch = n;
    p.F = F;
    p.knobs = kn;
    DirOps& f = p.dir[0];
    DirOps& t = p.dir[1];
    int64_t rpt_t_words = 0;
    p.records.resize(n);
    p.build_threads = kThreads;
    for (int i = 0; i < n; ++i)
        if (b->nnz[i] > 4 * kThreads) p.build_threads = kBuildThreadsLarge;
    int64_t nz_pack = 0;
    int64_t scratch_words = 0;
    int build_lds_words = 0;
    for (DirOps* o : {&f, &t}) {
        o->m.reserve(n), o->k.reserve(n), o->nnz.reserve(n), o->rpt_off.reserve(n);
        o->nz_off.reserve(n), o->in_off.reserve(n), o->out_off.reserve(n);
    }
    for (int i = 0; i < n; ++i) {
        if (kn.symmetric && b->rows[i] != b->cols[i]) return BSPMM_EINVAL;
        f.m.push_back(b->rows[i]);
        f.k.push_back(b->cols[i]);
        f.nnz.push_back(b->nnz[i]);
        f.rpt_off.push_back(b->rpt_off[i]);
        f.nz_off.push_back(b->nz_off[i]);
        f.in_off.push_back(b->b_row_off[i]);
        f.out_off.push_back(b->c_row_off[i]);
        // transposed: rows and columns swap, dense input is indexed like C, output like B;
        // the transposed entries are packed back to back in operation order
        t.m.push_back(b->cols[i]);
        t.k.push_back(b->rows[i]);
        t.nnz.push_back(b->nnz[i]);
        // (a symmetric operand is its own transpose: the same arrays serve both directions)
        t.rpt_off.push_back(kn.symmetric ? b->rpt_off[i] : rpt_t_words);
        t.nz_off.push_back(kn.symmetric ? b->nz_off[i] : nz_pack);
        t.in_off.push_back(b->c_row_off[i]);
        t.out_off.push_back(b->b_row_off[i]);

        OpRecord& r = p.records[i];
        r.rpt_off = b->rpt_off[i];
        r.nz_off = b->nz_off[i];
        r.rpt_t_off = rpt_t_words;
        r.nz_t_off = nz_pack;
        r.m = b->rows[i];
        r.k = b->cols[i];
        r.nnz = b->nnz[i];
        build_lds_words = std::max<int64_t>(
            build_lds_words,
            classify_build(r, b->cols[i], b->rows[i], b->nnz[i], true, p.build_threads, &scratch_words));
        rpt_t_words += (int64_t)b->cols[i] + 1;
        nz_pack += b->nnz[i];
    }
    p.build_lds_bytes = (int)round_up(build_lds_words * 4 + 16, 256);
    p.scratch_words = scratch_words;

    const int ck = n > 0 ? overlap_kind(b->c_row_off, b->rows, n) : 0;
    const int bk = n > 0 ? overlap_kind(b->b_row_off, b->cols, n) : 0;
    if (ck == 2 || (ck == 1 && !kn.accumulate)) return BSPMM_EOVERLAP;
    p.transposed_supported = bk == 0 || (bk == 1 && kn.accumulate);

    if (kn.front > 0 && (F % 16 != 0 || kn.front % 4 != 0 || kn.hubs || kn.pad != 0))
        return BSPMM_EINVAL;
    p.sched[0] = make_schedule(f, F, kn);
    if (p.sched[0].error) return p.sched[0].error;
    if (kn.front > 0 && kn.accumulate) {
        // the whole layer in one launch: every operation must be a channel of a set, all sets
        // with the same number of channels, the channels of a set sharing the layer input
        const Schedule& sc = p.sched[0];
        size_t in_sets = 0, with_rows = 0;
        for (const auto& mem : sc.merged_sets) {
            if (mem.size() != sc.merged_sets[0].size()) return BSPMM_EINVAL;
            in_sets += mem.size();
        }
        for (int i = 0; i < n; ++i) with_rows += b->rows[i] > 0;
        if (in_sets != with_rows) return sc.fused_tasks > 0 ? BSPMM_ETOOBIG : BSPMM_EINVAL;
        p.front_channels = sc.merged_sets.empty() ? 1 : (int)sc.merged_sets[0].size();
    }
    // Square operations whose input and output blocks sit at the same rows (adjacency matrices
    // of a GCN batch) have the same schedule in both directions: only the location of the
    // CSR arrays differs.
    bool same_shape = kn.front == 0;
    for (int i = 0; i < n && same_shape; ++i)
        same_shape = b->rows[i] == b->cols[i] && b->b_row_off[i] == b->c_row_off[i];
    if (p.transposed_supported && same_shape) {
        p.sched[1] = p.sched[0];
        Schedule& st = p.sched[1];
        for (size_t j = 0; j < st.items.size(); ++j) {
            const int op = st.item_op[j];
            if (op < 0 || op >= n) continue;     // (stand-ins of summed sets: see describe_sets)
            st.items[j].rpt_off = t.rpt_off[op];
            st.items[j].nz_off = t.nz_off[op];
        }
    } else if (p.transposed_supported) {
        Knobs kt = kn;
        kt.front = 0;                     // the layer input is a forward-only guest
        p.sched[1] = make_schedule(t, F, kt);
        if (p.sched[1].error) {          // the forward product still works
            if (kn.need_both && p.sched[1].error == BSPMM_ETOOBIG) return BSPMM_ETOOBIG;
            p.sched[1] = Schedule();
            p.transposed_supported = false;
        }
    }

    // compulsory traffic: CSR once, every distinct dense input block once, every output once
    int64_t csr_f = 0, csr_t = 0, out_f = 0, out_t = 0, in_f = 0, in_t = 0, nnz = 0;
    // a dense block counts once as an input and once as an output, however many operations
    // read it or are summed into it
    auto distinct_rows = [n](const int64_t* off, const int32_t* len) {
        bool increasing = true;        // the usual case: blocks back to back in operation order
        for (int i = 1; i < n && increasing; ++i) increasing = off[i] >= off[i - 1] + len[i - 1];
        int64_t rows = 0;
        if (increasing) {
            for (int i = 0; i < n; ++i) rows += len[i];
            return rows;
        }
        std::vector<std::pair<int64_t, int32_t>> v(n);
        for (int i = 0; i < n; ++i) v[i] = {off[i], len[i]};
        std::sort(v.begin(), v.end());
        for (int i = 0; i < n; ++i)
            if (i == 0 || v[i] != v[i - 1]) rows += v[i].second;
        return rows;
    };
    const int64_t b_rows = distinct_rows(b->b_row_off, b->cols);
    const int64_t c_rows = distinct_rows(b->c_row_off, b->rows);
    in_f = out_t = 4 * b_rows * F;
    in_t = out_f = 4 * c_rows * F;
    for (int i = 0; i < n; ++i) {
        csr_f += 4 * ((int64_t)b->rows[i] + 1) + 8 * (int64_t)b->nnz[i];
        csr_t += 4 * ((int64_t)b->cols[i] + 1) + 8 * (int64_t)b->nnz[i];
        nnz += b->nnz[i];
        if (b->rows[i] > 0 && b->cols[i] > 0) p.reads_dense = true;
    }
    p.effective_bytes[0] = csr_f + in_f + out_f;
    p.effective_bytes[1] = csr_t + in_t + out_t;
    p.flops = 2 * nnz * F;

    // workspace layout
    Layout& L = p.lay;
    size_t at = 0;
    for (int d = 0; d < 2; ++d) {
        L.items[d] = at;
        at = align_up(at + p.sched[d].items.size() * sizeof(WorkItem));
    }
    for (int d = 0; d < 2; ++d) {
        if (d == 1 && p.transposed_supported && same_shape && p.sched[1].items.size() == p.lean_items[0].size() &&
            !p.lean_items[0].empty()) {
            // (the same items again: only the CSR arrays are elsewhere)
            p.lean_items[1] = p.lean_items[0];
            p.lean_blocks[1] = p.lean_blocks[0];
            p.lean_rows[1] = p.lean_rows[0];
            p.lean_out_rows[1] = p.lean_out_rows[0];
            bool fits = true;
            for (size_t j = 0; j < p.lean_items[1].size() && fits; ++j) {
                const WorkItem& w = p.sched[1].items[j];
                if (w.nrows <= 0) continue;
                fits = w.rpt_off < ((int64_t)1 << 31) && w.nz_off < ((int64_t)1 << 31);
                p.lean_items[1][j].rpt_off = (uint32_t)w.rpt_off;
                p.lean_items[1][j].nz_off = (uint32_t)w.nz_off;
            }
            if (!fits) make_lean_items(p, d);
        } else {
            make_lean_items(p, d);
        }
        L.lean[d] = at;
        at = align_up(at + p.lean_items[d].size() * sizeof(LeanItem));
    }
    L.op_records = at;
    at = align_up(at + (size_t)n * sizeof(OpRecord));
    L.build_order = at;
    at = align_up(at + (size_t)n * sizeof(int32_t));
    p.build_order.resize(n);
    for (int i = 0; i < n; ++i) p.build_order[i] = i;
    std::stable_sort(p.build_order.begin(), p.build_order.end(),
                     [b](int32_t x, int32_t y) { return b->nnz[x] > b->nnz[y]; });
    L.rpt_t = at;
    at = align_up(at + (size_t)rpt_t_words * 4);
    L.colids_t = at;
    at = align_up(at + (size_t)nz_pack * 4);
    L.values_t = at;
    at = align_up(at + (size_t)nz_pack * 4);
    L.scratch = at;
    at = align_up(at + (size_t)scratch_words * 4);
    L.flag = at;
    at = align_up(at + 4);
    for (int d = 0; d < 2; ++d) {
        describe_sets(p, d);
        L.sets[d] = at;
        at = align_up(at + p.set_records[d].size() * sizeof(SetRecord));
        L.merged[d] = at;
        at = align_up(at + (size_t)p.merged_words[d] * 4);
    }
    make_stream_plan(p);
    L.stream_records = at;
    at = align_up(at + p.stream.records.size() * sizeof(SetRecord));
    L.stream_merged = at;
    at = align_up(at + (size_t)p.stream.merged_words * 4);
    L.stream_sets = at;
    at = align_up(at + p.stream.sets.size() * sizeof(StreamSet));
    L.stream_list = at;
    at = align_up(at + p.stream.list.size() * sizeof(int32_t));
    L.stream_rest = at;
    at = align_up(at + p.stream.rest.size() * sizeof(WorkItem));
    L.total = at;
    return BSPMM_OK;
}

// What the device says about itself does not change between plans: asked once per
// (device, LDS size, kernel variant) and thread.
struct DeviceFacts {
    int dev = -1, lds_bytes = 0;
    bool hubs = false;
    int cus = 0, resident = 0, resident_slices = 0;
};

const DeviceFacts& device_facts(int lds_bytes, bool hubs)
{
    thread_local DeviceFacts f;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        dev = -2;
    }
    if (f.dev != dev || f.lds_bytes != lds_bytes || f.hubs != hubs) {
        f = DeviceFacts();
        f.dev = dev;
        f.lds_bytes = lds_bytes;
        f.hubs = hubs;
        if (dev >= 0) {
            int cus = 0;
            if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess)
                f.cus = cus;
            else
                (void)hipGetLastError();
            f.resident = bspmm_max_resident_workgroups(lds_bytes, false, hubs);
            f.resident_slices = bspmm_max_resident_workgroups(lds_bytes, true, hubs);
        }
    }
    return f;
}

Knobs knobs_for(const bspmm_options* o, bool ask_device)
{
    Knobs kn = resolve_knobs(o);
    kn.device_ok = ask_device;
    const bool cus_given = o && o->compute_units > 0;
    int r = 0, rs = 0;
    if (ask_device) {
        const DeviceFacts& f = device_facts(kn.lds_words * 4, kn.hubs);
        if (!cus_given && f.cus > 0) kn.compute_units = f.cus;
        r = f.resident;
        rs = f.resident_slices;
    }
    if (!(o && o->target_workgroups > 0)) kn.target_wgs = workgroups_per_cu(kn.front) * kn.compute_units;
    kn.capacity_wgs = r > 0 ? r : 6 * kn.compute_units;
    kn.capacity_wgs_slices = rs > 0 ? rs : 4 * kn.compute_units;
    return kn;
}

// Host planning with the LDS budget the caller gave.  When the caller left it open and the
// batch does not fit the default (operations summed into one block share a workgroup's LDS; an
// operation of the fused front shares it with its layer input), larger budgets are tried
// before the batch is refused: first asking for both directions, then for the forward product
// alone.
template <class Batch, class PlanFn>
int plan_with_budget(bspmm_plan& p, const Batch* b, int32_t F, const bspmm_options* options,
                     bool dry, PlanFn plan_fn)
{
    const bool open = !(options && options->lds_bytes > 0);
    const bool front = options && options->front_features > 0;   // its default is 80 KiB already
    Knobs kn = knobs_for(options, !dry);
    if (open && front && b->batch > 0) {
        // A fused-front launch of several rounds of workgroups: a workgroup goes through its
        // phases (descriptor, staging, matrix cores, gather, store) one after the other, so the
        // launch runs at the rate at which the workgroups of a CU overlap, and a smaller budget
        // (narrower tiles for the operations that need them, four to six workgroups per CU
        // instead of two) is faster.  Measured on MI355X, F = 128, molecule graphs: one channel,
        // 1024 graphs, n_X = 32 / 48 / 64 / 100 / 128: 15.3 -> 13.6, 20.1 -> 16.1, 20.5 -> 19.1,
        // 39.8 -> 28.5, 39.5 -> 32.3 us (384 graphs, n_X = 64: 11.6 -> 8.9 us); whole layers of
        // four channels, n_X = 32: 384 graphs 28.9 -> 21.9 us, 512 graphs 25.2 -> 20.8 us, 2048
        // graphs 76.8 -> 68.3 us.  Launches of one or two rounds (up to 256 graphs) do not change.
        int channels = 1;
        if (options->flags & BSPMM_ACCUMULATE) {
            channels = 0;
            for (int i = 0; i < b->batch; ++i) channels += b->c_row_off[i] == b->c_row_off[0] ? 1 : 0;
        }
        if (b->batch / std::max(1, channels) >= kn.compute_units + kn.compute_units / 2) {
            const int first = channels > 1 ? 52 * 1024 : (options->front_features < 64 ? 24 * 1024 : 40 * 1024);
            const int second = first == 24 * 1024 ? 40 * 1024 : 0;
            for (int bytes : {first, second}) {
                if (bytes == 0) break;
                bspmm_options o = *options;
                o.lds_bytes = bytes;
                Knobs small = knobs_for(&o, !dry);
                small.need_both = false;
                small.lds_given = false;      // (the library's choice, not the caller's)
                p = bspmm_plan();
                const int rc = plan_fn(p, b, F, small);
                if (rc != BSPMM_ETOOBIG) return rc;
            }
            p = bspmm_plan();
        }
    }
    kn.need_both = open && !front;
    int rc = plan_fn(p, b, F, kn);
    if (rc == BSPMM_OK && open && !front && !p.coo_direct && F >= 512 && p.effective_bytes[0] > 28000000 &&
        p.sched[0].grid > kn.capacity_wgs) {
        // Wide feature matrices moved by a launch of more than one round of workgroups, which
        // runs at the rate of the memory system: with 24 KiB the larger operations get tiles of
        // 32 columns (row segments of 128 bytes), each staging the operation's CSR again.  A
        // budget of a third of a CU's LDS doubles the tiles; it is kept when the launch then
        // takes at most a tenth more rounds than before, since three workgroups per CU are resident
        // instead of six (measured, 128 graphs of 20-100 nodes: F = 1024, six seeds, 1.35-1.45
        // rounds before and 1.39-1.47 after, 14.3-15.2 -> 13.4-14.4 us, 4.24-4.34 -> 4.49-4.56 TB/s;
        // F = 512, 0.71 -> 1.33 rounds, 7.46 -> 8.79 us: not taken; 1024 graphs of 25 nodes at
        // F = 512, 2.19 -> 2.82 rounds, 21.0 -> 21.3 us: not taken).
        bspmm_options o = options ? *options : bspmm_options{};
        o.lds_bytes = 53248;
        Knobs wide = knobs_for(&o, !dry);
        if (dry) wide.capacity_wgs = 3 * wide.compute_units;
        wide.need_both = kn.need_both;
        wide.lds_given = false;
        bspmm_plan q;
        if (plan_fn(q, b, F, wide) == BSPMM_OK &&
            10 * (int64_t)q.sched[0].grid * kn.capacity_wgs <= 11 * (int64_t)p.sched[0].grid * wide.capacity_wgs)
            p = std::move(q);
        return BSPMM_OK;
    }
    if (rc != BSPMM_ETOOBIG || !open) return rc;
    static const struct { int bytes; bool both; } attempts[] = {
        {kHalfLdsBytes, true}, {kMaxLdsBytes, true}, {0, false}, {kHalfLdsBytes, false}, {kMaxLdsBytes, false}};
    for (const auto& a : attempts) {
        if (front && !(a.bytes == kMaxLdsBytes && !a.both)) continue;
        bspmm_options o = options ? *options : bspmm_options{};
        o.lds_bytes = a.bytes;
        kn = knobs_for(&o, !dry);
        kn.need_both = a.both;
        kn.lds_given = false;
        p = bspmm_plan();
        rc = plan_fn(p, b, F, kn);
        if (rc != BSPMM_ETOOBIG) return rc;
    }
    return rc;
}

// A one-off build recorded into a stream capture runs when the graph is replayed, not now: the
// plan must not count it as done (a later eager run builds again; the graph keeps its copy).
bool capturing(hipStream_t s)
{
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &st) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return st == hipStreamCaptureStatusActive;
}

int enqueue_build(bspmm_plan* p, hipStream_t s)
{
    if (p->transposed_built || p->knobs.symmetric) return BSPMM_OK;
    hipError_t e = launch_build_transpose(
        reinterpret_cast<const OpRecord*>(p->ws + p->lay.op_records), p->batch,
        p->build_threads, p->build_lds_bytes, p->rpt, p->colids, p->values,
        reinterpret_cast<int32_t*>(p->ws + p->lay.rpt_t),
        reinterpret_cast<int32_t*>(p->ws + p->lay.colids_t),
        reinterpret_cast<float*>(p->ws + p->lay.values_t),
        reinterpret_cast<int32_t*>(p->ws + p->lay.scratch),
        reinterpret_cast<const int32_t*>(p->ws + p->lay.build_order), s);
    if (e != hipSuccess) return hip_fail(e);
    p->transposed_built = !capturing(s);
    return BSPMM_OK;
}

// The merged CSR of the summed sets of direction d (once per plan; for d = 1 after the
// transposed CSR has been built).
int enqueue_merge(bspmm_plan* p, int d, hipStream_t s)
{
    if (p->merged_built[d] || p->set_records[d].empty()) return BSPMM_OK;
    const bool own = d == 0 || p->knobs.symmetric;
    const int32_t* rpt = own ? p->rpt : reinterpret_cast<const int32_t*>(p->ws + p->lay.rpt_t);
    const int32_t* colids = own ? p->colids : reinterpret_cast<const int32_t*>(p->ws + p->lay.colids_t);
    const float* values = own ? p->values : reinterpret_cast<const float*>(p->ws + p->lay.values_t);
    hipError_t e = launch_merge_sets(reinterpret_cast<const SetRecord*>(p->ws + p->lay.sets[d]),
                                     (int)p->set_records[d].size(), rpt, colids, values,
                                     reinterpret_cast<int32_t*>(p->ws + p->lay.merged[d]), s);
    if (e != hipSuccess) return hip_fail(e);
    p->merged_built[d] = !capturing(s);
    return BSPMM_OK;
}

// CSR arrays a run of direction d reads.
void csr_of_direction(const bspmm_plan* p, int d, const int32_t** rpt, const int32_t** colids,
                      const float** values)
{
    if (d == 0 || p->knobs.symmetric) {
        *rpt = p->rpt;
        *colids = p->colids;
        *values = p->values;
    } else {
        *rpt = reinterpret_cast<const int32_t*>(p->ws + p->lay.rpt_t);
        *colids = reinterpret_cast<const int32_t*>(p->ws + p->lay.colids_t);
        *values = reinterpret_cast<const float*>(p->ws + p->lay.values_t);
    }
}

// The merged CSR blocks of the groups of the streaming launch (once per plan).
int enqueue_stream_merge(bspmm_plan* p, hipStream_t s)
{
    if (p->stream.merged_built || !p->stream.on()) return BSPMM_OK;
    hipError_t e = launch_merge_sets(reinterpret_cast<const SetRecord*>(p->ws + p->lay.stream_records),
                                     (int)p->stream.records.size(), p->rpt, p->colids, p->values,
                                     reinterpret_cast<int32_t*>(p->ws + p->lay.stream_merged), s);
    if (e != hipSuccess) return hip_fail(e);
    p->stream.merged_built = !capturing(s);
    return BSPMM_OK;
}

// Row blocks of the generic bin in a lean table: the device writes each block's entry range
// into its item (once per plan and direction; for d = 1 after the transposed CSR is built).
int enqueue_hints(bspmm_plan* p, int d, hipStream_t s)
{
    if (p->lean_hints_built[d] || !p->lean_blocks[d] || p->lean_items[d].empty()) return BSPMM_OK;
    const int32_t* rpt;
    const int32_t* colids;
    const float* values;
    csr_of_direction(p, d, &rpt, &colids, &values);
    hipError_t e = launch_lean_hints(reinterpret_cast<LeanItem*>(p->ws + p->lay.lean[d]),
                                     (int)p->lean_items[d].size(), rpt, s);
    if (e != hipSuccess) return hip_fail(e);
    p->lean_hints_built[d] = !capturing(s);
    return BSPMM_OK;
}

int run_direction(bspmm_plan* p, int d, const float* in, float* out, int64_t ld_in,
                  int64_t ld_out, hipStream_t s)
{
    if (p->coo_direct) {
        const CooSchedule& cs = p->coo_sched[d];
        if (cs.items.empty()) return BSPMM_OK;
        if ((!in && p->reads_dense) || !out || ld_in < p->F || ld_out < p->F) return BSPMM_EINVAL;
        CooLaunchParams C;
        C.items = reinterpret_cast<const CooItem*>(p->ws + p->lay.items[d]);
        C.ids = p->ids;
        C.values = p->coo_values;
        C.in = in;
        C.out = out;
        C.ld_in = ld_in;
        C.ld_out = ld_out;
        C.transposed = d;
        const bool v4 = p->F % 4 == 0 && ld_in % 4 == 0 && ld_out % 4 == 0 &&
                        (reinterpret_cast<uintptr_t>(in) & 15) == 0 &&
                        (reinterpret_cast<uintptr_t>(out) & 15) == 0;
        hipError_t ce = launch_bspmm_coo(C, (int)cs.items.size(), cs.lds_words * 4, v4, s);
        return ce == hipSuccess ? BSPMM_OK : hip_fail(ce);
    }
    const Schedule& sc = p->sched[d];
    if (sc.grid == 0) return BSPMM_OK;
    // when no operation has both rows and columns nothing is read: the input may have no rows at all
    if ((!in && p->reads_dense) || !out || ld_in < p->F || ld_out < p->F) return BSPMM_EINVAL;
    const int mrc = enqueue_merge(p, d, s);
    if (mrc != BSPMM_OK) return mrc;
    LaunchParams P;
    P.items = reinterpret_cast<const WorkItem*>(p->ws + p->lay.items[d]);
    csr_of_direction(p, d, &P.rpt, &P.colids, &P.values);
    P.in = in;
    P.out = out;
    P.ld_in = ld_in;
    P.ld_out = ld_out;
    for (int r = 0; r < kRanges; ++r) {
        P.wg_end[r] = sc.wg_end[r];
        P.item_base[r] = sc.item_base[r];
    }
    P.n_tasks = sc.grid;
    P.fused_stride = sc.fused_stride;
    P.lds_floats = p->knobs.lds_words;
    P.pad = p->knobs.pad;
    P.w = reinterpret_cast<const float*>(p->ws + p->lay.merged[d]);   // see LaunchParams
    P.bias = nullptr;
    P.ld_w = 0;
    P.n_front = 0;
    P.accumulate = 0;
    const bool vec4 = p->F % 4 == 0 && ld_in % 4 == 0 && ld_out % 4 == 0 &&
                      (reinterpret_cast<uintptr_t>(in) & 15) == 0 &&
                      (reinterpret_cast<uintptr_t>(out) & 15) == 0;
    // the lean kernel forms 32-bit byte offsets inside an operation's dense blocks and multiplies
    // in 24 bits: leading dimensions below 4 Mi floats, blocks below 4 GiB
    constexpr int64_t kMul24 = (int64_t)1 << 22, kOff32 = (int64_t)1 << 30;
    const bool lean = vec4 && !p->lean_items[d].empty() && ld_in < kMul24 && ld_out < kMul24 &&
                      (int64_t)p->lean_rows[d] * ld_in < kOff32 &&
                      (int64_t)p->lean_out_rows[d] * ld_out < kOff32;
    if (lean) {
        const int hrc = enqueue_hints(p, d, s);
        if (hrc != BSPMM_OK) return hrc;
    }
    hipError_t e = lean
        ? launch_bspmm_lean(reinterpret_cast<const LeanItem*>(p->ws + p->lay.lean[d]), P,
                            sc.launch_grid, p->knobs.lds_words * 4, s)
        : launch_bspmm(P, sc.launch_grid, p->knobs.lds_words * 4, vec4, sc.has_slices,
                       p->knobs.hubs, !sc.merged_sets.empty(), s);
    return e == hipSuccess ? BSPMM_OK : hip_fail(e);
}

int check_coo_batch(const bspmm_coo_batch* b, int32_t F, bool need_device)
{
    if (!b || F <= 0 || b->batch < 0) return BSPMM_EINVAL;
    if (b->batch == 0) return BSPMM_OK;
    if (!b->rows || !b->cols || !b->nnz || !b->nz_off || !b->b_row_off || !b->c_row_off)
        return BSPMM_EINVAL;
    int64_t total_nnz = 0;
    for (int i = 0; i < b->batch; ++i) {
        if (b->rows[i] < 0 || b->cols[i] < 0 || b->nnz[i] < 0) return BSPMM_EINVAL;
        if (b->nz_off[i] < 0 || b->b_row_off[i] < 0 || b->c_row_off[i] < 0) return BSPMM_EINVAL;
        if ((b->rows[i] == 0 || b->cols[i] == 0) && b->nnz[i] != 0) return BSPMM_EINVAL;
        total_nnz += b->nnz[i];
    }
    if (need_device && total_nnz > 0 && (!b->ids || !b->values)) return BSPMM_EINVAL;
    return BSPMM_OK;
}

// Plan of the direct COO kernel: two item tables (forward, transposed), the validation
// records and the flag word; no CSR, no build.
int plan_host_coo_direct(bspmm_plan& p, const bspmm_coo_batch* b, int32_t F, const Knobs& kn)
{
    const int n = b->batch;
    if (kn.accumulate || kn.hubs) return BSPMM_EINVAL;
    p.batch = n;
    p.F = F;
    p.knobs = kn;
    p.from_coo = true;
    p.coo_direct = true;
    DirOps& f = p.dir[0];
    DirOps& t = p.dir[1];
    int64_t nnz = 0, in_f = 0, out_f = 0;
    std::set<std::pair<int64_t, int32_t>> blocks_b;
    for (DirOps* o : {&f, &t}) {
        o->m.reserve(n), o->k.reserve(n), o->nnz.reserve(n), o->rpt_off.reserve(n);
        o->nz_off.reserve(n), o->in_off.reserve(n), o->out_off.reserve(n);
    }
    for (int i = 0; i < n; ++i) {
        if (kn.symmetric && b->rows[i] != b->cols[i]) return BSPMM_EINVAL;
        f.m.push_back(b->rows[i]);
        f.k.push_back(b->cols[i]);
        t.m.push_back(b->cols[i]);
        t.k.push_back(b->rows[i]);
        for (DirOps* d : {&f, &t}) {
            d->nnz.push_back(b->nnz[i]);
            d->rpt_off.push_back(0);
            d->nz_off.push_back(b->nz_off[i]);
        }
        f.in_off.push_back(b->b_row_off[i]);
        f.out_off.push_back(b->c_row_off[i]);
        t.in_off.push_back(b->c_row_off[i]);
        t.out_off.push_back(b->b_row_off[i]);
        nnz += b->nnz[i];
        if (b->rows[i] > 0 && b->cols[i] > 0) p.reads_dense = true;
        if (blocks_b.emplace(b->b_row_off[i], b->cols[i]).second) in_f += 4 * (int64_t)b->cols[i] * F;
        out_f += 4 * (int64_t)b->rows[i] * F;
    }
    if (n > 0 && overlap_kind(b->c_row_off, b->rows, n) != 0) return BSPMM_EOVERLAP;
    p.transposed_supported = n == 0 || overlap_kind(b->b_row_off, b->cols, n) == 0;
    p.coo_sched[0] = make_coo_schedule(f, F, kn);
    if (p.transposed_supported) p.coo_sched[1] = make_coo_schedule(t, F, kn);
    // compulsory traffic: every entry once (two indices and a value), distinct dense inputs
    // once, outputs once
    p.effective_bytes[0] = 12 * nnz + in_f + out_f;
    p.effective_bytes[1] = 12 * nnz + out_f + in_f;
    p.flops = 2 * nnz * F;
    Layout& L = p.lay;
    size_t at = 0;
    for (int d = 0; d < 2; ++d) {
        L.items[d] = at;
        at = align_up(at + p.coo_sched[d].items.size() * sizeof(CooItem));
    }
    L.coo_records = at;
    at = align_up(at + (size_t)n * sizeof(OpRecord));
    L.flag = at;
    at = align_up(at + 4);
    L.total = at;
    return BSPMM_OK;
}

// Plan for COO operands: the CSR arrays (row pointers and entries packed back to back in
// operation order) are built inside the workspace, and everything else is the CSR plan of them.
int plan_host_coo(bspmm_plan& p, const bspmm_coo_batch* b, int32_t F, const Knobs& kn)
{
    const int n = b->batch;
    std::vector<int64_t> rpt_off(n), nz_pack(n);
    int64_t rpt_words = 0, nz = 0, scratch_words = 0, lds_words = 0;
    p.coo_records.resize(n);
    int threads = kThreads;
    for (int i = 0; i < n; ++i)
        if (b->nnz[i] > 4 * kThreads) threads = kBuildThreadsLarge;
    for (int i = 0; i < n; ++i) {
        rpt_off[i] = rpt_words;
        nz_pack[i] = nz;
        OpRecord& r = p.coo_records[i];
        r.rpt_off = 0;
        r.nz_off = b->nz_off[i];          // where the caller's pairs and values sit
        r.rpt_t_off = rpt_words;          // where the built row pointers go
        r.nz_t_off = nz;                  // where the built entries go
        r.m = b->cols[i];                 // bound of the payload (column)
        r.k = b->rows[i];                 // number of keys (rows)
        r.nnz = b->nnz[i];
        lds_words = std::max(lds_words, classify_build(r, b->rows[i], b->cols[i], b->nnz[i], false,
                                                       threads, &scratch_words));
        rpt_words += (int64_t)b->rows[i] + 1;
        nz += b->nnz[i];
    }
    if (kn.coo_direct) return plan_host_coo_direct(p, b, F, kn);
    bspmm_batch ib;
    ib.batch = n;
    ib.rows = b->rows;
    ib.cols = b->cols;
    ib.nnz = b->nnz;
    ib.rpt_off = rpt_off.data();
    ib.nz_off = nz_pack.data();
    ib.b_row_off = b->b_row_off;
    ib.c_row_off = b->c_row_off;
    ib.rpt = nullptr;
    ib.colids = nullptr;
    ib.values = nullptr;
    const int rc = plan_host(p, &ib, F, kn);
    if (rc != BSPMM_OK) return rc;
    p.from_coo = true;
    p.coo_build_lds_bytes = (int)round_up(lds_words * 4 + 16, 256);
    p.csr_rpt_words = rpt_words;
    p.csr_nz = nz;
    p.coo_scratch_words = scratch_words;
    Layout& L = p.lay;
    size_t at = L.total;
    L.coo_records = at;
    at = align_up(at + (size_t)n * sizeof(OpRecord));
    L.csr_rpt = at;
    at = align_up(at + (size_t)rpt_words * 4);
    L.csr_colids = at;
    at = align_up(at + (size_t)nz * 4);
    L.csr_values = at;
    at = align_up(at + (size_t)nz * 4);
    L.coo_scratch = at;
    at = align_up(at + (size_t)scratch_words * 4);
    L.total = at;
    return BSPMM_OK;
}

// Device half of plan creation: tables to the workspace, conversions enqueued on `s`.
int upload_plan(bspmm_plan* p, const bspmm_options* options, void* workspace,
                size_t workspace_bytes, hipStream_t s)
{
    // The one-launch layer kernel's workgroup size, decided here (plans made by
    // bspmm_workspace_bytes never asked the device) and not in the first run, which may be
    // inside a stream capture.  A launch of up to two workgroups per CU lasts as long as its
    // largest item, and workgroups of eight wavefronts halve that item's matrix blocks per
    // wavefront and the passes of its gather.  Measured on 256 CUs, F = 128, four against eight
    // wavefronts: one channel at n_X = 64, 32 graphs (320 workgroups) 6.4 -> 5.1 us; n_X = 128,
    // 128 graphs (312) 9.3 -> 8.7; four channels at n_X = 64, 64 graphs (512) 9.3 -> 7.9, 32
    // graphs 7.1 -> 6.2.  Beyond two per CU the launch of twice the wavefronts costs more than it
    // gains (128 graphs at n_X = 64, 544 workgroups: 6.6 -> 6.9 us; four channels, 1024
    // workgroups: 11.9 -> 12.3).
    p->front_wide = 0;
    if (p->knobs.front > 0) {
        const Schedule& sc = p->sched[0];
        const int64_t grid = p->stream.on() ? (int64_t)p->stream.rest.size() : sc.grid;
        const int per_cu = std::min(2, front_workgroups_per_cu(!sc.merged_sets.empty(), true, sc.front_lds_words * 4));
        p->front_wide = grid > 0 && grid <= (int64_t)per_cu * p->knobs.compute_units ? 1 : 0;
    }
    if (options && (options->flags & BSPMM_FLOOR_PROBE))
        for (int d = 0; d < 2; ++d) {
            for (WorkItem& w : p->sched[d].items) w.nrows = w.m = w.k = w.nnz = 0;
            for (LeanItem& w : p->lean_items[d])
                w.nrows = w.m = w.k = w.nnz = w.tile_vecs = w.count = w.flags = w.b_byte = 0;
            for (CooItem& w : p->coo_sched[d].items) w.nrows = w.nnz = 0;
        }
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0)
        return BSPMM_EINVAL;
    if (workspace_bytes < p->lay.total) return BSPMM_ENOSPACE;
    p->ws = static_cast<char*>(workspace);
    // The host tables stay alive inside the plan, so the asynchronous copies may read them
    // at any time before bspmm_destroy.
    hipError_t e = hipSuccess;
    if (!p->coo_direct) {
        // The item tables of both directions and the operation records sit back to back at the
        // front of the workspace: one copy from one host image of that stretch (every copy from
        // pageable memory costs several microseconds of host time, whatever its size).
        const size_t bytes = p->lay.build_order + p->build_order.size() * sizeof(int32_t);
        p->tables.assign(bytes, 0);
        for (int d = 0; d < 2; ++d)
            if (!p->sched[d].items.empty())
                std::memcpy(p->tables.data() + p->lay.items[d], p->sched[d].items.data(),
                            p->sched[d].items.size() * sizeof(WorkItem));
        for (int d = 0; d < 2; ++d)
            if (!p->lean_items[d].empty())
                std::memcpy(p->tables.data() + p->lay.lean[d], p->lean_items[d].data(),
                            p->lean_items[d].size() * sizeof(LeanItem));
        if (!p->records.empty())
            std::memcpy(p->tables.data() + p->lay.op_records, p->records.data(),
                        p->records.size() * sizeof(OpRecord));
        if (!p->build_order.empty())
            std::memcpy(p->tables.data() + p->lay.build_order, p->build_order.data(),
                        p->build_order.size() * sizeof(int32_t));
        if (bytes > 0)
            e = hipMemcpyAsync(p->ws, p->tables.data(), bytes, hipMemcpyHostToDevice, s);
    }
    for (int d = 0; d < 2 && e == hipSuccess; ++d)
        if (!p->set_records[d].empty())
            e = hipMemcpyAsync(p->ws + p->lay.sets[d], p->set_records[d].data(),
                               p->set_records[d].size() * sizeof(SetRecord), hipMemcpyHostToDevice, s);
    if (e == hipSuccess && p->stream.on()) {
        e = hipMemcpyAsync(p->ws + p->lay.stream_records, p->stream.records.data(),
                           p->stream.records.size() * sizeof(SetRecord), hipMemcpyHostToDevice, s);
        if (e == hipSuccess)
        e = hipMemcpyAsync(p->ws + p->lay.stream_sets, p->stream.sets.data(),
                           p->stream.sets.size() * sizeof(StreamSet), hipMemcpyHostToDevice, s);
        if (e == hipSuccess)
            e = hipMemcpyAsync(p->ws + p->lay.stream_list, p->stream.list.data(),
                               p->stream.list.size() * sizeof(int32_t), hipMemcpyHostToDevice, s);
        if (e == hipSuccess && !p->stream.rest.empty())
            e = hipMemcpyAsync(p->ws + p->lay.stream_rest, p->stream.rest.data(),
                               p->stream.rest.size() * sizeof(WorkItem), hipMemcpyHostToDevice, s);
    }
    if (p->coo_direct) {
        for (int d = 0; d < 2 && e == hipSuccess; ++d)
            if (!p->coo_sched[d].items.empty())
                e = hipMemcpyAsync(p->ws + p->lay.items[d], p->coo_sched[d].items.data(),
                                   p->coo_sched[d].items.size() * sizeof(CooItem),
                                   hipMemcpyHostToDevice, s);
        if (e == hipSuccess && !p->coo_records.empty())
            e = hipMemcpyAsync(p->ws + p->lay.coo_records, p->coo_records.data(),
                               p->coo_records.size() * sizeof(OpRecord), hipMemcpyHostToDevice, s);
        return e == hipSuccess ? BSPMM_OK : hip_fail(e);
    }
    if (e == hipSuccess && p->from_coo) {
        int32_t* rpt = reinterpret_cast<int32_t*>(p->ws + p->lay.csr_rpt);
        int32_t* colids = reinterpret_cast<int32_t*>(p->ws + p->lay.csr_colids);
        float* values = reinterpret_cast<float*>(p->ws + p->lay.csr_values);
        p->rpt = rpt;
        p->colids = colids;
        p->values = values;
        if (!p->coo_records.empty()) {
            e = hipMemcpyAsync(p->ws + p->lay.coo_records, p->coo_records.data(),
                               p->coo_records.size() * sizeof(OpRecord), hipMemcpyHostToDevice, s);
            if (e == hipSuccess)
                e = launch_build_from_coo(
                    reinterpret_cast<const OpRecord*>(p->ws + p->lay.coo_records), p->batch,
                    p->build_threads, p->coo_build_lds_bytes, p->ids, p->coo_values, rpt, colids, values,
                    reinterpret_cast<int32_t*>(p->ws + p->lay.coo_scratch),
                    reinterpret_cast<const int32_t*>(p->ws + p->lay.build_order), s);
        }
    }
    if (e != hipSuccess) return hip_fail(e);
    if (options && (options->flags & BSPMM_BUILD_TRANSPOSE)) {
        int rc = enqueue_merge(p, 0, s);
        if (rc == BSPMM_OK) rc = enqueue_stream_merge(p, s);
        if (rc == BSPMM_OK && p->transposed_supported) rc = enqueue_build(p, s);
        if (rc == BSPMM_OK && p->transposed_supported) rc = enqueue_merge(p, 1, s);
        if (rc == BSPMM_OK) rc = enqueue_hints(p, 0, s);
        if (rc == BSPMM_OK && p->transposed_supported) rc = enqueue_hints(p, 1, s);
        return rc;
    }
    return BSPMM_OK;
}

// One channel of the graph-convolution layer: the forward schedule with the dense tile made
// on chip from X_i, W and bias.
int run_gcn(bspmm_plan* p, const float* X, int64_t ldx, const float* W, int64_t ldw,
            const float* bias, float* Y, int64_t ldy, int accumulate, hipStream_t s)
{
    const Schedule& sc = p->sched[0];
    if (sc.grid == 0) return BSPMM_OK;
    const int nx = p->knobs.front;
    auto misaligned = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15) != 0; };
    if (!X || !W || !bias || !Y || ldx < nx || ldw < p->F || ldy < p->F) return BSPMM_EINVAL;
    if (ldx % 4 || ldw % 4 || ldy % 4 || misaligned(X) || misaligned(W) || misaligned(Y))
        return BSPMM_EINVAL;
    const bool sets = !sc.merged_sets.empty();
    if (p->stream.on()) {
        const int mrc = enqueue_stream_merge(p, s);
        if (mrc != BSPMM_OK) return mrc;
    }
    if (sets && (!p->stream.on() || !p->stream.rest.empty())) {
        const int mrc = enqueue_merge(p, 0, s);
        if (mrc != BSPMM_OK) return mrc;
    }
    const bspmm_plan::Stream& st = p->stream;
    if (st.on()) {
        // graphs inside the LDS budget: resident workgroups stream them; the others (if any)
        // follow in a launch of the one-launch kernel over their items
        if (ldx >= (int64_t(1) << 31) || ldy >= (int64_t(1) << 31)) return BSPMM_EINVAL;
        StreamParams S;
        S.sets = reinterpret_cast<const StreamSet*>(p->ws + p->lay.stream_sets);
        S.list = reinterpret_cast<const int32_t*>(p->ws + p->lay.stream_list);
        S.merged = reinterpret_cast<const int32_t*>(p->ws + p->lay.stream_merged);
        S.x = X;
        S.w = W;
        S.bias = bias;
        S.y = Y;
        StreamShape& sh = S.shape;
        sh.ld_x = ldx, sh.ld_w = ldw, sh.ld_y = ldy, sh.bias_stride = p->F;
        sh.tiles = st.tiles, sh.fw = st.fw, sh.channels = st.channels;
        sh.accumulate = accumulate ? 1 : 0;
        sh.tile_words = st.tile_words, sh.x_words = st.x_words, sh.csr_words = st.csr_words;
        sh.big_csr_words = st.big_csr_words;
        sh.lists = st.lists;
        sh.compact = st.compact ? 1 : 0;
        sh.real_channels = sets ? p->front_channels : 1;
        sh.reserved_ = 0;
        const hipError_t es = launch_bspmm_gcn_stream(S, st.nx16, st.units, st.waves, (st.lists + 7) / 8 * 8 * st.tiles,
                                                      st.lds_bytes(), s);
        if (es != hipSuccess) return hip_fail(es);
        if (st.rest.empty()) return BSPMM_OK;
    }
    LaunchParams P;
    P.items = st.on() ? reinterpret_cast<const WorkItem*>(p->ws + p->lay.stream_rest)
                      : reinterpret_cast<const WorkItem*>(p->ws + p->lay.items[0]);
    // (channel sets: every item reads the merged CSR of its set; P.rpt carries its base)
    P.rpt = sets ? reinterpret_cast<const int32_t*>(p->ws + p->lay.merged[0]) : p->rpt;
    P.colids = p->colids;
    P.values = p->values;
    P.in = X;
    P.out = Y;
    P.ld_in = ldx;
    P.ld_out = ldy;
    for (int r = 0; r < kRanges; ++r) {
        P.wg_end[r] = sc.wg_end[r];
        P.item_base[r] = sc.item_base[r];
    }
    P.n_tasks = sc.grid;
    P.fused_stride = p->F;                 // this launch: floats between the channels' bias rows
    P.lds_floats = sc.front_lds_words;     // what the launch gets: decides the rows of X_i per pass
    P.pad = 0;
    P.w = W;
    P.bias = bias;
    P.ld_w = ldw;
    P.n_front = nx;
    P.accumulate = accumulate ? 1 : 0;
    const int grid = st.on() ? (int)st.rest.size() : sc.grid;
    hipError_t e = launch_bspmm_gcn(P, grid, sc.front_lds_words * 4, accumulate != 0, sets, p->front_wide == 1, s);
    return e == hipSuccess ? BSPMM_OK : hip_fail(e);
}

// The static workspace of the current device.  Its device address is asked for once per device
// (with that device current) and kept; every later use goes through the kept pointer.  The
// generation counts the plans handed out on a device: only the latest owns the array.
constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
void* g_static_ptr[kMaxDevices] = {};
std::atomic<uint64_t> g_static_generation[kMaxDevices];

int static_workspace(int* device, void** ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return BSPMM_EINVAL;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void* q = nullptr;
        e = hipGetSymbolAddress(&q, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (!q || (reinterpret_cast<uintptr_t>(q) & (kAlign - 1)) != 0) return BSPMM_EINVAL;
        g_static_ptr[dev] = q;
    }
    *device = dev;
    *ptr = g_static_ptr[dev];
    return BSPMM_OK;
}

// A plan made by bspmm_create_static that a later one on the same device has displaced must
// not run: the tables it points at are no longer its own.
bool displaced(const bspmm_plan* p)
{
    return p->static_device >= 0 &&
           g_static_generation[p->static_device].load(std::memory_order_acquire) != p->static_generation;
}

// bspmm_workspace_bytes has to schedule the batch to know the size; a bspmm_create that follows
// on the same thread with the same arguments takes that plan over instead of scheduling again.
// "The same" is checked on the values themselves: F, the options, and every host array of the
// batch against what the remembered plan was made from.
struct PlanKey {
    int32_t batch = -1, F = 0;
    bool coo = false, has_options = false;
    bspmm_options options;
};

thread_local std::unique_ptr<bspmm_plan> t_memo;
thread_local PlanKey t_memo_key;

PlanKey make_key(int32_t batch, int32_t F, const bspmm_options* o, bool coo)
{
    PlanKey k;
    k.batch = batch;
    k.F = F;
    k.coo = coo;
    k.has_options = o != nullptr;
    std::memset(&k.options, 0, sizeof(k.options));
    if (o) k.options = *o;
    return k;
}

void remember(bspmm_plan* p, const PlanKey& k)
{
    t_memo.reset(p);
    t_memo_key = k;
}

// The remembered plan, if it was made from exactly this batch.  `rpt_off` is null for COO batches
// (their plans keep the row-pointer offsets the library chose itself).
template <class Batch>
bspmm_plan* recall(const PlanKey& k, const Batch* b, const int64_t* rpt_off)
{
    if (!t_memo) return nullptr;
    const PlanKey& m = t_memo_key;
    if (m.batch != k.batch || m.F != k.F || m.coo != k.coo || m.has_options != k.has_options ||
        std::memcmp(&m.options, &k.options, sizeof(k.options)) != 0)
        return nullptr;
    const bspmm_plan& p = *t_memo;
    const DirOps& f = p.dir[0];
    const size_t n = (size_t)k.batch;
    if (p.batch != k.batch || f.m.size() != n) return nullptr;
    auto same = [n](const auto& kept, const auto* given) {
        return std::memcmp(kept.data(), given, n * sizeof(*given)) == 0;
    };
    if (!same(f.m, b->rows) || !same(f.k, b->cols) || !same(f.nnz, b->nnz) ||
        !same(f.in_off, b->b_row_off) || !same(f.out_off, b->c_row_off))
        return nullptr;
    if (rpt_off) {
        if (!same(f.rpt_off, rpt_off) || !same(f.nz_off, b->nz_off)) return nullptr;
    } else {
        for (size_t i = 0; i < n; ++i)
            if (p.coo_records[i].nz_off != b->nz_off[i]) return nullptr;
    }
    return t_memo.release();
}

}  // namespace

extern "C" {

int bspmm_workspace_bytes(const bspmm_batch* b, int32_t F, const bspmm_options* options,
                          size_t* bytes)
{
    if (!bytes) return BSPMM_EINVAL;
    *bytes = 0;
    int rc = check_batch(b, F, false);
    if (rc != BSPMM_OK) return rc;
    bspmm_plan* p = new (std::nothrow) bspmm_plan;
    if (!p) return BSPMM_EINVAL;
    const bool dry = options && (options->flags & BSPMM_DRY_RUN);
    rc = plan_with_budget(*p, b, F, options, dry, plan_host);
    if (rc != BSPMM_OK) {
        delete p;
        return rc;
    }
    *bytes = p->lay.total;
    remember(p, make_key(b->batch, F, options, false));
    return BSPMM_OK;
}

int bspmm_create(bspmm_plan** plan, const bspmm_batch* b, int32_t F,
                 const bspmm_options* options, void* workspace, size_t workspace_bytes,
                 void* stream)
{
    if (!plan) return BSPMM_EINVAL;
    *plan = nullptr;
    const bool dry = options && (options->flags & BSPMM_DRY_RUN);
    int rc = check_batch(b, F, !dry);
    if (rc != BSPMM_OK) return rc;
    bspmm_plan* p = b->batch > 0 ? recall(make_key(b->batch, F, options, false), b, b->rpt_off) : nullptr;
    if (!p) {
        p = new (std::nothrow) bspmm_plan;
        if (!p) return BSPMM_EINVAL;
        rc = plan_with_budget(*p, b, F, options, dry, plan_host);
    }
    p->dry = dry;
    if (rc == BSPMM_OK && !dry) {
        p->rpt = b->rpt;
        p->colids = b->colids;
        p->values = b->values;
        rc = upload_plan(p, options, workspace, workspace_bytes, static_cast<hipStream_t>(stream));
    }
    if (rc != BSPMM_OK) {
        delete p;
        return rc;
    }
    *plan = p;
    return BSPMM_OK;
}

int bspmm_create_static(bspmm_plan** plan, const bspmm_batch* b, int32_t F,
                        const bspmm_options* options, void* stream)
{
    if (!plan) return BSPMM_EINVAL;
    *plan = nullptr;
    if (options && (options->flags & BSPMM_DRY_RUN)) return BSPMM_EINVAL;
    int rc = check_batch(b, F, true);
    if (rc != BSPMM_OK) return rc;
    int dev = -1;
    void* ws = nullptr;
    rc = static_workspace(&dev, &ws);
    if (rc != BSPMM_OK) return rc;
    bspmm_plan* p = new (std::nothrow) bspmm_plan;
    if (!p) return BSPMM_EINVAL;
    rc = plan_with_budget(*p, b, F, options, false, plan_host);
    if (rc == BSPMM_OK && p->lay.total > (size_t)BSPMM_STATIC_WORKSPACE_BYTES) rc = BSPMM_ENOSPACE;
    if (rc == BSPMM_OK) {
        p->rpt = b->rpt;
        p->colids = b->colids;
        p->values = b->values;
        // from here on the array belongs to this plan: earlier static plans of the device are
        // displaced before anything is written over their tables
        p->static_device = dev;
        p->static_generation =
            g_static_generation[dev].fetch_add(1, std::memory_order_acq_rel) + 1;
        rc = upload_plan(p, options, ws, (size_t)BSPMM_STATIC_WORKSPACE_BYTES,
                         static_cast<hipStream_t>(stream));
    }
    if (rc != BSPMM_OK) {
        delete p;
        return rc;
    }
    *plan = p;
    return BSPMM_OK;
}

int bspmm_workspace_bytes_coo(const bspmm_coo_batch* b, int32_t F, const bspmm_options* options,
                              size_t* bytes)
{
    if (!bytes) return BSPMM_EINVAL;
    *bytes = 0;
    int rc = check_coo_batch(b, F, false);
    if (rc != BSPMM_OK) return rc;
    bspmm_plan* p = new (std::nothrow) bspmm_plan;
    if (!p) return BSPMM_EINVAL;
    const bool dry = options && (options->flags & BSPMM_DRY_RUN);
    rc = plan_with_budget(*p, b, F, options, dry, plan_host_coo);
    if (rc != BSPMM_OK) {
        delete p;
        return rc;
    }
    *bytes = p->lay.total;
    remember(p, make_key(b->batch, F, options, true));
    return BSPMM_OK;
}

int bspmm_create_coo(bspmm_plan** plan, const bspmm_coo_batch* b, int32_t F,
                     const bspmm_options* options, void* workspace, size_t workspace_bytes,
                     void* stream)
{
    if (!plan) return BSPMM_EINVAL;
    *plan = nullptr;
    const bool dry = options && (options->flags & BSPMM_DRY_RUN);
    int rc = check_coo_batch(b, F, !dry);
    if (rc != BSPMM_OK) return rc;
    bspmm_plan* p = b->batch > 0 ? recall(make_key(b->batch, F, options, true), b, static_cast<const int64_t*>(nullptr)) : nullptr;
    if (!p) {
        p = new (std::nothrow) bspmm_plan;
        if (!p) return BSPMM_EINVAL;
        rc = plan_with_budget(*p, b, F, options, dry, plan_host_coo);
    }
    p->dry = dry;
    if (rc == BSPMM_OK && !dry) {
        p->ids = b->ids;
        p->coo_values = b->values;
        rc = upload_plan(p, options, workspace, workspace_bytes, static_cast<hipStream_t>(stream));
    }
    if (rc != BSPMM_OK) {
        delete p;
        return rc;
    }
    *plan = p;
    return BSPMM_OK;
}

int bspmm_export_csr(bspmm_plan* plan, int32_t* rpt, int32_t* colids, float* values, void* stream)
{
    if (!plan) return BSPMM_EINVAL;
    if (plan->dry || !plan->from_coo || plan->coo_direct) return BSPMM_ESTATE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = hipSuccess;
    if (plan->csr_rpt_words) {
        if (!rpt) return BSPMM_EINVAL;
        e = hipMemcpyAsync(rpt, plan->rpt, (size_t)plan->csr_rpt_words * 4, hipMemcpyDeviceToDevice, s);
    }
    if (e == hipSuccess && plan->csr_nz) {
        if (!colids || !values) return BSPMM_EINVAL;
        e = hipMemcpyAsync(colids, plan->colids, (size_t)plan->csr_nz * 4, hipMemcpyDeviceToDevice, s);
        if (e == hipSuccess)
            e = hipMemcpyAsync(values, plan->values, (size_t)plan->csr_nz * 4,
                               hipMemcpyDeviceToDevice, s);
    }
    return e == hipSuccess ? BSPMM_OK : hip_fail(e);
}

int bspmm_run(bspmm_plan* plan, const float* B, float* C, int64_t ldb, int64_t ldc,
              void* stream)
{
    if (!plan) return BSPMM_EINVAL;
    if (plan->dry || displaced(plan)) return BSPMM_ESTATE;
    return run_direction(plan, 0, B, C, ldb, ldc, static_cast<hipStream_t>(stream));
}

int bspmm_run_gcn(bspmm_plan* plan, const float* X, int64_t ldx, const float* W, int64_t ldw,
                  const float* bias, float* Y, int64_t ldy, int32_t accumulate, void* stream)
{
    if (!plan) return BSPMM_EINVAL;
    if (plan->dry || plan->knobs.front <= 0 || plan->coo_direct || displaced(plan)) return BSPMM_ESTATE;
    return run_gcn(plan, X, ldx, W, ldw, bias, Y, ldy, accumulate, static_cast<hipStream_t>(stream));
}

int bspmm_run_transposed(bspmm_plan* plan, const float* dY, float* G, int64_t ldy, int64_t ldg,
                         void* stream)
{
    if (!plan) return BSPMM_EINVAL;
    if (plan->dry || !plan->transposed_supported || displaced(plan)) return BSPMM_ESTATE;
    if (plan->coo_direct)
        return run_direction(plan, 1, dY, G, ldy, ldg, static_cast<hipStream_t>(stream));
    if (plan->sched[1].grid > 0 && ((!dY && plan->reads_dense) || !G || ldy < plan->F || ldg < plan->F))
        return BSPMM_EINVAL;
    int rc = enqueue_build(plan, static_cast<hipStream_t>(stream));
    if (rc != BSPMM_OK) return rc;
    return run_direction(plan, 1, dY, G, ldy, ldg, static_cast<hipStream_t>(stream));
}

int bspmm_export_transposed(bspmm_plan* plan, int32_t* rpt_t, int32_t* colids_t,
                            float* values_t, void* stream)
{
    if (!plan) return BSPMM_EINVAL;
    if (plan->dry || plan->coo_direct || plan->knobs.symmetric || displaced(plan)) return BSPMM_ESTATE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc = enqueue_build(plan, s);
    if (rc != BSPMM_OK) return rc;
    size_t rpt_words = 0, nz = 0;
    for (int i = 0; i < plan->batch; ++i) {
        rpt_words += (size_t)plan->dir[1].m[i] + 1;
        nz += (size_t)plan->dir[1].nnz[i];
    }
    hipError_t e = hipSuccess;
    if (rpt_words) {
        if (!rpt_t) return BSPMM_EINVAL;
        e = hipMemcpyAsync(rpt_t, plan->ws + plan->lay.rpt_t, rpt_words * 4,
                           hipMemcpyDeviceToDevice, s);
    }
    if (e == hipSuccess && nz) {
        if (!colids_t || !values_t) return BSPMM_EINVAL;
        e = hipMemcpyAsync(colids_t, plan->ws + plan->lay.colids_t, nz * 4,
                           hipMemcpyDeviceToDevice, s);
        if (e == hipSuccess)
            e = hipMemcpyAsync(values_t, plan->ws + plan->lay.values_t, nz * 4,
                               hipMemcpyDeviceToDevice, s);
    }
    return e == hipSuccess ? BSPMM_OK : hip_fail(e);
}

int bspmm_validate(bspmm_plan* plan, int32_t* bad_op, void* stream)
{
    if (!plan) return BSPMM_EINVAL;
    if (plan->dry || displaced(plan)) return BSPMM_ESTATE;
    if (bad_op) *bad_op = -1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t* flag = reinterpret_cast<int32_t*>(plan->ws + plan->lay.flag);
    hipError_t e = plan->from_coo
        ? launch_validate_coo(reinterpret_cast<const OpRecord*>(plan->ws + plan->lay.coo_records),
                              plan->batch, plan->ids, flag, s)
        : launch_validate(reinterpret_cast<const OpRecord*>(plan->ws + plan->lay.op_records),
                          plan->batch, plan->rpt, plan->colids, flag, s);
    if (e != hipSuccess) return hip_fail(e);
    int32_t host_flag = 0;
    e = hipMemcpyAsync(&host_flag, flag, 4, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(e);
    if (host_flag != 0x7fffffff) {
        if (bad_op) *bad_op = host_flag;
        return BSPMM_EBADCSR;
    }
    return BSPMM_OK;
}

int bspmm_kernel_info(int32_t kernel, int32_t dynamic_lds_bytes, bspmm_kernel_resources* out)
{
    if (!out || kernel < 0 || kernel > BSPMM_KERNEL_LAYER_STREAM || dynamic_lds_bytes < 0) return BSPMM_EINVAL;
    int v[7] = {0, 0, 0, 0, 0, 0, 0};
    const hipError_t e = kernel_resources(kernel, dynamic_lds_bytes, v);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return hip_fail(e);
    }
    out->vgprs = v[0];
    out->sgprs = v[1];
    out->static_lds_bytes = v[2];
    out->scratch_bytes = v[3];
    out->threads = v[4];
    out->workgroups_per_cu = v[5];
    out->compute_units = v[6];
    out->reserved_ = 0;
    return BSPMM_OK;
}

int bspmm_plan_info(const bspmm_plan* plan, bspmm_info* info)
{
    if (!plan || !info) return BSPMM_EINVAL;
    std::memset(info, 0, sizeof(*info));
    info->batch = plan->batch;
    info->F = plan->F;
    info->lds_bytes = plan->knobs.lds_words * 4;
    if (plan->coo_direct)      // the direct COO launches ask for their largest item's LDS
        info->lds_bytes = 4 * std::max(plan->coo_sched[0].lds_words, plan->coo_sched[1].lds_words);
    info->compute_units = plan->knobs.compute_units;
    for (int d = 0; d < 2; ++d) {
        info->tile[d] = plan->sched[d].tile;
        info->workgroups[d] = plan->sched[d].launch_grid;
        info->tasks[d] = plan->sched[d].grid;
        info->items[d] = (int32_t)plan->sched[d].view.size();
        for (int b = 0; b < BSPMM_NUM_BINS; ++b)
            info->items_in_bin[d][b] = plan->sched[d].items_in_bin[b];
        info->effective_bytes[d] = plan->effective_bytes[d];
        info->fused_tasks[d] = plan->sched[d].fused_tasks;
        if (plan->coo_direct) {
            info->tile[d] = plan->coo_sched[d].tile;
            info->workgroups[d] = info->tasks[d] = info->items[d] =
                (int32_t)plan->coo_sched[d].items.size();
        }
    }
    info->transposed_supported = plan->transposed_supported ? 1 : 0;
    info->transposed_built = plan->transposed_built ? 1 : 0;
    for (int d = 0; d < 2; ++d) info->lean[d] = plan->lean_items[d].empty() ? 0 : 1;
    if (plan->stream.on()) {
        info->front_stream[0] = plan->stream.graphs;
        info->front_stream[1] = plan->stream.lists * plan->stream.tiles;
        info->front_stream[2] = plan->stream.lds_bytes();
        int32_t left = 0;
        for (const WorkItem& w : plan->stream.rest) left += w.f0 == 0 ? 1 : 0;
        info->front_stream[3] = left;
    }
    info->flops = plan->flops;
    info->workspace_bytes = plan->lay.total;
    return BSPMM_OK;
}

int bspmm_plan_items(const bspmm_plan* plan, int32_t transposed, bspmm_item* items,
                     int32_t capacity, int32_t* count)
{
    if (!plan || !count || capacity < 0 || (capacity > 0 && !items)) return BSPMM_EINVAL;
    const std::vector<bspmm_item>& v = plan->coo_direct ? plan->coo_sched[transposed ? 1 : 0].view
                                                        : plan->sched[transposed ? 1 : 0].view;
    *count = (int32_t)v.size();
    const size_t n = std::min<size_t>(v.size(), (size_t)capacity);
    if (n) std::memcpy(items, v.data(), n * sizeof(bspmm_item));
    return BSPMM_OK;
}

void bspmm_destroy(bspmm_plan* plan) { delete plan; }

const char* bspmm_strerror(int code)
{
    switch (code) {
        case BSPMM_OK: return "ok";
        case BSPMM_EINVAL: return "invalid argument";
        case BSPMM_ENOSPACE: return "workspace too small";
        case BSPMM_EHIP: return "HIP runtime error";
        case BSPMM_EOVERLAP: return "output blocks overlap";
        case BSPMM_ESTATE: return "operation not available on this plan";
        case BSPMM_EBADCSR: return "malformed CSR arrays on the device";
        case BSPMM_ETOOBIG: return "operations do not fit on chip (those summed into one block together, or one with the fused front)";
        default: return "unknown error";
    }
}

int bspmm_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"

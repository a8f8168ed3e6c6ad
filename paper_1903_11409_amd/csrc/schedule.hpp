// Host-side batch scheduler of libbspmm: bins operations by size, tiles the feature
// dimension, orders the work largest-first and maps it onto workgroups XCD-aware.
#pragma once

#include <cstdint>
#include <vector>

#include "../../include/bspmm.h"
#include "plan.hpp"

namespace bspmm {

// The operations of one direction (forward, or transposed with the roles swapped).
struct DirOps {
    std::vector<int32_t> m, k, nnz;
    std::vector<int64_t> rpt_off, nz_off, in_off, out_off;
    std::vector<int32_t> chan;   // empty, or per operation: channels of the fused front it carries
                                 // (an operation standing in for a set of summed channels)
    int channels(int i) const { return chan.empty() ? 1 : chan[i]; }
    int size() const { return (int)m.size(); }
};

// Scheduler knobs with defaults filled in.
struct Knobs {
    int force_bin = -1;       // -1 automatic, else BSPMM_BIN_*
    int lds_words = 6144;     // 24 KiB: six workgroups per CU
    int min_tile = 32;
    int max_tile = 256;
    int target_wgs = 1024;
    bool target_given = false;   // the caller fixed target_wgs
    int compute_units = 256;
    int pad = 0;
    int max_passes = 1;
    int generic_rows = 8;
    int wg_passes = 0;        // 0 automatic, >0 cap on passes of a workgroup item, <0 never cut
    int capacity_wgs = 1536;  // workgroups the chip holds at once (lean kernel variant)
    int capacity_wgs_slices = 1024;   // same for the kernel variant with 32/16-lane slots
    bool accumulate = false;  // operations naming one output block are summed (else an error)
    bool hubs = false;        // split hub rows across the workgroup (reserves LDS for it)
    int front = 0;            // > 0: columns of the layer input of bspmm_run_gcn (whole workgroups,
                              // tiles in multiples of 16 columns)
    bool symmetric = false;   // A_i == A_i^T promised: the transposed product reads the same CSR
    bool coo_direct = false;  // COO plans: run the direct kernel instead of converting to CSR
    int persistent_wgs = 0;   // > 0: launch only this many workgroups and let them stride
    bool one_front_launch = false;   // whole layers: never the streaming launch
    bool lds_given = false;   // the caller fixed lds_words
    bool device_ok = false;   // planning may ask the current device (occupancy); false: dry runs
    bool need_both = false;   // planning: a transposed product that does not fit is an error too
};

struct Schedule {
    std::vector<WorkItem> items;     // device table, launch order, padded with empty items
    std::vector<int32_t> item_op;    // operation of every entry of `items` (-1: empty item)
    std::vector<bspmm_item> view;    // the non-empty items, for inspection
    int32_t wg_end[kRanges] = {0, 0, 0, 0, 0};
    int32_t item_base[kRanges] = {0, 0, 0, 0, 0};
    int fused_stride = 1;            // item slots per fused task
    int fused_tasks = 0;
    std::vector<std::vector<int>> fused_sets;   // the sets of summed operations (members in order)
    std::vector<int> task_set;       // set of every fused task, in task order
    std::vector<std::vector<int>> merged_sets;  // sets that one operation with the summed matrix
                                     // stands in for; its index is first_stand_in + position
    int first_stand_in = 0;          // == number of operations of the batch
    int error = 0;                   // BSPMM_E* when the batch cannot be scheduled
    int grid = 0;                    // number of tasks
    int launch_grid = 0;             // workgroups of the persistent launch
    bool lean = false;               // every task is one staged workgroup item with a direct
                                     // tile: the launch may take the lean kernel
    bool has_slices = false;         // any 32- or 16-lane item: needs the larger kernel variant
    int tile = 0;
    int front_lds_words = 0;         // LDS the fused-front launch asks for (its largest item)
    int items_in_bin[BSPMM_NUM_BINS] = {0, 0, 0, 0, 0};
};

// Schedule of the direct COO kernel: one workgroup per item, largest first.
struct CooSchedule {
    std::vector<CooItem> items;
    std::vector<bspmm_item> view;
    int tile = 0;
    int error = 0;
    int lds_words = 0;     // what the launch asks for: the largest item's
};

int workgroups_per_cu(int front_features);
Knobs resolve_knobs(const bspmm_options* o);

// Items of the direct COO kernel for `ops` (rpt_off unused, nz_off = the caller's entry offsets).
CooSchedule make_coo_schedule(const DirOps& ops, int F, const Knobs& kn);

// Build the single-launch schedule for `ops` at feature width F.
Schedule make_schedule(const DirOps& ops, int F, const Knobs& kn);

}  // namespace bspmm

"""Seeded random batches and scheduler options for the property tests.

One seed gives one case: a mix of operation shapes (empty, tiny, molecule-sized, a few hundred
rows, strongly rectangular), a feature width and a handful of scheduler knobs.  The CPU tests
check the schedule of every case against the coverage and capacity invariants; the GPU tests
run the same cases and compare with the oracle, so a corner of the scheduler that the
workload configurations never reach is still exercised on both sides.
"""
import numpy as np

from paper_1903_11409_amd import bspmm as K
from paper_1903_11409_amd import workloads as W

FEATURES = [1, 2, 4, 7, 8, 12, 16, 20, 32, 48, 64, 100, 128, 200, 256, 384]


def _shape(rng, kind):
    if kind == 0:   # nothing to do
        return [(0, 0, 0), (0, 5, 0), (5, 0, 0), (4, 4, 0)][int(rng.integers(4))]
    if kind == 1:   # a few rows
        m, n = int(rng.integers(1, 9)), int(rng.integers(1, 9))
    elif kind == 2:   # molecule-sized, square
        m = n = int(rng.integers(10, 61))
    elif kind == 3:   # a few hundred rows, square
        m = n = int(rng.integers(61, 400))
    elif kind == 4:   # short and wide / tall and narrow
        m, n = int(rng.integers(1, 6)), int(rng.integers(200, 1500))
        if rng.integers(2):
            m, n = n, m
    else:   # larger than any LDS budget at full width
        m = n = int(rng.integers(400, 2500))
    per_row = [0.3, 1.0, 2.5, 5.0, 20.0][int(rng.integers(5))]
    return (m, n, int(min(per_row * m, 40000)))


def random_case(seed, max_ops=200, max_nnz=250_000, with_dY=True):
    """(batch, options as keyword dict) of one seed."""
    rng = np.random.default_rng(0xB5B0 + seed)
    batch = [1, 2, 5, 17, 60, max_ops][int(rng.integers(6))]
    kinds_p = np.array([1, 3, 6, 2, 1, 0.5])
    if batch > 60:
        kinds_p[5] = 0.05
    kinds = rng.choice(6, size=batch, p=kinds_p / kinds_p.sum())
    shapes, total = [], 0
    for kd in kinds:
        s = _shape(rng, int(kd))
        if total + s[2] > max_nnz:
            s = (s[0], s[1], min(s[2], s[0]))
        total += s[2]
        shapes.append(s)
    F = FEATURES[int(rng.integers(len(FEATURES)))]
    b = W.random_general(1000 + seed, F=F, shapes=shapes, sort_columns=bool(rng.integers(2)),
                         with_dY=with_dY, shuffle_blocks=bool(rng.integers(2)))
    opts = {}
    pick = lambda values: values[int(rng.integers(len(values)))]
    if rng.random() < 0.4:
        opts["lds_bytes"] = pick([4096, 8192, 16384, 32768, 65536])
    if rng.random() < 0.3:
        opts["min_tile"] = pick([4, 8, 16, 32])
    if rng.random() < 0.3:
        opts["max_tile"] = pick([32, 64, 128, 256])
    if rng.random() < 0.4:
        opts["target_workgroups"] = pick([1, 64, 512, 4096])
    if rng.random() < 0.35:
        opts["force_bin"] = pick([K.BIN_WORKGROUP, K.BIN_WAVE, K.BIN_SLICE32, K.BIN_SLICE16,
                                  K.BIN_GENERIC])
    if rng.random() < 0.3:
        opts["wg_passes"] = pick([1, 2, -1])
    if rng.random() < 0.25:
        opts["max_passes"] = pick([1, 2, 4])
    if rng.random() < 0.2:
        opts["lds_pad"] = pick([4, 8])
    if rng.random() < 0.2:
        opts["flags"] = K.SPLIT_HUB_ROWS
    if rng.random() < 0.2:
        opts["resident_workgroups"] = pick([8, 64, 300])
    if rng.random() < 0.2:
        opts["generic_rows"] = pick([4, 8, 64])
    return b, opts


def _random_csr(rng, m, n, z, sort_columns):
    r = rng.integers(0, max(m, 1), size=z)
    c = rng.integers(0, max(n, 1), size=z)
    v = rng.uniform(-1.0, 1.0, size=z)
    order = np.lexsort((c, r)) if sort_columns else np.argsort(r, kind="stable")
    r, c, v = r[order], c[order], v[order]
    rpt = np.zeros(m + 1, dtype=np.int32)
    rpt[1:] = np.cumsum(np.bincount(r, minlength=m) if z else np.zeros(m, dtype=np.int64))
    return rpt, c.astype(np.int32), v.astype(np.float32)


def random_summed_case(seed, with_dY=True):
    """Groups of one to eight operations that are added into one output block (the layer's
    channel sum with BSPMM_ACCUMULATE): the members of a group share the row count; they read
    one shared dense block (same column count) or a block each (any column counts; back to back
    in the packed input, or with unused rows in between)."""
    rng = np.random.default_rng(0x5B77 + seed)
    groups = [1, 3, 12, 50][int(rng.integers(4))]
    ops, b_block_of_op, b_block_rows, c_block_of_op = [], [], [], []
    for g in range(groups):
        m = int(rng.integers(1, 140)) if rng.random() < 0.9 else int(rng.integers(140, 600))
        members = int(rng.integers(1, 9))
        shared = bool(rng.integers(2))
        spaced = bool(rng.integers(2))
        n_shared = m if rng.integers(2) else int(rng.integers(1, 140))
        if shared:
            b_block_rows.append(n_shared)
        for _ in range(members):
            n = n_shared if shared else int(rng.integers(1, 140))
            per_row = [0.0, 0.3, 1.0, 3.0, 8.0][int(rng.integers(5))]
            rpt, ci, va = _random_csr(rng, m, n, int(per_row * m), bool(rng.integers(2)))
            ops.append((m, n, rpt, ci, va))
            if not shared:
                if spaced:      # a block nobody reads in between: the members' blocks are apart
                    b_block_rows.append(int(rng.integers(1, 4)))
                b_block_rows.append(n)
            b_block_of_op.append(len(b_block_rows) - 1)
            c_block_of_op.append(g)
    F = [1, 4, 8, 20, 32, 63, 64, 100, 128, 256][int(rng.integers(10))]
    b = W.assemble("summed", F, ops, b_block_of_op, b_block_rows, rng, with_dY=with_dY,
                   n_graphs=groups, c_block_of_op=c_block_of_op)
    opts = {"flags": K.ACCUMULATE}
    pick = lambda values: values[int(rng.integers(len(values)))]
    if rng.random() < 0.3:
        opts["lds_bytes"] = pick([16384, 32768, 65536])
    if rng.random() < 0.3:
        opts["min_tile"] = pick([4, 8, 16])
    if rng.random() < 0.3:
        opts["max_tile"] = pick([32, 64, 128])
    if rng.random() < 0.3:
        opts["target_workgroups"] = pick([1, 64, 4096])
    if rng.random() < 0.2:
        opts["resident_workgroups"] = pick([8, 64])
    if rng.random() < 0.2:
        opts["lds_pad"] = 4
    return b, opts

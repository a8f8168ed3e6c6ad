"""Host logic of libbspmm without a GPU: exported symbols, argument checking, and the
scheduler's invariants (every output element of every operation is computed exactly once,
staged items fit their LDS share, workgroups are well formed)."""
import ctypes
import os
import re

import dataclasses

import numpy as np
import pytest

from paper_1903_11409_amd import bspmm as K
from paper_1903_11409_amd import build as B
from paper_1903_11409_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(K.LIB_PATH):
        B.build()


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "bspmm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(bspmm_[a-z_]+)\s*\(", text))
    assert declared == set(K.EXPORTS)
    raw = ctypes.CDLL(K.LIB_PATH)
    for name in declared:
        assert hasattr(raw, name), name


def test_struct_sizes_match_header():
    assert ctypes.sizeof(K.bspmm_item) == 32
    assert ctypes.sizeof(K.bspmm_options) == 56
    assert ctypes.sizeof(K.bspmm_batch) == 8 + 10 * 8
    assert ctypes.sizeof(K.bspmm_info) == 16 + 8 + 8 + 8 + 8 + 40 + 8 + 8 + 8 + 16 + 16 + 8 + 8


def _slot_lanes(bin_):
    return {K.BIN_WORKGROUP: 256, K.BIN_WAVE: 64, K.BIN_SLICE32: 32, K.BIN_SLICE16: 16,
            K.BIN_GENERIC: 256}[bin_]


def _lds_words(m, k, nnz, fw, pad, lanes, hubs):
    cv = (m + 1 + 1) // 2 * 2
    b_off = (cv + 2 * nnz + 3) // 4 * 4
    words = b_off + k * ((fw + 3) // 4 * 4 + pad)
    if lanes == 256 and hubs:   # hub-row list and reduction scratch of workgroup items
        words += (1 + nnz // 64 + 3) // 4 * 4 + 4 * ((fw + 3) // 4 * 4)
    return words


def _check_schedule(b, F, transposed=False, **opts):
    h = K.dry_plan(b, F, **opts)
    try:
        info = K.bspmm_plan_info(h)
        items = K.bspmm_plan_items(h, transposed)
        d = 1 if transposed else 0
        assert info.items[d] == len(items)
        m_of = b.cols if transposed else b.rows
        k_of = b.rows if transposed else b.cols
        cover = [np.zeros((int(m), F), dtype=np.int32) for m in m_of]
        seen = set()
        out_of = b.b_row_off if transposed else b.c_row_off
        blocks = {}
        for i in range(b.batch):
            if int(m_of[i]) > 0:
                blocks.setdefault((int(out_of[i]), int(m_of[i])), []).append(i)
        summed = {i for ops in blocks.values() if len(ops) > 1 for i in ops}
        pad = max(opts.get("lds_pad", 0), 0)
        for it in items:
            assert 0 <= it.op < b.batch
            assert it.nrows > 0 and it.fw > 0
            cover[it.op][it.row0:it.row0 + it.nrows, it.f0:it.f0 + it.fw] += 1
            lanes = _slot_lanes(it.bin)
            if it.op in summed:
                assert 0 <= it.slot < 8          # member index inside the fused task
            else:
                assert 0 <= it.slot < 256 // lanes
            assert 0 <= it.workgroup < info.tasks[d]
            assert (it.workgroup, it.slot) not in seen
            seen.add((it.workgroup, it.slot))
            fused_member = it.op in summed
            if it.bin != K.BIN_GENERIC and not fused_member:
                if it.bin != K.BIN_WORKGROUP:   # only workgroup items may be cut into row ranges
                    assert it.row0 == 0 and it.nrows == int(m_of[it.op])
                need = _lds_words(int(m_of[it.op]), int(k_of[it.op]), int(b.nnz[it.op]), it.fw, pad, lanes, bool(opts.get('flags', 0) & K.SPLIT_HUB_ROWS))
                front = opts.get("front_features", 0) if not transposed else 0
                if front:   # 16 rows of X_i at least, the weight tile and the bias tile ride
                    #          along; whole workgroups, 16-column blocks for the matrix cores
                    need += 16 * front + front * it.fw + it.fw
                    assert it.bin == K.BIN_WORKGROUP and it.fw % 16 == 0 and it.f0 % 16 == 0
                assert need * 4 <= info.lds_bytes * lanes // 256
                if F % 4 == 0:
                    assert it.f0 % 4 == 0 and it.fw % 4 == 0
        for c in cover:
            assert np.all(c == 1)
        # sub-workgroup ranges come after the one-item-per-workgroup range, smaller slots last
        order = {K.BIN_WORKGROUP: 0, K.BIN_GENERIC: 0, K.BIN_WAVE: 1, K.BIN_SLICE32: 2,
                 K.BIN_SLICE16: 3}
        hi = [-1, -1, -1, -1]
        lo = [10 ** 9] * 4
        for it in items:
            r = order[it.bin]
            hi[r] = max(hi[r], it.workgroup)
            lo[r] = min(lo[r], it.workgroup)
        prev = -1
        for r in range(4):
            if hi[r] >= 0:
                assert lo[r] > prev
                prev = hi[r]
        return info, items
    finally:
        K.bspmm_destroy(h)


@pytest.mark.parametrize("cfg,kw", [(1, {}), (2, {"F": 64}), (2, {"F": 128}),
                                    (3, {"graphs": 96}), (4, {"F": 256, "graphs": 32}),
                                    (4, {"F": 1024, "graphs": 32}), (5, {"graphs": 128})])
def test_every_output_element_scheduled_once(cfg, kw):
    b = W.CONFIGS[cfg](**kw)
    info, _ = _check_schedule(b, b.F)
    assert info.flops == W.flops(b)
    assert info.effective_bytes[0] == W.effective_bytes(b)
    if info.transposed_supported:
        _check_schedule(b, b.F, transposed=True)
        assert info.effective_bytes[1] == W.effective_bytes(b, transposed=True)


@pytest.mark.parametrize("F", [1, 3, 4, 5, 63, 64, 65, 100, 260, 1000])
def test_odd_feature_widths_and_shapes(F):
    shapes = [(1, 1, 1), (0, 0, 0), (7, 13, 25), (13, 7, 25), (40, 40, 0), (300, 300, 2000),
              (2, 900, 50), (900, 2, 50)]
    b = W.random_general(F, F=F, shapes=shapes, with_dY=False)
    _check_schedule(b, F)
    _check_schedule(b, F, transposed=True)


@pytest.mark.parametrize("bin_", [K.BIN_WORKGROUP, K.BIN_WAVE, K.BIN_SLICE32, K.BIN_SLICE16,
                                  K.BIN_GENERIC])
def test_forced_bins_still_cover(bin_):
    b = W.config2_molecule(graphs=48, F=64)
    info, items = _check_schedule(b, 64, force_bin=bin_)
    if bin_ in (K.BIN_WORKGROUP, K.BIN_GENERIC):
        assert all(it.bin == bin_ for it in items)
    else:
        assert any(it.bin == bin_ for it in items)


@pytest.mark.parametrize("opts", [{"lds_pad": 4}, {"min_tile": 16}, {"max_tile": 64},
                                  {"lds_bytes": 65536}, {"lds_bytes": 8192}, {"lds_bytes": 163840},
                                  {"target_workgroups": 64}, {"max_passes": 4},
                                  {"wg_passes": 1}, {"wg_passes": -1, "target_workgroups": 4096},
                                  {"resident_workgroups": 64}, {"resident_workgroups": 24},
                                  {"flags": K.SPLIT_HUB_ROWS},
                                  {"generic_rows": 8, "lds_bytes": 4096}])
def test_knobs_keep_the_invariants(opts):
    b = W.config5_skewed(graphs=64, F=128)
    _check_schedule(b, 128, **opts)


def test_generic_row_blocks_share_an_xcd():
    """Row blocks of a large operation read one dense tile: their workgroup indices agree
    modulo 8 (workgroups are dealt round-robin to the 8 XCDs)."""
    b = W.random_general(3, F=256, shapes=[(700, 700, 5000), (30, 30, 90), (650, 650, 3000)],
                         with_dY=False)
    info, items = _check_schedule(b, 256)
    for op in (0, 2):
        for f0 in {it.f0 for it in items if it.op == op}:
            mods = {it.workgroup % 8 for it in items if it.op == op and it.f0 == f0}
            assert len(mods) == 1
            assert all(it.bin == K.BIN_GENERIC for it in items if it.op == op)


def test_channels_of_one_graph_share_an_xcd_or_workgroup():
    b = W.config3_multichannel(graphs=40)
    info, items = _check_schedule(b, b.F)
    by_block = {}
    for it in items:
        by_block.setdefault((int(b.b_row_off[it.op]), it.f0), []).append(it)
    for group in by_block.values():
        wgs = {it.workgroup for it in group}
        if all(it.bin == K.BIN_WORKGROUP for it in group):
            assert len({w % 8 for w in wgs}) == 1


def test_argument_errors():
    b = W.config1_tiny()

    def create(**over):
        f = dict(rows=b.rows, cols=b.cols, nnz=b.nnz, rpt_off=b.rpt_off, nz_off=b.nz_off,
                 b_row_off=b.b_row_off, c_row_off=b.c_row_off)
        f.update(over)
        hb = K.HostBatch(**f)
        return K.bspmm_create(hb, over.get("F", 64), K.make_options(flags=K.DRY_RUN))

    bad_rows = b.rows.copy()
    bad_rows[2] = -1
    with pytest.raises(K.BspmmError) as e:
        create(rows=bad_rows)
    assert e.value.code == K.EINVAL
    overlap = b.c_row_off.copy()
    overlap[1] = overlap[0] + 1
    with pytest.raises(K.BspmmError) as e:
        create(c_row_off=overlap)
    assert e.value.code == K.EOVERLAP
    neg = b.nz_off.copy()
    neg[0] = -5
    with pytest.raises(K.BspmmError) as e:
        create(nz_off=neg)
    assert e.value.code == K.EINVAL
    hb = K.HostBatch(b.rows, b.cols, b.nnz, b.rpt_off, b.nz_off, b.b_row_off, b.c_row_off)
    with pytest.raises(K.BspmmError) as e:
        K.bspmm_create(hb, 0, K.make_options(flags=K.DRY_RUN))
    assert e.value.code == K.EINVAL
    # without DRY_RUN the device pointers and a workspace are required
    with pytest.raises(K.BspmmError) as e:
        K.bspmm_create(hb, 64, K.make_options(), None, 0, stream=0)
    assert e.value.code == K.EINVAL
    assert K.lib().bspmm_strerror(K.EOVERLAP) == b"output blocks overlap"
    assert K.lib().bspmm_run(None, None, None, 1, 1, None) == K.EINVAL


def test_dry_plan_refuses_to_run_and_shared_inputs_disable_transposed():
    b = W.config3_multichannel(graphs=8)
    h = K.dry_plan(b)
    try:
        info = K.bspmm_plan_info(h)
        assert info.transposed_supported == 0
        assert info.workgroups[1] == 0
        assert K.lib().bspmm_run(h, 1, 1, 128, 128, None) == K.ESTATE
        assert K.lib().bspmm_run_transposed(h, 1, 1, 128, 128, None) == K.ESTATE
    finally:
        K.bspmm_destroy(h)


def test_empty_batch_and_workspace_size():
    e = W.random_general(1, F=8, shapes=[], with_dY=False)
    h = K.dry_plan(e)
    info = K.bspmm_plan_info(h)
    assert info.workgroups[0] == 0 and info.tasks[0] == 0 and info.items[0] == 0
    K.bspmm_destroy(h)
    b = W.config2_molecule(graphs=16)
    hb = K.HostBatch(b.rows, b.cols, b.nnz, b.rpt_off, b.nz_off, b.b_row_off, b.c_row_off)
    o = K.make_options(flags=K.DRY_RUN)
    n = K.bspmm_workspace_bytes(hb, b.F, o)
    h = K.bspmm_create(hb, b.F, o)
    assert K.bspmm_plan_info(h).workspace_bytes == n and n % 256 == 0
    # the transposed CSR (row pointers, columns, values) lives in the workspace
    assert n >= 4 * (int((b.cols.astype(np.int64) + 1).sum()) + 2 * int(b.nnz.sum()))
    K.bspmm_destroy(h)


def test_summed_operations_share_one_task():
    """With BSPMM_ACCUMULATE the channels of a graph (same output block) become members of
    one task per (tile, row range); every member still covers its rows exactly once.  Channels
    whose dense inputs are one block of the packed input (the same block, or blocks lying back
    to back in channel order) are the product with their matrices side by side, an ordinary
    workgroup item; otherwise (here: the blocks of channels 0 and 1 swapped) a fused task."""
    fused = {}
    for own, swapped in ((False, False), (True, False), (True, True)):
        b = W.config3_multichannel(graphs=48, accumulate=True, own_inputs=own)
        if swapped:
            off = b.b_row_off.copy()
            off[0::4], off[1::4] = b.b_row_off[1::4], b.b_row_off[0::4]
            b = dataclasses.replace(b, b_row_off=off)
        info, items = _check_schedule(b, b.F, flags=K.ACCUMULATE)
        fused[(own, swapped)] = info.fused_tasks[0]
        assert info.transposed_supported == 1
        ch = b.meta["channels"]
        by_task = {}
        for it in items:
            by_task.setdefault(it.workgroup, []).append(it)
        for members in by_task.values():
            assert len(members) == ch
            assert len({m.op // ch for m in members}) == 1           # one graph
            assert sorted(m.slot for m in members) == list(range(ch))
            assert len({(m.row0, m.nrows, m.f0, m.fw) for m in members}) == 1
        _check_schedule(b, b.F, transposed=True, flags=K.ACCUMULATE)
        assert info.effective_bytes[0] == W.effective_bytes(b)
    # (with a block per channel the largest graphs do not fit a plain item and stay fused tasks)
    assert fused[(False, False)] == 0 and fused[(True, True)] > 4 * fused[(True, False)]
    # shared inputs, separate outputs: the transposed product sums into the shared input block
    # (the channels' output blocks lie back to back: no fused task in that direction either)
    b = W.config3_multichannel(graphs=16)
    info, _ = _check_schedule(b, b.F, flags=K.ACCUMULATE)
    assert info.fused_tasks[0] == 0 and info.transposed_supported == 1
    info_t, items_t = _check_schedule(b, b.F, transposed=True, flags=K.ACCUMULATE)
    assert info_t.fused_tasks[1] == 0 and len({(it.workgroup, it.slot) for it in items_t}) == len(items_t)


def test_summed_operations_need_the_flag_and_must_fit():
    b = W.config3_multichannel(graphs=4, accumulate=True)
    hb = K.HostBatch(b.rows, b.cols, b.nnz, b.rpt_off, b.nz_off, b.b_row_off, b.c_row_off)
    with pytest.raises(K.BspmmError) as e:
        K.bspmm_create(hb, b.F, K.make_options(flags=K.DRY_RUN))
    assert e.value.code == K.EOVERLAP
    # nine operations into one block: more members than a fused task holds
    many = W.config3_multichannel(graphs=2, channels=9, accumulate=True)
    hb = K.HostBatch(many.rows, many.cols, many.nnz, many.rpt_off, many.nz_off, many.b_row_off,
                     many.c_row_off)
    with pytest.raises(K.BspmmError) as e:
        K.bspmm_create(hb, many.F, K.make_options(flags=K.DRY_RUN | K.ACCUMULATE))
    assert e.value.code == K.ETOOBIG
    # two large operations into one block: their arrays do not fit LDS together
    big = W.random_general(5, F=64, shapes=[(3000, 3000, 9000), (3000, 3000, 9000)], with_dY=False)
    big.c_row_off[1] = big.c_row_off[0]
    hb = K.HostBatch(big.rows, big.cols, big.nnz, big.rpt_off, big.nz_off, big.b_row_off,
                     big.c_row_off)
    with pytest.raises(K.BspmmError) as e:
        K.bspmm_create(hb, 64, K.make_options(flags=K.DRY_RUN | K.ACCUMULATE))
    assert e.value.code == K.ETOOBIG
    # partial overlap is an error with or without the flag
    b2 = W.config1_tiny()
    off = b2.c_row_off.copy()
    off[1] = off[0] + 1
    hb = K.HostBatch(b2.rows, b2.cols, b2.nnz, b2.rpt_off, b2.nz_off, b2.b_row_off, off)
    with pytest.raises(K.BspmmError) as e:
        K.bspmm_create(hb, 64, K.make_options(flags=K.DRY_RUN | K.ACCUMULATE))
    assert e.value.code == K.EOVERLAP


# ---------------------------------------------------------------------------------------------
# COO / SparseTensor plans: the schedule is the CSR plan's; the workspace also holds the CSR
# ---------------------------------------------------------------------------------------------
def test_coo_struct_size():
    assert ctypes.sizeof(K.bspmm_coo_batch) == 8 + 8 * 8


@pytest.mark.parametrize("maker", [lambda: W.config2_molecule(graphs=64, F=128),
                                   lambda: W.config5_skewed(graphs=32, F=64),
                                   lambda: W.random_general(5, F=20, shapes=[(7, 13, 25), (0, 0, 0),
                                                                             (40, 3, 70)])])
def test_coo_plan_schedules_like_the_csr_plan(maker):
    b = maker()
    hc = K.dry_plan(b, coo=True)
    h = K.dry_plan(b)
    try:
        for t in (False, True):
            a = [(i.op, i.bin, i.row0, i.nrows, i.f0, i.fw, i.workgroup, i.slot)
                 for i in K.bspmm_plan_items(hc, t)]
            c = [(i.op, i.bin, i.row0, i.nrows, i.f0, i.fw, i.workgroup, i.slot)
                 for i in K.bspmm_plan_items(h, t)]
            assert a == c
        ic, i0 = K.bspmm_plan_info(hc), K.bspmm_plan_info(h)
        assert ic.flops == i0.flops and list(ic.effective_bytes) == list(i0.effective_bytes)
        # room for the built CSR: row pointers, column indices and values
        extra = 4 * int((b.rows.astype(np.int64) + 1).sum()) + 8 * int(b.nnz.sum())
        assert ic.workspace_bytes >= i0.workspace_bytes + extra
        hb = K.HostCooBatch(b.rows, b.cols, b.nnz, b.nz_off, b.b_row_off, b.c_row_off)
        assert K.bspmm_workspace_bytes_coo(hb, b.F, K.make_options(flags=K.DRY_RUN)) == ic.workspace_bytes
    finally:
        K.bspmm_destroy(hc)
        K.bspmm_destroy(h)


def test_coo_argument_errors():
    b = W.config1_tiny()
    opts = K.make_options(flags=K.DRY_RUN)
    good = K.HostCooBatch(b.rows, b.cols, b.nnz, b.nz_off, b.b_row_off, b.c_row_off)
    with pytest.raises(K.BspmmError) as e:
        K.bspmm_create_coo(good, 0, opts)
    assert e.value.code == K.EINVAL
    neg = K.HostCooBatch(b.rows, b.cols, -b.nnz, b.nz_off, b.b_row_off, b.c_row_off)
    with pytest.raises(K.BspmmError) as e:
        K.bspmm_create_coo(neg, b.F, opts)
    assert e.value.code == K.EINVAL
    same_c = K.HostCooBatch(b.rows, b.cols, b.nnz, b.nz_off, b.b_row_off, np.zeros_like(b.c_row_off))
    with pytest.raises(K.BspmmError) as e:
        K.bspmm_create_coo(same_c, b.F, opts)
    assert e.value.code == K.EOVERLAP
    h = K.bspmm_create_coo(good, b.F, opts)
    try:   # a dry plan has nothing on the device to export
        rc = K.lib().bspmm_export_csr(h, None, None, None, None)
        assert rc == K.ESTATE
    finally:
        K.bspmm_destroy(h)
    raw = K.lib()
    assert raw.bspmm_workspace_bytes_coo(None, 8, None, ctypes.byref(ctypes.c_size_t())) == K.EINVAL


@pytest.mark.parametrize("maker,F,kw", [
    (lambda: W.config2_molecule(graphs=64, F=128), 128, {}),
    (lambda: W.config5_skewed(graphs=64, F=256), 256, {}),
    (lambda: W.config4_wide(graphs=16, F=1024), 1024, {}),
    (lambda: W.random_general(5, F=1, shapes=[(7, 13, 25), (0, 0, 0), (40, 3, 70), (9, 9, 0)]), 63, {}),
    # tiles that cannot hold all rows: row ranges
    (lambda: W.random_general(6, F=1, shapes=[(5000, 40, 900), (3, 3, 3)]), 64, {"lds_bytes": 8192}),
    (lambda: W.config2_molecule(graphs=8, F=1), 100, {"target_workgroups": 4000}),
])
@pytest.mark.parametrize("transposed", [False, True])
def test_direct_coo_schedule_covers_every_element_once(maker, F, kw, transposed):
    _check_direct_coo_schedule(maker(), F, kw, transposed)


def _check_direct_coo_schedule(b, F, kw, transposed):
    h = K.dry_plan(b, F, coo=True, flags=K.COO_DIRECT, **kw)
    try:
        info = K.bspmm_plan_info(h)
        items = K.bspmm_plan_items(h, transposed)
        d = 1 if transposed else 0
        assert info.items[d] == info.workgroups[d] == len(items)
        m_of = b.cols if transposed else b.rows
        cover = [np.zeros((int(m), F), dtype=np.int32) for m in m_of]
        for n, it in enumerate(items):
            assert it.bin == K.BIN_COO and it.workgroup == n
            assert it.nrows > 0 and it.fw > 0 and it.fw <= 256
            assert F % 4 != 0 or (it.f0 % 4 == 0 and it.fw % 4 == 0)
            # the output tile of the item, and whatever else it stages (slot = mode bits: 1 the
            # dense tile, 2 the entries), sit in LDS together; mode bit 4: the entries are
            # sorted by row on chip (pairs of dense row and value, row counts and row pointers)
            # and there is no output tile
            k_of = b.rows if transposed else b.cols
            stride = (it.fw + 3) // 4 * 4
            assert it.slot in (0, 2, 3, 6, 7)
            if it.slot & 4:
                words = 2 * int(b.nnz[it.op]) + 2 * it.nrows + 4
            else:
                words = it.nrows * stride
                if it.slot & 2:
                    words += 3 * int(b.nnz[it.op]) + 1
            if it.slot & 1:
                words += int(k_of[it.op]) * stride
            assert words * 4 <= info.lds_bytes
            cover[it.op][it.row0:it.row0 + it.nrows, it.f0:it.f0 + it.fw] += 1
        for c in cover:
            assert np.all(c == 1)
        assert info.flops == 2 * int(b.nnz.sum()) * F
    finally:
        K.bspmm_destroy(h)


def test_wide_traffic_bound_launches_take_a_third_of_the_lds():
    """F >= 512, more than 28 MB moved, more than one round of workgroups: the plan takes 52 KiB
    per workgroup (tiles twice as wide) when the launch then needs at most a tenth more rounds
    than with 24 KiB; a budget from the caller is kept as given."""
    def info_of(b, **kw):
        h = K.dry_plan(b, b.F, **kw)
        try:
            return K.bspmm_plan_info(h)
        finally:
            K.bspmm_destroy(h)
    wide = info_of(W.config4_wide(F=1024))
    assert wide.lds_bytes == 53248 and wide.workgroups[0] * 6 <= 2168 * 3 and list(wide.lean) == [1, 1]
    assert info_of(W.config4_wide(F=1024), lds_bytes=24576).lds_bytes == 24576
    assert info_of(W.config4_wide(F=512)).lds_bytes == 24576          # one round at 24 KiB, two at 52
    assert info_of(W.config2_molecule(F=1024, graphs=512)).lds_bytes == 24576   # small graphs: wide tiles already
    assert info_of(W.config5_skewed()).lds_bytes == 24576             # F = 256
    for seed in (7000, 7007, 7008, 7009):                             # other batches of the same kind
        assert info_of(W.config4_wide(seed=seed, F=1024)).lds_bytes == 53248
    assert info_of(W.config2_molecule(F=512, graphs=1024)).lds_bytes == 24576   # 2.2 -> 2.8 rounds


def test_direct_coo_sorts_on_chip_where_the_entries_fit():
    """Without a caller's budget the launch takes the smallest LDS size at which every operation's
    entries are sorted on chip (slot bit 4); a small budget from the caller is kept and the
    operations that do not fit fall back to the output tile with row ranges."""
    for b, lds_most in ((W.config2_molecule(), 24576), (W.config5_skewed(), 32768)):
        h = K.dry_plan(b, b.F, coo=True, flags=K.COO_DIRECT)
        try:
            info = K.bspmm_plan_info(h)
            assert all(it.slot & 4 for it in K.bspmm_plan_items(h, False))
            assert all(it.slot & 4 for it in K.bspmm_plan_items(h, True))
            assert 0 < info.lds_bytes <= lds_most
        finally:
            K.bspmm_destroy(h)
    b = W.config5_skewed()
    h = K.dry_plan(b, b.F, coo=True, flags=K.COO_DIRECT, lds_bytes=8192)
    try:
        slots = {it.slot for it in K.bspmm_plan_items(h, False)}
        assert slots & {0, 2} and K.bspmm_plan_info(h).lds_bytes <= 8192
    finally:
        K.bspmm_destroy(h)


def test_direct_coo_rejects_what_it_cannot_do():
    b = W.config3_multichannel(graphs=4, F=32, accumulate=True)
    hc = K.HostCooBatch(b.rows, b.cols, b.nnz, b.nz_off, b.b_row_off, b.c_row_off)
    for flags in (K.COO_DIRECT | K.ACCUMULATE, K.COO_DIRECT | K.SPLIT_HUB_ROWS):
        with pytest.raises(K.BspmmError) as e:
            K.bspmm_create_coo(hc, 32, K.make_options(flags=K.DRY_RUN | flags))
        assert e.value.code == K.EINVAL
    with pytest.raises(K.BspmmError) as e:       # summed output blocks need the CSR route
        K.bspmm_create_coo(hc, 32, K.make_options(flags=K.DRY_RUN | K.COO_DIRECT))
    assert e.value.code == K.EOVERLAP
    # inputs shared by several operations: forward works, the transposed product is refused
    b2 = W.config3_multichannel(graphs=4, F=32)
    h = K.dry_plan(b2, coo=True, flags=K.COO_DIRECT)
    try:
        assert K.bspmm_plan_info(h).transposed_supported == 0
    finally:
        K.bspmm_destroy(h)


# ---------------------------------------------------------------------------------------------
# fused front of the layer (bspmm_run_gcn): the forward schedule also holds X_i in LDS
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("maker,F,nx", [
    (lambda: W.config2_molecule(graphs=64, F=128), 128, 64),
    (lambda: W.config2_molecule(graphs=64, F=64), 64, 76),
    (lambda: W.config3_multichannel(graphs=32, F=128), 128, 32),
    (lambda: W.config4_wide(graphs=16, F=512), 512, 128),
])
@pytest.mark.parametrize("transposed", [False, True])
def test_front_schedule_invariants(maker, F, nx, transposed):
    if transposed and nx == 32:
        pytest.skip("channels share their input block: no transposed product without ACCUMULATE")
    _check_schedule(maker(), F, transposed=transposed, front_features=nx)
    _check_schedule(maker(), F, transposed=transposed, front_features=nx, min_tile=8, max_tile=100)


def test_front_argument_errors():
    b = W.config2_molecule(graphs=8, F=128)
    for kw, code in [(dict(front_features=64, flags=K.ACCUMULATE), K.EINVAL),
                     (dict(front_features=64, flags=K.SPLIT_HUB_ROWS), K.EINVAL),
                     (dict(front_features=63), K.EINVAL),
                     (dict(front_features=64, lds_pad=4), K.EINVAL)]:
        with pytest.raises(K.BspmmError) as e:
            K.dry_plan(b, 128, **kw)
        assert e.value.code == code, kw
    with pytest.raises(K.BspmmError) as e:      # F must be a multiple of 16
        K.dry_plan(b, 100, front_features=64)
    assert e.value.code == K.EINVAL
    big = W.config5_skewed(graphs=64, F=128)     # graphs of hundreds of nodes in 16 KiB: no room
    with pytest.raises(K.BspmmError) as e:
        K.dry_plan(big, 128, front_features=128, lds_bytes=16384)
    assert e.value.code == K.ETOOBIG
    h = K.dry_plan(b, 128)                       # a plan without the front refuses the call
    try:
        assert K.lib().bspmm_run_gcn(h, None, 0, None, 0, None, None, 0, 0, None) == K.ESTATE
    finally:
        K.bspmm_destroy(h)


def test_workspace_query_hands_its_schedule_to_create_only_for_the_same_batch():
    """bspmm_workspace_bytes keeps its plan for the next bspmm_create on the thread; a batch
    whose arrays changed in place (same addresses) must be scheduled afresh."""
    b = W.config2_molecule(graphs=16, F=64)
    hb = K.HostBatch(b.rows, b.cols, b.nnz, b.rpt_off, b.nz_off, b.b_row_off, b.c_row_off)
    opts = K.make_options(flags=K.DRY_RUN)
    n0 = K.bspmm_workspace_bytes(hb, 64, opts)
    h = K.bspmm_create(hb, 64, opts)
    flops0 = K.bspmm_plan_info(h).flops
    assert K.bspmm_plan_info(h).workspace_bytes == n0
    K.bspmm_destroy(h)
    K.bspmm_workspace_bytes(hb, 64, opts)
    hb.arrays[2][3] += 5                      # nnz of operation 3, edited in place
    h = K.bspmm_create(hb, 64, opts)
    try:
        assert K.bspmm_plan_info(h).flops == flops0 + 2 * 5 * 64
    finally:
        K.bspmm_destroy(h)
    # different F or options: no hand-over either
    K.bspmm_workspace_bytes(hb, 64, opts)
    h = K.bspmm_create(hb, 32, opts)
    try:
        assert K.bspmm_plan_info(h).F == 32
    finally:
        K.bspmm_destroy(h)
    K.bspmm_workspace_bytes(hb, 64, opts)
    h = K.bspmm_create(hb, 64, K.make_options(flags=K.DRY_RUN, max_tile=32))
    try:
        assert K.bspmm_plan_info(h).tile[0] <= 32
    finally:
        K.bspmm_destroy(h)


def test_square_batches_share_the_schedule_of_both_directions():
    b = W.config2_molecule(graphs=32, F=128)
    h = K.dry_plan(b)
    try:
        f = [(i.op, i.bin, i.row0, i.nrows, i.f0, i.fw, i.workgroup, i.slot) for i in K.bspmm_plan_items(h, False)]
        t = [(i.op, i.bin, i.row0, i.nrows, i.f0, i.fw, i.workgroup, i.slot) for i in K.bspmm_plan_items(h, True)]
        assert f == t and len(f) > 0
    finally:
        K.bspmm_destroy(h)


def test_symmetric_flag_needs_square_operations():
    b = W.random_general(3, F=8, shapes=[(5, 5, 9), (4, 6, 7)], with_dY=False)
    with pytest.raises(K.BspmmError) as e:
        K.dry_plan(b, 8, flags=K.SYMMETRIC)
    assert e.value.code == K.EINVAL
    sq = W.config2_molecule(graphs=8, F=16)
    h = K.dry_plan(sq, 16, flags=K.SYMMETRIC)
    try:
        assert K.bspmm_plan_info(h).transposed_supported == 1
    finally:
        K.bspmm_destroy(h)


def test_empty_batches_through_every_creation_path():
    z32, z64 = np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.int64)
    hc = K.HostCooBatch(z32, z32, z32, z64, z64, z64)
    for flags in (K.DRY_RUN, K.DRY_RUN | K.COO_DIRECT, K.DRY_RUN | K.SYMMETRIC):
        h = K.bspmm_create_coo(hc, 16, K.make_options(flags=flags))
        try:
            info = K.bspmm_plan_info(h)
            assert info.batch == 0 and info.workgroups[0] == 0 and info.workgroups[1] == 0
        finally:
            K.bspmm_destroy(h)
    hb = K.HostBatch(z32, z32, z32, z64, z64, z64, z64)
    h = K.bspmm_create(hb, 16, K.make_options(flags=K.DRY_RUN, front_features=8))
    try:
        assert K.bspmm_plan_info(h).workgroups[0] == 0
    finally:
        K.bspmm_destroy(h)


@pytest.mark.parametrize("block", range(16))
def test_random_batches_and_knobs_keep_the_invariants(block):
    """Seeded random mixes of shapes, feature widths and knobs, both directions."""
    from random_cases import random_case
    for seed in range(16 * block, 16 * block + 16):
        b, opts = random_case(seed, with_dY=False)
        try:
            _check_schedule(b, b.F, **opts)
            _check_schedule(b, b.F, transposed=True, **opts)
        except AssertionError as e:
            raise AssertionError(f"seed {seed} F={b.F} batch={b.batch} opts={opts}: {e}") from e


def test_random_batches_through_the_direct_coo_schedule():
    from random_cases import random_case
    for seed in range(200, 240, 3):
        b, kw = random_case(seed, max_ops=120, max_nnz=120_000, with_dY=False)
        few = {k: v for k, v in kw.items() if k in ("lds_bytes", "min_tile", "max_tile")}
        for transposed in (False, True):
            try:
                _check_direct_coo_schedule(b, b.F, few, transposed)
            except AssertionError as e:
                raise AssertionError(f"seed {seed} F={b.F} {few} transposed={transposed}: {e}") from e


def test_random_summed_groups_keep_the_invariants():
    """Random groups of operations added into one block, both directions; a group that does
    not fit on chip at any tile width is refused as a whole."""
    from random_cases import random_summed_case
    fitted = 0
    for seed in range(60):
        b, opts = random_summed_case(seed, with_dY=False)
        try:
            info, _ = _check_schedule(b, b.F, **opts)
            if info.transposed_supported:
                _check_schedule(b, b.F, transposed=True, **opts)
            fitted += 1
        except K.BspmmError as e:
            assert e.code == K.ETOOBIG, f"seed {seed}: {e}"
        except AssertionError as e:
            raise AssertionError(f"seed {seed} F={b.F} batch={b.batch} opts={opts}: {e}") from e
    assert fitted >= 30


def test_whole_layer_plans_need_uniform_channel_sets():
    """front_features with BSPMM_ACCUMULATE: the channels of a graph (shared layer input, one
    output block) become one item per (tile, row range); every operation must be a channel of
    a set and all sets must have the same number of channels."""
    b = W.config3_multichannel(graphs=40, F=64, channels=4, accumulate=True)
    info, items = _check_schedule(b, 64, flags=K.ACCUMULATE, front_features=32)
    assert info.fused_tasks[0] == 0 and all(it.bin == K.BIN_WORKGROUP for it in items)
    by_task = {}
    for it in items:
        by_task.setdefault(it.workgroup, []).append(it)
    assert all(sorted(m.slot for m in mem) == [0, 1, 2, 3] for mem in by_task.values())
    # channels with an input block each do not share the layer input
    own = W.config3_multichannel(graphs=8, F=64, channels=4, accumulate=True, own_inputs=True)
    # one graph with three channels among graphs with four
    c_off = b.c_row_off.copy()
    c_off[3] = int(b.c_row_off.max()) + int(b.rows.max()) + 7
    odd = dataclasses.replace(b, c_row_off=c_off)
    for bad in (own, odd):
        hb = K.HostBatch(bad.rows, bad.cols, bad.nnz, bad.rpt_off, bad.nz_off, bad.b_row_off,
                         bad.c_row_off)
        with pytest.raises(K.BspmmError) as e:
            K.bspmm_create(hb, 64, K.make_options(flags=K.DRY_RUN | K.ACCUMULATE, front_features=32))
        assert e.value.code in (K.EINVAL, K.ETOOBIG)


def test_large_front_batches_take_a_smaller_lds_budget():
    """A fused-front launch of several rounds of workgroups is planned with a smaller LDS budget
    first (more workgroups per CU); small batches, budgets that do not hold the batch and
    budgets the caller gives are not touched."""
    for graphs, nx, want in [(128, 32, 81920), (300, 64, 81920), (1024, 32, 24576), (1024, 48, 24576),
                             (1024, 64, 40960), (1024, 128, 40960)]:
        b = W.config2_molecule(graphs=graphs, F=128)
        info, _ = _check_schedule(b, 128, front_features=nx)
        assert info.lds_bytes == want, (graphs, nx, info.lds_bytes)
    b = W.config2_molecule(graphs=1024, F=128)
    info, _ = _check_schedule(b, 128, front_features=32, lds_bytes=65536)
    assert info.lds_bytes == 65536
    layer = W.config3_multichannel(graphs=512, F=128, channels=4, accumulate=True)
    info, _ = _check_schedule(layer, 128, flags=K.ACCUMULATE, front_features=32)
    assert info.lds_bytes == 53248
    info, _ = _check_schedule(layer, 128, flags=K.ACCUMULATE, front_features=64)
    assert info.lds_bytes == 81920      # nothing smaller holds four weight tiles beside a graph
    small = W.config3_multichannel(graphs=256, F=128, channels=4, accumulate=True)
    info, _ = _check_schedule(small, 128, flags=K.ACCUMULATE, front_features=32)
    assert info.lds_bytes == 81920


def test_a_plan_is_handed_from_workspace_bytes_to_create_only_for_the_same_batch():
    """bspmm_workspace_bytes keeps the plan it had to make; bspmm_create takes it over when its
    batch has the same contents, and plans afresh when any host array differs (same sizes, other
    output blocks; same everything, other operation sizes)."""
    import dataclasses
    b1 = W.config2_molecule(graphs=12, F=64)
    opts = K.make_options(flags=K.DRY_RUN)

    def hb(b):
        return K.HostBatch(b.rows, b.cols, b.nnz, b.rpt_off, b.nz_off, b.b_row_off, b.c_row_off)

    def items_of(b_sized, b_created):
        K.bspmm_workspace_bytes(hb(b_sized), 64, opts)
        h = K.bspmm_create(hb(b_created), 64, opts)
        got = sorted((it.op, it.row0, it.nrows, it.f0, it.fw) for it in K.bspmm_plan_items(h))
        info = K.bspmm_plan_info(h)
        K.bspmm_destroy(h)
        return got, int(info.effective_bytes[0])

    def fresh(b):
        h = K.bspmm_create(hb(b), 64, opts)
        got = sorted((it.op, it.row0, it.nrows, it.f0, it.fw) for it in K.bspmm_plan_items(h))
        info = K.bspmm_plan_info(h)
        K.bspmm_destroy(h)
        return got, int(info.effective_bytes[0])

    assert items_of(b1, b1) == fresh(b1)
    # the same operations with their output blocks in reverse order
    off = np.concatenate([[0], np.cumsum(b1.rows[::-1][:-1])])[::-1].astype(np.int64)
    b2 = dataclasses.replace(b1, c_row_off=np.ascontiguousarray(off))
    assert items_of(b1, b2) == fresh(b2)
    # another batch of the same length
    b3 = W.config2_molecule(seed=5, graphs=12, F=64)
    assert items_of(b1, b3) == fresh(b3) and fresh(b3) != fresh(b1)


def _lean_of(b, F=None, **opts):
    h = K.dry_plan(b, F if F is not None else b.F, **opts)
    try:
        info = K.bspmm_plan_info(h)
        return [int(info.lean[0]), int(info.lean[1])], info, K.bspmm_plan_items(h)
    finally:
        K.bspmm_destroy(h)


@pytest.mark.parametrize("maker,kw", [(W.config2_molecule, {"F": 64}), (W.config2_molecule, {}),
                                      (W.config4_wide, {"F": 256}), (W.config4_wide, {}),
                                      (W.config5_skewed, {})])
def test_whole_workgroup_launches_take_the_lean_kernel(maker, kw):
    """The benchmark's launches (molecule graphs, wide features, the skewed training batch) are
    made only of whole-workgroup items, staged operations and row blocks of the generic bin, with
    tile rows of a power-of-two number of float4: both directions are marked for the lean
    kernel."""
    b = maker(**kw)
    lean, info, items = _lean_of(b)
    assert lean == [1, 1]
    assert all(it.bin in (K.BIN_WORKGROUP, K.BIN_GENERIC) for it in items)
    for it in items:
        nvec = it.fw // 4
        assert it.fw % 4 == 0 and nvec & (nvec - 1) == 0 and 0 < nvec <= 64


@pytest.mark.parametrize("why,maker,F,opts", [
    ("odd width: scalar path", W.config2_molecule, 63, {}),
    ("tile rows not a power of two", W.config2_molecule, 96, {"min_tile": 96, "max_tile": 96}),
    ("hub rows", W.config2_molecule, 128, {"flags": K.SPLIT_HUB_ROWS}),
    ("padding", W.config2_molecule, 128, {"lds_pad": 4}),
    ("resident workgroups", W.config2_molecule, 128, {"resident_workgroups": 64}),
    ("sub-workgroup slots", W.config2_molecule, 128, {"force_bin": K.BIN_WAVE}),
])
def test_what_the_lean_kernel_does_not_do_keeps_the_general_one(why, maker, F, opts):
    b = maker(F=F)
    lean, _, _ = _lean_of(b, F, **opts)
    assert lean == [0, 0], why


def test_summed_channels_and_fused_fronts_keep_the_general_kernel():
    c = W.config3_multichannel(graphs=32, accumulate=True)
    assert _lean_of(c, flags=K.ACCUMULATE)[0] == [0, 0]
    assert _lean_of(c, flags=K.ACCUMULATE, front_features=32)[0][0] == 0
    # the same channels as separate outputs are plain whole-workgroup items (their transposed
    # products would be sums into the shared input block: not planned without the flag)
    lean, info, _ = _lean_of(W.config3_multichannel(graphs=32))
    assert lean == [1, 0] and not info.transposed_supported


def _stream_of(graphs, F, n_x, chans, seed=3, **kw):
    b = W.config3_multichannel(seed=seed, graphs=graphs, F=F, channels=chans, accumulate=True)
    flags = kw.pop("flags", 0) | K.ACCUMULATE
    h = K.dry_plan(b, F, flags=flags, front_features=n_x, **kw)
    try:
        return [int(v) for v in K.bspmm_plan_info(h).front_stream], b
    finally:
        K.bspmm_destroy(h)


@pytest.mark.parametrize("graphs,F,n_x,chans,kw", [
    (2048, 128, 64, 4, {}), (2048, 128, 32, 4, {}), (600, 128, 16, 4, {}), (1100, 128, 128, 2, {}),
    (600, 128, 64, 3, {}), (600, 128, 32, 5, {}),          # run as four and as eight channels
    (64, 128, 64, 4, {"compute_units": 4}), (64, 64, 32, 8, {"compute_units": 4}),
    (64, 128, 64, 4, {"compute_units": 4, "lds_bytes": 65536}),
])
def test_whole_layers_of_many_rounds_are_streamed(graphs, F, n_x, chans, kw):
    """Plans with front_features and BSPMM_ACCUMULATE whose launch would take many rounds of
    workgroups run as resident workgroups that stream the graphs: every graph is either in a
    list or left to a launch of its own, the launch's LDS stays inside a third of a CU's (half
    for layers of more than four channels; or what the caller gave), and there are workgroups for
    every feature tile."""
    (streamed, workgroups, lds, left), b = _stream_of(graphs, F, n_x, chans, **kw)
    assert streamed > 0 and streamed + left == graphs
    # (five to eight channels: workgroups of eight wavefronts, two per CU)
    assert 0 < lds <= kw.get("lds_bytes", 81920 if chans > 4 else 53248)
    tiles = {2: (32, 64), 3: (16, 32), 4: (16, 32), 5: (16, 32), 8: (16, 32)}[chans]
    assert any(workgroups % (F // t) == 0 for t in tiles)
    assert workgroups <= 3 * kw.get("compute_units", 256) + F // 16


def test_single_channels_stream_from_a_size_of_the_layer_input():
    """One channel per launch: the streaming workgroups take over where the layer input has about
    700,000 elements (on 256 CUs); below that the one-launch kernel is the faster one."""
    def stream_of(graphs, n_x, **kw):
        b = W.config2_molecule(F=128, graphs=graphs)
        h = K.dry_plan(b, 128, front_features=n_x, **kw)
        try:
            return [int(v) for v in K.bspmm_plan_info(h).front_stream]
        finally:
            K.bspmm_destroy(h)
    assert stream_of(256, 64) == [0, 0, 0, 0] and stream_of(384, 64) == [0, 0, 0, 0]
    assert stream_of(512, 32) == [0, 0, 0, 0] and stream_of(200, 128) == [0, 0, 0, 0]
    for graphs, n_x in ((512, 64), (1024, 32), (256, 128), (4096, 128)):
        streamed, workgroups, lds, left = stream_of(graphs, n_x)
        assert streamed + left == graphs and streamed > 0 and workgroups > 0 and 0 < lds <= 53248
    # the size scales with the chip
    assert stream_of(64, 64, compute_units=16)[0] > 0


@pytest.mark.parametrize("why,graphs,F,n_x,chans,kw", [
    ("less than two workgroups per CU", 100, 128, 64, 4, {}),
    ("the caller keeps the one-launch path", 2048, 128, 64, 4, {"flags": K.ONE_FRONT_LAUNCH}),
    ("input width not a multiple of 16", 60, 128, 20, 4, {"compute_units": 1}),
])
def test_what_the_streaming_launch_does_not_do_stays_on_the_one_launch_path(why, graphs, F, n_x,
                                                                            chans, kw):
    stream, _ = _stream_of(graphs, F, n_x, chans, **kw)
    assert stream == [0, 0, 0, 0], why

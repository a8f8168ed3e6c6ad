"""GPU parity for COO / SparseTensor operands (Sec. II-B, Fig. 1 - Fig. 3): plans made from
unsorted (row, column) pairs, through the C ABI, against the CPU oracle's entry-by-entry loop
nest and its stable conversion.

The device-built CSR is index work: bit for bit.  Products: |got - ref| <= 1e-5 * S per
element, exactly 0 where no entry contributes (same bar as the CSR path).
"""
import dataclasses

import numpy as np
import pytest

from paper_1903_11409_amd import bspmm as K
from paper_1903_11409_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = 1e-5
SENTINEL = -12345.0


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    K.lib()   # raises if the HIP library has not been built: no fallback
    return torch


def _owned(off, length, n):
    m = np.zeros(n, dtype=bool)
    for o, l in zip(off, length):
        m[int(o):int(o) + int(l)] = True
    return m


def _assert_close(got, ref, scale, owned, what):
    got = got.astype(np.float64)
    assert np.all(got[~owned] == SENTINEL), f"{what}: rows outside every operation were written"
    g, r, s = got[owned], ref[owned], scale[owned]
    assert not np.any(np.isnan(g)), f"{what}: NaN in output"
    err = np.abs(g - r)
    bad = err > TOL * s
    assert not np.any(bad), (f"{what}: {int(bad.sum())} elements beyond 1e-5*S, worst "
                             f"ratio {float((err / np.maximum(s, 1e-300)).max()):.3e}")
    assert np.all(g[s == 0.0] == 0.0), f"{what}: nonzero where no entry contributes"


def _check(torch, oracle, b, ids, vals, opts=None, what="", transposed=True, csr=True):
    print(f"coo case {what or b.name}: batch={b.batch} F={b.F} nnz={int(b.nnz.sum())}", flush=True)
    plan = K.Plan(b, options=opts, coo=(ids, vals))
    assert plan.validate() == -1
    if csr:
        rp, ci, va = plan.export_csr()
        torch.cuda.synchronize()
        _, erp, eci, eva = oracle.coo_to_csr(b.rows, b.cols, b.nnz, b.nz_off, ids, vals)
        # the oracle keeps the caller's entry offsets, the plan packs operations back to back
        pack = np.concatenate([np.arange(int(o), int(o) + int(n)) for o, n in zip(b.nz_off, b.nnz)]
                              + [np.zeros(0, dtype=np.int64)]).astype(np.int64)
        assert np.array_equal(rp.cpu().numpy(), erp)
        assert np.array_equal(ci.cpu().numpy(), eci[pack])
        assert np.array_equal(va.cpu().numpy(), eva[pack])
    Bd = torch.from_numpy(b.B).cuda()
    Cd = torch.full((b.n_c_rows, b.F), SENTINEL, dtype=torch.float32, device="cuda")
    plan.run(Bd, Cd)
    torch.cuda.synchronize()
    ref, S = oracle.coo_product(b.rows, b.cols, b.nnz, b.nz_off, b.b_row_off, b.c_row_off, ids,
                                vals, b.B, b.n_c_rows)
    _assert_close(Cd.cpu().numpy(), ref, S, _owned(b.c_row_off, b.rows, b.n_c_rows),
                  (what or b.name) + " coo")
    if transposed and b.dY is not None:
        Yd = torch.from_numpy(b.dY).cuda()
        Gd = torch.full((b.n_b_rows, b.F), SENTINEL, dtype=torch.float32, device="cuda")
        plan.run_transposed(Yd, Gd)
        torch.cuda.synchronize()
        ref, S = oracle.coo_product(b.rows, b.cols, b.nnz, b.nz_off, b.b_row_off, b.c_row_off,
                                    ids, vals, b.dY, b.n_b_rows, transposed_=True)
        _assert_close(Gd.cpu().numpy(), ref, S, _owned(b.b_row_off, b.cols, b.n_b_rows),
                      (what or b.name) + " coo transposed")
    return plan


@pytest.mark.parametrize("maker", [
    lambda: W.config1_tiny(),
    lambda: W.config2_molecule(),                                    # the headline batch
    lambda: W.config3_multichannel(),
    lambda: W.config4_wide(F=256),
    lambda: W.config5_skewed(),
    lambda: W.config5_skewed(graphs=200, F=64, asymmetric=True),
])
def test_workload_configurations_from_coo(torch_cuda, oracle, maker):
    b = maker()
    ids, vals = W.coo_view(b, seed=W.config_seed(9))
    _check(torch_cuda, oracle, b, ids, vals)


@pytest.mark.parametrize("F", [1, 5, 64, 100])
def test_ragged_repeated_pairs_and_empty_operations(torch_cuda, oracle, F):
    b = W.random_general(91, F=F, shapes=[(9, 5, 40), (5, 9, 40), (30, 30, 0), (1, 1, 1),
                                          (0, 0, 0), (17, 17, 60), (300, 200, 5000),
                                          (1, 64, 64), (64, 1, 64)], shuffle_blocks=True)
    ids, vals = W.coo_view(b, seed=F)
    _check(torch_cuda, oracle, b, ids, vals)


def test_entry_offsets_with_gaps_in_any_order(torch_cuda, oracle):
    """The caller's entry offsets need be neither dense nor increasing."""
    b = W.config5_skewed(graphs=40, F=32, asymmetric=True)
    ids, vals = W.coo_view(b, seed=4)
    rng = np.random.default_rng(11)
    order = rng.permutation(b.batch)
    new_off = np.zeros(b.batch, dtype=np.int64)
    cur = 5
    for i in order:
        new_off[i] = cur
        cur += int(b.nnz[i]) + int(rng.integers(0, 7))
    ids2 = np.full(2 * cur, -7, dtype=np.int32)        # gaps hold invalid indices: never read
    vals2 = np.full(cur, np.nan, dtype=np.float32)
    for i in range(b.batch):
        o, n, z = int(b.nz_off[i]), int(new_off[i]), int(b.nnz[i])
        ids2[2 * n:2 * (n + z)] = ids[2 * o:2 * (o + z)]
        vals2[n:n + z] = vals[o:o + z]
    b2 = dataclasses.replace(b, nz_off=new_off)
    _check(torch_cuda, oracle, b2, ids2, vals2)


def test_conversion_falls_back_to_global_scratch(torch_cuda, oracle):
    """An operation whose counters and positions exceed LDS sorts through device scratch."""
    b = W.random_general(78, F=8, shapes=[(4000, 3000, 20000), (10, 10, 30)])
    ids, vals = W.coo_view(b, seed=3)
    _check(torch_cuda, oracle, b, ids, vals)


def test_hub_rows_from_coo(torch_cuda, oracle):
    b = W.hub_batch(5, F=64, n=700)
    ids, vals = W.coo_view(b, seed=6)
    _check(torch_cuda, oracle, b, ids, vals)
    _check(torch_cuda, oracle, b, ids, vals, opts=K.make_options(flags=K.SPLIT_HUB_ROWS),
           what="hub split", csr=False)


def test_channel_sum_from_coo(torch_cuda, oracle):
    b = W.config3_multichannel(graphs=64, F=128, accumulate=True, with_dY=True)
    ids, vals = W.coo_view(b, seed=8)
    _check(torch_cuda, oracle, b, ids, vals, opts=K.make_options(flags=K.ACCUMULATE))


def test_coo_and_csr_plans_agree_bitwise_and_runs_repeat(torch_cuda):
    """Entries in stored order give the very CSR the batch holds: same bits out; and the same
    plan run twice gives the same bits (no atomics on the output)."""
    torch = torch_cuda
    b = W.config2_molecule()
    ids, vals = W.coo_view(b, shuffle=False)
    pc, p0 = K.Plan(b, coo=(ids, vals)), K.Plan(b)
    Bd = torch.from_numpy(b.B).cuda()
    out = [torch.empty((b.n_c_rows, b.F), dtype=torch.float32, device="cuda") for _ in range(3)]
    pc.run(Bd, out[0])
    p0.run(Bd, out[1])
    pc.run(Bd, out[2])
    torch.cuda.synchronize()
    assert torch.equal(out[0], out[1]) and torch.equal(out[0], out[2])
    ids2, vals2 = W.coo_view(b, seed=1)
    ps = K.Plan(b, coo=(ids2, vals2))
    o1 = torch.empty_like(out[0]); o2 = torch.empty_like(out[0])
    ps.run(Bd, o1); ps.run(Bd, o2)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2)


def test_validate_reports_out_of_range_pairs_and_the_run_skips_them(torch_cuda, oracle):
    torch = torch_cuda
    b = W.config2_molecule(graphs=16, F=32)
    ids, vals = W.coo_view(b, seed=2)
    bad = ids.copy()
    z0 = int(b.nz_off[5])
    bad[2 * (z0 + 1) + 1] = int(b.cols[5])            # column one past the end
    z1 = int(b.nz_off[11])
    bad[2 * (z1 + 2)] = -1                            # negative row
    plan = K.Plan(b, coo=(bad, vals))
    assert plan.validate() == 5
    # the product of the remaining entries is still right: drop the two entries for the oracle
    keep = np.ones(vals.shape[0], dtype=bool)
    keep[z0 + 1] = keep[z1 + 2] = False
    nnz2 = b.nnz.copy(); nnz2[5] -= 1; nnz2[11] -= 1
    ids_k = bad.reshape(-1, 2)[keep].reshape(-1)
    vals_k = vals[keep]
    off2 = np.zeros(b.batch, dtype=np.int64); off2[1:] = np.cumsum(nnz2[:-1])
    ref, S = oracle.coo_product(b.rows, b.cols, nnz2, off2, b.b_row_off, b.c_row_off, ids_k,
                                vals_k, b.B, b.n_c_rows)
    Cd = torch.full((b.n_c_rows, b.F), SENTINEL, dtype=torch.float32, device="cuda")
    plan.run(torch.from_numpy(b.B).cuda(), Cd)
    torch.cuda.synchronize()
    _assert_close(Cd.cpu().numpy(), ref, S, _owned(b.c_row_off, b.rows, b.n_c_rows), "skipped pairs")


def test_export_csr_needs_a_coo_plan(torch_cuda):
    b = W.config1_tiny()
    plan = K.Plan(b)
    with pytest.raises(K.BspmmError) as e:
        plan.export_csr()
    assert e.value.code == K.ESTATE


# ---------------------------------------------------------------------------------------------
# BSPMM_COO_DIRECT: the kernel of Fig. 3 / Fig. 5(a,b), no conversion
# ---------------------------------------------------------------------------------------------
DIRECT = dict(flags=K.COO_DIRECT)


@pytest.mark.parametrize("maker", [
    lambda: W.config1_tiny(),
    lambda: W.config2_molecule(),                                    # the headline batch
    lambda: W.config4_wide(F=512),
    lambda: W.config5_skewed(),
    lambda: W.config5_skewed(graphs=200, F=64, asymmetric=True),
])
def test_direct_workload_configurations(torch_cuda, oracle, maker):
    b = maker()
    ids, vals = W.coo_view(b, seed=W.config_seed(9))
    _check(torch_cuda, oracle, b, ids, vals, opts=K.make_options(**DIRECT), what=b.name + " direct",
           csr=False)


def test_direct_shared_inputs_forward_only(torch_cuda, oracle):
    b = W.config3_multichannel()
    ids, vals = W.coo_view(b, seed=12)
    plan = _check(torch_cuda, oracle, b, ids, vals, opts=K.make_options(**DIRECT),
                  what="cfg3 direct", csr=False, transposed=False)
    Y = torch_cuda.zeros((b.n_c_rows, b.F), device="cuda")
    G = torch_cuda.zeros((b.n_b_rows, b.F), device="cuda")
    with pytest.raises(K.BspmmError) as e:
        plan.run_transposed(Y, G)
    assert e.value.code == K.ESTATE
    with pytest.raises(K.BspmmError) as e:
        plan.export_csr()
    assert e.value.code == K.ESTATE


@pytest.mark.parametrize("F", [1, 5, 64, 100, 260])
def test_direct_ragged_repeated_pairs_and_empty_operations(torch_cuda, oracle, F):
    b = W.random_general(92, F=F, shapes=[(9, 5, 40), (5, 9, 40), (30, 30, 0), (1, 1, 1),
                                          (0, 0, 0), (17, 17, 60), (300, 200, 5000),
                                          (1, 64, 64), (64, 1, 64)], shuffle_blocks=True)
    ids, vals = W.coo_view(b, seed=F)
    _check(torch_cuda, oracle, b, ids, vals, opts=K.make_options(**DIRECT), what=f"direct F={F}",
           csr=False)


@pytest.mark.parametrize("kw", [{"lds_bytes": 4096}, {"lds_bytes": 65536}, {"max_tile": 64},
                                {"min_tile": 8, "target_workgroups": 5000},
                                {"target_workgroups": 1}, {"wg_passes": -1}])
def test_direct_row_ranges_and_knobs(torch_cuda, oracle, kw):
    """Tiles that cannot hold all rows of an operation are cut into row ranges."""
    b = W.random_general(93, F=96, shapes=[(4000, 3000, 20000), (10, 10, 30), (700, 700, 9000)])
    ids, vals = W.coo_view(b, seed=3)
    _check(torch_cuda, oracle, b, ids, vals, opts=K.make_options(**DIRECT, **kw),
           what=f"direct {kw}", csr=False)


def test_direct_hub_rows_and_skipped_pairs(torch_cuda, oracle):
    torch = torch_cuda
    b = W.hub_batch(5, F=64, n=700)
    ids, vals = W.coo_view(b, seed=6)
    _check(torch, oracle, b, ids, vals, opts=K.make_options(**DIRECT), what="hub direct", csr=False)
    # out-of-range pairs are reported by validate and left out of the product
    b = W.config2_molecule(graphs=16, F=32)
    ids, vals = W.coo_view(b, seed=2)
    bad = ids.copy()
    z0 = int(b.nz_off[5])
    bad[2 * (z0 + 1) + 1] = int(b.cols[5])
    plan = K.Plan(b, coo=(bad, vals), options=K.make_options(**DIRECT))
    assert plan.validate() == 5
    good_ids, good_vals = ids.copy(), vals.copy()
    good_vals[z0 + 1] = 0.0                            # same product as leaving the entry out
    ref, S = oracle.coo_product(b.rows, b.cols, b.nnz, b.nz_off, b.b_row_off, b.c_row_off,
                                good_ids, good_vals, b.B, b.n_c_rows)
    Cd = torch.full((b.n_c_rows, b.F), SENTINEL, dtype=torch.float32, device="cuda")
    plan.run(torch.from_numpy(b.B).cuda(), Cd)
    torch.cuda.synchronize()
    _assert_close(Cd.cpu().numpy(), ref, S, _owned(b.c_row_off, b.rows, b.n_c_rows), "direct skipped")


def test_direct_scalar_path_for_unaligned_operands(torch_cuda, oracle):
    torch = torch_cuda
    b = W.config2_molecule(graphs=24, F=64)
    ids, vals = W.coo_view(b, seed=2)
    plan = K.Plan(b, coo=(ids, vals), options=K.make_options(**DIRECT))
    ld = b.F + 3
    Bd = torch.zeros((b.n_b_rows, ld), dtype=torch.float32, device="cuda")
    Bd[:, :b.F] = torch.from_numpy(b.B).cuda()
    store = torch.full((b.n_c_rows * ld + 9,), SENTINEL, dtype=torch.float32, device="cuda")
    Cd = store[1:1 + b.n_c_rows * ld].view(b.n_c_rows, ld)
    plan.run(Bd, Cd)
    torch.cuda.synchronize()
    ref, S = oracle.coo_product(b.rows, b.cols, b.nnz, b.nz_off, b.b_row_off, b.c_row_off, ids,
                                vals, b.B, b.n_c_rows)
    _assert_close(Cd[:, :b.F].cpu().numpy(), ref, S, _owned(b.c_row_off, b.rows, b.n_c_rows),
                  "direct unaligned")
    assert torch.all(Cd[:, b.F:] == SENTINEL) and float(store[0]) == SENTINEL


@pytest.mark.parametrize("block", range(4))
def test_random_batches_and_knobs_from_coo(torch_cuda, oracle, block):
    """Seeded random shapes, feature widths and knobs: the converted route with every knob,
    the direct kernel on every third case with the knobs it knows."""
    from random_cases import random_case
    for seed in range(200 + 10 * block, 200 + 10 * block + 10):
        b, kw = random_case(seed, max_ops=120, max_nnz=120_000)
        ids, vals = W.coo_view(b, seed=seed)
        flags = kw.pop("flags", 0)
        force_bin = kw.pop("force_bin", None)
        what = f"seed {seed} {kw} flags={flags} bin={force_bin}"
        _check(torch_cuda, oracle, b, ids, vals, what=what,
               opts=K.make_options(flags=flags, force_bin=force_bin, **kw))
        if seed % 3 == 0:
            few = {k: v for k, v in kw.items() if k in ("lds_bytes", "min_tile", "max_tile")}
            _check(torch_cuda, oracle, b, ids, vals, what=what + " direct", csr=False,
                   opts=K.make_options(flags=K.COO_DIRECT, **few))


@pytest.mark.parametrize("own_inputs", [False, True])
def test_channel_sum_from_coo(torch_cuda, oracle, own_inputs):
    """BSPMM_ACCUMULATE on a plan made from COO operands: the summed sets are merged from the CSR
    arrays the conversion built in the workspace."""
    torch = torch_cuda
    b = W.config3_multichannel(graphs=64, F=64, accumulate=True, own_inputs=own_inputs, with_dY=True)
    ids, vals = W.coo_view(b, seed=12)
    plan = K.Plan(b, options=K.make_options(flags=K.ACCUMULATE), coo=(ids, vals))
    Bd = torch.from_numpy(b.B).cuda()
    Cd = torch.full((b.n_c_rows, b.F), SENTINEL, dtype=torch.float32, device="cuda")
    plan.run(Bd, Cd)
    torch.cuda.synchronize()
    ref, S = oracle.forward_batch(b)       # same entries, summed per output block
    _assert_close(Cd.cpu().numpy(), ref, S, _owned(b.c_row_off, b.rows, b.n_c_rows), "coo channel sum")
    Yd = torch.from_numpy(b.dY).cuda()
    Gd = torch.full((b.n_b_rows, b.F), SENTINEL, dtype=torch.float32, device="cuda")
    plan.run_transposed(Yd, Gd)
    torch.cuda.synchronize()
    ref, S = oracle.transposed_batch(b)
    _assert_close(Gd.cpu().numpy(), ref, S, _owned(b.b_row_off, b.cols, b.n_b_rows),
                  "coo channel sum transposed")

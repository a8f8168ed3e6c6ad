"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, element by
element on the same seeded inputs.

Bar (fp32 path, fp64 oracle): |C_gpu - C_ref| <= 1e-5 * S per element with
S = sum_k |A_ik| |B_kj|; where S == 0 (rows without entries) the GPU value must be exactly 0.
fp32 FMA accumulation of a row with d entries is off by at most about d * 2^-24 * S
(6e-8 * d), so 1e-5 leaves room for rows of more than a hundred entries.
Index work (the transposed CSR) is compared bit for bit.
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


def _owned_rows(off, length, n):
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


def _forward(torch, b, opts=None, ld_extra=0, offset=0):
    plan = K.Plan(b, options=opts)
    ld = b.F + ld_extra
    Bd = torch.zeros((b.n_b_rows, ld), dtype=torch.float32, device="cuda")
    Bd[:, :b.F] = torch.from_numpy(b.B).cuda()
    store = torch.full((b.n_c_rows * ld + offset + 8,), SENTINEL, dtype=torch.float32, device="cuda")
    Cd = store[offset:offset + b.n_c_rows * ld].view(b.n_c_rows, ld)
    plan.run(Bd, Cd)
    torch.cuda.synchronize()
    out = Cd[:, :b.F].cpu().numpy()
    if ld_extra:
        assert torch.all(Cd[:, b.F:] == SENTINEL)
    assert float(store[offset + b.n_c_rows * ld:].min()) == SENTINEL
    return plan, out


def _transposed(torch, b, opts=None, plan=None):
    plan = plan or K.Plan(b, options=opts)
    Yd = torch.from_numpy(b.dY).cuda()
    Gd = torch.full((b.n_b_rows, b.F), SENTINEL, dtype=torch.float32, device="cuda")
    plan.run_transposed(Yd, Gd)
    torch.cuda.synchronize()
    return plan, Gd.cpu().numpy()


def _check_forward(torch, oracle, b, opts=None, what="", **kw):
    plan, got = _forward(torch, b, opts, **kw)
    ref, S = oracle.forward_batch(b)
    _assert_close(got, ref, S, _owned_rows(b.c_row_off, b.rows, b.n_c_rows), what or b.name)
    return plan, got


def _check_transposed(torch, oracle, b, opts=None, what="", plan=None):
    plan, got = _transposed(torch, b, opts, plan)
    ref, S = oracle.transposed_batch(b)
    _assert_close(got, ref, S, _owned_rows(b.b_row_off, b.cols, b.n_b_rows),
                  (what or b.name) + " transposed")
    return plan, got


# ---------------------------------------------------------------------------------------------
# the five workload configurations at full size
# ---------------------------------------------------------------------------------------------

def test_config1_tiny(torch_cuda, oracle):
    b = W.config1_tiny()
    plan, _ = _check_forward(torch_cuda, oracle, b)
    assert plan.validate() == -1


@pytest.mark.parametrize("F", [64, 128])
def test_config2_molecule(torch_cuda, oracle, F):
    b = W.config2_molecule(F=F)
    plan, _ = _check_forward(torch_cuda, oracle, b)
    info = plan.info()
    assert info.workgroups[0] > 0 and info.items_in_bin[0][K.BIN_GENERIC] == 0


def test_config3_multichannel_shared_input(torch_cuda, oracle):
    b = W.config3_multichannel()
    plan, got = _check_forward(torch_cuda, oracle, b)
    assert plan.info().transposed_supported == 0
    with pytest.raises(K.BspmmError) as e:
        plan.run_transposed(torch_cuda.zeros((b.n_c_rows, b.F), device="cuda"),
                            torch_cuda.zeros((b.n_b_rows, b.F), device="cuda"))
    assert e.value.code == K.ESTATE
    # row-normalised channels: with B = 1 the rows that have an edge of the channel give 1
    ones = dataclasses.replace(b, B=np.ones_like(b.B))
    _, c1 = _forward(torch_cuda, ones)
    has = np.concatenate([np.diff(b.op_csr(i)[0]) > 0 for i in range(b.batch)])
    assert np.allclose(c1[has], 1.0, rtol=1e-6) and np.all(c1[~has] == 0.0)


@pytest.mark.parametrize("F", [256, 512, 1024])
def test_config4_wide(torch_cuda, oracle, F):
    b = W.config4_wide(F=F)
    _check_forward(torch_cuda, oracle, b)


def test_config5_skewed_forward_and_backward(torch_cuda, oracle):
    b = W.config5_skewed()
    plan, _ = _check_forward(torch_cuda, oracle, b)
    info = plan.info()
    assert info.items_in_bin[0][K.BIN_GENERIC] > 0      # the largest graphs leave LDS
    _check_transposed(torch_cuda, oracle, b, plan=plan)
    assert plan.info().transposed_built == 1


def test_config5_asymmetric_twin_catches_a_missing_transpose(torch_cuda, oracle):
    b = W.config5_skewed(asymmetric=True)
    plan, got = _check_transposed(torch_cuda, oracle, b)
    # the forward product of the same dense operand is NOT within tolerance of A^T dY
    as_fwd = dataclasses.replace(b, B=b.dY)
    wrong, S = oracle.forward_batch(as_fwd)
    assert np.mean(np.abs(got - wrong) > TOL * S) > 0.5


# ---------------------------------------------------------------------------------------------
# index work: the device-built transposed CSR, bit for bit
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("maker", [
    lambda: W.config5_skewed(graphs=200, F=4, asymmetric=True),
    lambda: W.random_general(77, F=4, shapes=[(9, 5, 40), (5, 9, 40), (30, 30, 0), (1, 1, 1),
                                              (0, 0, 0), (17, 17, 60), (300, 200, 5000)]),
    lambda: W.hub_batch(5, F=4, n=700),
    # large enough that counters + positions exceed LDS: the build falls back to global scratch
    lambda: W.random_general(78, F=4, shapes=[(4000, 3000, 20000), (10, 10, 30)]),
])
def test_transposed_csr_bit_exact(torch_cuda, oracle, maker):
    b = maker()
    plan = K.Plan(b, options=K.make_options(flags=K.BUILD_TRANSPOSE))
    rt, ct, vt = plan.export_transposed()
    torch_cuda.cuda.synchronize()
    _, ert, ect, evt = oracle.csr_transpose(b.rows, b.cols, b.nnz, b.rpt_off, b.nz_off, b.rpt,
                                            b.colids, b.values)
    assert np.array_equal(rt.cpu().numpy(), ert)
    # the oracle packs the transposed entries like the input; so do the generators (dense)
    assert np.array_equal(ct.cpu().numpy(), ect)
    assert np.array_equal(vt.cpu().numpy(), evt)
    _check_transposed(torch_cuda, oracle, b, plan=plan)


# ---------------------------------------------------------------------------------------------
# edge cases
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("F", [1, 3, 4, 5, 63, 64, 65, 100, 260])
def test_ragged_shapes_unsorted_duplicates(torch_cuda, oracle, F):
    shapes = [(1, 1, 1), (0, 0, 0), (7, 13, 25), (13, 7, 25), (40, 40, 0), (300, 300, 2000),
              (2, 900, 50), (900, 2, 50), (64, 64, 64), (65, 63, 400), (5, 5, 100)]
    b = W.random_general(500 + F, F=F, shapes=shapes, shuffle_blocks=True)
    plan, _ = _check_forward(torch_cuda, oracle, b, what=f"general F={F}")
    _check_transposed(torch_cuda, oracle, b, plan=plan, what=f"general F={F}")


def test_identity_is_bitwise_and_hub_rows(torch_cuda, oracle):
    b = W.identity_batch(7, F=128, sizes=[1, 5, 33, 200, 700])
    _, got = _forward(torch_cuda, b)
    assert np.array_equal(got, b.B)
    h = W.hub_batch(9, F=64, n=600)
    plan, _ = _check_forward(torch_cuda, oracle, h)
    _check_transposed(torch_cuda, oracle, h, plan=plan)
    small_hub = W.hub_batch(10, F=32, n=100, copies=5)
    _check_forward(torch_cuda, oracle, small_hub)


@pytest.mark.parametrize("maker", [
    lambda: W.hub_batch(21, F=32, n=100, copies=5),        # staged, 8 lanes per row
    lambda: W.hub_batch(22, F=128, n=150, copies=3),       # staged, tile of 32 or more
    lambda: W.hub_batch(23, F=256, n=90, copies=2),        # one wavefront per row
    lambda: W.hub_batch(24, F=64, n=700),                  # generic bin
    lambda: W.hub_batch(25, F=256, n=2000, copies=1),      # generic, wide tile
    lambda: W.hub_batch(26, F=20, n=300),                  # 5 float4 per row: idle lanes
    lambda: W.hub_batch(27, F=63, n=300),                  # scalar path
    lambda: W.config5_skewed(graphs=64, F=128),            # no hub rows at all
])
def test_split_hub_rows(torch_cuda, oracle, maker):
    """Rows with hundreds of entries are split across the workgroup and reduced; results stay
    inside the same tolerance and are bitwise repeatable."""
    b = maker()
    opts = K.make_options(flags=K.SPLIT_HUB_ROWS)
    plan, got = _check_forward(torch_cuda, oracle, b, opts, what=f"hub split {b.name} F={b.F}")
    _check_transposed(torch_cuda, oracle, b, plan=plan, what=f"hub split {b.name} F={b.F}")
    _, again = _forward(torch_cuda, b, opts)
    assert np.array_equal(got, again)


@pytest.mark.parametrize("F", [128, 32, 100, 63, 256])
@pytest.mark.parametrize("own_inputs", [False, True, "apart"])
def test_channel_sum_in_one_pass(torch_cuda, oracle, F, own_inputs):
    """BSPMM_ACCUMULATE: the channels of a graph name one output block and are summed in
    registers (forward), and their transposed products are summed into the shared input
    gradient (transposed).  Shared input: one operation over the summed matrix; an input per
    channel, back to back: one operation over the matrices side by side; "apart" (the blocks of
    channels 0 and 1 swapped, so they are not one block in channel order): fused tasks."""
    b = W.config3_multichannel(graphs=96, F=F, accumulate=True, own_inputs=bool(own_inputs),
                               with_dY=True)
    if own_inputs == "apart":
        off = b.b_row_off.copy()
        off[0::4], off[1::4] = b.b_row_off[1::4], b.b_row_off[0::4]
        b = dataclasses.replace(b, b_row_off=off)
    opts = K.make_options(flags=K.ACCUMULATE)
    plan, got = _check_forward(torch_cuda, oracle, b, opts, what=f"channel sum F={F}")
    info = plan.info()
    assert info.transposed_supported == 1
    assert own_inputs != "apart" or info.fused_tasks[0] > 0
    _check_transposed(torch_cuda, oracle, b, plan=plan, what=f"channel sum F={F}")
    _, again = _forward(torch_cuda, b, opts)
    assert np.array_equal(got, again)


def test_channel_sum_full_size_and_shared_input_gradient(torch_cuda, oracle):
    b = W.config3_multichannel(accumulate=True, with_dY=True)
    opts = K.make_options(flags=K.ACCUMULATE)
    plan, _ = _check_forward(torch_cuda, oracle, b, opts)
    _check_transposed(torch_cuda, oracle, b, plan=plan)
    # the multi-channel configuration as specified (4 outputs per graph, one shared input): forward
    # is unchanged, and the transposed product now sums the 4 channels into the shared block
    c3 = W.config3_multichannel(with_dY=True)
    plan3, _ = _check_forward(torch_cuda, oracle, c3, opts)
    assert plan3.info().fused_tasks[0] == 0
    _check_transposed(torch_cuda, oracle, c3, plan=plan3)
    # unit entries: the channel matrices partition the edges, the sum is the neighbour sum
    u = W.config3_multichannel(graphs=64, F=64, accumulate=True, normalise=False)
    u = dataclasses.replace(u, B=np.ones_like(u.B))
    _, ones = _forward(torch_cuda, u, opts)
    ch = u.meta["channels"]
    deg = np.concatenate([sum(np.diff(u.op_csr(g * ch + k)[0]) for k in range(ch))
                          for g in range(u.n_graphs)])
    assert np.array_equal(ones, np.repeat(deg[:, None], u.F, axis=1).astype(np.float32))


def test_empty_batch_and_all_empty_matrices(torch_cuda, oracle):
    e = W.random_general(1, F=8, shapes=[])
    plan = K.Plan(e)
    plan.run(torch_cuda.zeros((1, 8), device="cuda"), torch_cuda.zeros((1, 8), device="cuda"))
    z = W.random_general(2, F=16, shapes=[(10, 10, 0), (33, 4, 0)])
    _, got = _check_forward(torch_cuda, oracle, z)
    assert np.all(got == 0.0)


@pytest.mark.parametrize("bin_", [K.BIN_WORKGROUP, K.BIN_WAVE, K.BIN_SLICE32, K.BIN_SLICE16,
                                  K.BIN_GENERIC])
@pytest.mark.parametrize("F", [16, 64, 128])
def test_every_bin_alone(torch_cuda, oracle, bin_, F):
    b = W.config2_molecule(graphs=64, F=F)
    b = dataclasses.replace(b, dY=np.random.default_rng(1).standard_normal(
        (b.n_c_rows, F)).astype(np.float32))
    plan, _ = _check_forward(torch_cuda, oracle, b, K.make_options(force_bin=bin_),
                             what=f"bin {K.BIN_NAMES[bin_]} F={F}")
    _check_transposed(torch_cuda, oracle, b, plan=plan)


@pytest.mark.parametrize("kw", [{"lds_pad": 4}, {"lds_pad": 8}, {"min_tile": 16},
                                {"max_tile": 64}, {"lds_bytes": 65536}, {"lds_bytes": 8192},
                                {"lds_bytes": 163840}, {"lds_bytes": 131072, "min_tile": 256},
                                {"target_workgroups": 64}, {"max_passes": 4},
                                {"wg_passes": 1}, {"wg_passes": -1, "target_workgroups": 4096},
                                {"resident_workgroups": 64}, {"resident_workgroups": 24},
                                {"resident_workgroups": 8, "lds_bytes": 16384},
                                {"generic_rows": 8, "lds_bytes": 4096}])
def test_scheduler_knobs_do_not_change_results(torch_cuda, oracle, kw):
    b = W.config5_skewed(graphs=96, F=128)
    plan, _ = _check_forward(torch_cuda, oracle, b, K.make_options(**kw), what=str(kw))
    _check_transposed(torch_cuda, oracle, b, plan=plan, what=str(kw))


def test_scalar_path_for_unaligned_operands(torch_cuda, oracle):
    b = W.config2_molecule(graphs=32, F=64)
    _check_forward(torch_cuda, oracle, b, ld_extra=3, what="ld = F+3")
    _check_forward(torch_cuda, oracle, b, offset=1, what="C misaligned by one float")
    _check_forward(torch_cuda, oracle, b, ld_extra=4, offset=4, what="ld = F+4, aligned")


def test_offsets_beyond_32_bits(torch_cuda, oracle):
    """Leading dimensions of 2^20 floats put the later blocks more than 2^31 elements from
    the base pointers: row offsets must be 64-bit all the way into the kernel."""
    b = W.config2_molecule(graphs=96, F=64)
    ld = 1 << 20
    assert int(b.b_row_off.max()) * ld > 2 ** 31 and int(b.c_row_off.max()) * ld > 2 ** 31
    plan = K.Plan(b)
    Bd = torch_cuda.empty((b.n_b_rows, ld), dtype=torch_cuda.float32, device="cuda")
    Cd = torch_cuda.empty((b.n_c_rows, ld), dtype=torch_cuda.float32, device="cuda")
    Bd[:, :b.F] = torch_cuda.from_numpy(b.B).cuda()
    Cd[:, :b.F + 4] = SENTINEL
    plan.run(Bd, Cd)
    gb = dataclasses.replace(b, dY=np.random.default_rng(2).standard_normal(
        (b.n_c_rows, b.F)).astype(np.float32))
    Cd2 = torch_cuda.empty((b.n_c_rows, ld), dtype=torch_cuda.float32, device="cuda")
    Cd2[:, :b.F] = torch_cuda.from_numpy(gb.dY).cuda()
    Gd = torch_cuda.empty((b.n_b_rows, ld), dtype=torch_cuda.float32, device="cuda")
    Gd[:, :b.F + 4] = SENTINEL
    plan.run_transposed(Cd2, Gd)
    torch_cuda.cuda.synchronize()
    ref, S = oracle.forward_batch(b)
    own = np.ones(b.n_c_rows, dtype=bool)
    _assert_close(Cd[:, :b.F].cpu().numpy(), ref, S, own, "ld = 2^20")
    assert torch_cuda.all(Cd[:, b.F:b.F + 4] == SENTINEL)
    refT, ST = oracle.transposed_batch(gb)
    _assert_close(Gd[:, :b.F].cpu().numpy(), refT, ST, np.ones(b.n_b_rows, dtype=bool),
                  "ld = 2^20 transposed")
    assert torch_cuda.all(Gd[:, b.F:b.F + 4] == SENTINEL)


@pytest.mark.parametrize("case", ["molecule_F128", "molecule_F64_transposed", "tall_narrow", "edgeless",
                                  "wide_rows"])
def test_lean_launch_matches_the_general_kernel_bit_for_bit(torch_cuda, oracle, case):
    """Launches made only of staged workgroup items take the lean kernel; the same batch planned
    with resident workgroups (which the lean kernel does not do) takes the general one.  Same
    order of additions inside a row, so the outputs agree in every bit, and both meet the
    oracle.  Shapes: the headline batch; a transposed product of rectangular operations with
    unsorted, repeated entries and shuffled output blocks; graphs of 300-700 nodes at
    F = 8 (row pointers and entries beyond one trip of the staging code, several row passes);
    operations without any entry; rows of 40-90 entries (several trips of the gather loop)."""
    torch = torch_cuda
    transposed = False
    kw = {}
    if case == "molecule_F128":
        b = W.config2_molecule(F=128)
    elif case == "molecule_F64_transposed":
        rng = np.random.default_rng(31)
        shapes = [(int(rng.integers(1, 90)), int(rng.integers(1, 90)), int(rng.integers(0, 500)))
                  for _ in range(48)]
        b = W.random_general(78, F=64, shapes=shapes, shuffle_blocks=True)
        transposed = True
    elif case == "tall_narrow":
        b = W.random_square(W.config_seed(7), 8, 6, (300, 700), (2, 4))
        kw = {"lds_bytes": 160 * 1024}
    elif case == "edgeless":
        b = W.random_general(77, F=32, shapes=[(20, 20, 0), (5, 9, 0), (9, 5, 17), (0, 0, 0), (31, 31, 0)])
    else:
        b = W.random_square(W.config_seed(7) + 1, 16, 10, (90, 120), (40, 90))
        kw = {"lds_bytes": 160 * 1024}
    lean = K.Plan(b, options=K.make_options(**kw))
    general = K.Plan(b, options=K.make_options(resident_workgroups=4096, **kw))
    d = 1 if transposed else 0
    assert lean.info().lean[d] == 1 and general.info().lean[d] == 0
    if transposed:
        _, got = _transposed(torch, b, plan=lean)
        _, ref_gpu = _transposed(torch, b, plan=general)
        ref, S = oracle.transposed_batch(b)
        own = _owned_rows(b.b_row_off, b.cols, b.n_b_rows)
    else:
        Bd = torch.from_numpy(b.B).cuda()
        outs = []
        for plan in (lean, general):
            Cd = torch.full((b.n_c_rows, b.F), SENTINEL, dtype=torch.float32, device="cuda")
            plan.run(Bd, Cd)
            torch.cuda.synchronize()
            outs.append(Cd.cpu().numpy())
        got, ref_gpu = outs
        ref, S = oracle.forward_batch(b)
        own = _owned_rows(b.c_row_off, b.rows, b.n_c_rows)
    assert np.array_equal(got.view(np.uint32), ref_gpu.view(np.uint32)), f"{case}: kernels differ"
    _assert_close(got, ref, S, own, f"lean kernel, {case}")


def test_run_to_run_determinism(torch_cuda):
    b = W.config5_skewed(graphs=256, F=128)
    _, a = _forward(torch_cuda, b)
    _, c = _forward(torch_cuda, b)
    assert np.array_equal(a, c)
    plan, g1 = _transposed(torch_cuda, b)
    _, g2 = _transposed(torch_cuda, b)
    assert np.array_equal(g1, g2)


def test_linearity_and_relabelling_on_the_gpu(torch_cuda, oracle):
    b = W.config2_molecule(graphs=32, F=32)
    rng = np.random.default_rng(4)
    B1 = (np.round(rng.uniform(-1, 1, b.B.shape) * 1024) / 1024).astype(np.float32)
    B2 = (np.round(rng.uniform(-1, 1, b.B.shape) * 1024) / 1024).astype(np.float32)
    comb = (2.0 * B1 - 0.5 * B2).astype(np.float32)
    _, c1 = _forward(torch_cuda, dataclasses.replace(b, B=B1))
    _, c2 = _forward(torch_cuda, dataclasses.replace(b, B=B2))
    _, c12 = _forward(torch_cuda, dataclasses.replace(b, B=comb))
    _, S = oracle.forward_batch(dataclasses.replace(b, B=np.abs(B1) * 2 + np.abs(B2) * 0.5))
    assert np.all(np.abs(c12.astype(np.float64) - (2.0 * c1.astype(np.float64) - 0.5 * c2)) <= 3 * TOL * S)


def test_validate_finds_the_malformed_operation(torch_cuda):
    b = W.config2_molecule(graphs=16, F=32)
    plan = K.Plan(b)
    assert plan.validate() == -1
    bad = dataclasses.replace(b, colids=b.colids.copy())
    z0 = int(b.nz_off[5])
    bad.colids[z0 + 1] = int(b.cols[5])          # one past the last valid column
    assert K.Plan(bad).validate() == 5
    bad2 = dataclasses.replace(b, rpt=b.rpt.copy())
    r0 = int(b.rpt_off[9])
    bad2.rpt[r0 + 2], bad2.rpt[r0 + 3] = b.rpt[r0 + 3] + 1, b.rpt[r0 + 2]   # not monotone
    assert K.Plan(bad2).validate() == 9


def test_run_argument_errors(torch_cuda):
    b = W.config1_tiny()
    plan = K.Plan(b)
    Bd = torch_cuda.zeros((b.n_b_rows, b.F), device="cuda")
    Cd = torch_cuda.zeros((b.n_c_rows, b.F), device="cuda")
    with pytest.raises(K.BspmmError) as e:
        K.bspmm_run(plan.handle, Bd, Cd, b.F - 1, b.F)
    assert e.value.code == K.EINVAL
    with pytest.raises(K.BspmmError) as e:
        K.bspmm_run(plan.handle, None, Cd, b.F, b.F)
    assert e.value.code == K.EINVAL
    hb = plan.hb
    with pytest.raises(K.BspmmError) as e:
        K.bspmm_create(hb, b.F, None, plan.workspace, 256)
    assert e.value.code == K.ENOSPACE


def test_non_default_stream(torch_cuda, oracle):
    b = W.config2_molecule(graphs=32, F=64)
    s = torch_cuda.cuda.Stream()
    with torch_cuda.cuda.stream(s):
        plan = K.Plan(b)
        Bd = torch_cuda.from_numpy(b.B).cuda()
        Cd = torch_cuda.full((b.n_c_rows, b.F), SENTINEL, dtype=torch_cuda.float32, device="cuda")
        plan.run(Bd, Cd)
    s.synchronize()
    ref, S = oracle.forward_batch(b)
    _assert_close(Cd.cpu().numpy(), ref, S, _owned_rows(b.c_row_off, b.rows, b.n_c_rows), "stream")


def test_plan_borrows_csr_tensors_that_are_already_on_the_device(torch_cuda, oracle):
    """The Python wrapper takes the CSR arrays as device tensors too (a pipeline that builds its
    adjacency lists on the GPU): they are used in place, not copied."""
    import dataclasses
    torch = torch_cuda
    b = W.config5_skewed(graphs=64, F=64, asymmetric=True)
    dev = dataclasses.replace(b, rpt=torch.from_numpy(b.rpt).cuda(),
                              colids=torch.from_numpy(b.colids).cuda(),
                              values=torch.from_numpy(b.values).cuda())
    plan = K.Plan(dev)
    assert plan.rpt.data_ptr() == dev.rpt.data_ptr() and plan.values.data_ptr() == dev.values.data_ptr()
    Bd = torch.from_numpy(b.B).cuda()
    Cd = torch.full((b.n_c_rows, b.F), SENTINEL, dtype=torch.float32, device="cuda")
    plan.run(Bd, Cd)
    torch.cuda.synchronize()
    ref, S = oracle.forward_batch(b)
    _assert_close(Cd.cpu().numpy(), ref, S, _owned_rows(b.c_row_off, b.rows, b.n_c_rows), "device csr")
    _check_transposed(torch, oracle, b, plan=plan, what="device csr")
    assert plan.validate() == -1


def test_symmetric_operands_need_no_transposed_build(torch_cuda, oracle):
    """Symmetrically normalised adjacency matrices equal their transposes: with
    BSPMM_SYMMETRIC the backward product gathers over the forward CSR and nothing is built."""
    torch = torch_cuda
    for b in (W.config5_skewed(graphs=128, F=64), W.config2_molecule(F=32)):
        if b.dY is None:
            b.dY = np.random.default_rng(1).standard_normal((b.n_c_rows, b.F)).astype(np.float32)
        plan = K.Plan(b, options=K.make_options(flags=K.SYMMETRIC))
        _check_transposed(torch, oracle, b, plan=plan, what=b.name + " symmetric flag")
        assert plan.info().transposed_built == 0
        with pytest.raises(K.BspmmError) as e:
            plan.export_transposed()
        assert e.value.code == K.ESTATE
        # and the same bits as the plan that builds the transposed CSR (sorted columns: the
        # stable transpose of a symmetric matrix is the matrix itself, entry for entry)
        built = K.Plan(b)
        Yd = torch.from_numpy(b.dY).cuda()
        G1 = torch.empty((b.n_b_rows, b.F), dtype=torch.float32, device="cuda")
        G2 = torch.empty_like(G1)
        plan.run_transposed(Yd, G1)
        built.run_transposed(Yd, G2)
        torch.cuda.synchronize()
        assert torch.equal(G1, G2)


def test_autograd_wrapper_backward_is_the_transposed_product(torch_cuda, oracle):
    torch = torch_cuda
    from paper_1903_11409_amd.autograd import batched_spmm
    b = W.config5_skewed(graphs=64, F=32, asymmetric=True)
    plan = K.Plan(b)
    Bd = torch.from_numpy(b.B).cuda().requires_grad_(True)
    C = batched_spmm(plan, Bd, b.n_c_rows)
    Yd = torch.from_numpy(b.dY).cuda()
    (C * Yd).sum().backward()
    torch.cuda.synchronize()
    ref, S = oracle.forward_batch(b)
    own = _owned_rows(b.c_row_off, b.rows, b.n_c_rows)
    assert np.all(np.abs(C.detach().cpu().numpy()[own] - ref[own]) <= TOL * S[own])
    G, SG = oracle.transposed_batch(b)
    own_b = _owned_rows(b.b_row_off, b.cols, b.n_b_rows)
    assert np.all(np.abs(Bd.grad.cpu().numpy()[own_b] - G[own_b]) <= TOL * SG[own_b])


@pytest.mark.parametrize("block", range(12))
def test_random_batches_and_knobs(torch_cuda, oracle, block):
    """The seeded random cases of the scheduler's property test, forward and transposed."""
    from random_cases import random_case
    for seed in range(16 * block, 16 * block + 16):
        b, kw = random_case(seed)
        what = f"seed {seed} F={b.F} batch={b.batch} {kw}"
        print(what, flush=True)
        flags = kw.pop("flags", 0)
        force_bin = kw.pop("force_bin", None)
        opts = K.make_options(flags=flags, force_bin=force_bin, **kw)
        plan, _ = _check_forward(torch_cuda, oracle, b, opts, what=what)
        if plan.info().transposed_supported:
            _check_transposed(torch_cuda, oracle, b, plan=plan, what=what)


@pytest.mark.parametrize("block", range(4))
def test_random_summed_groups(torch_cuda, oracle, block):
    """Random groups of one to eight operations added into one block (rectangular members,
    shared or own inputs, any feature width), forward and transposed; groups that do not fit
    on chip are refused at plan creation and skipped here."""
    from random_cases import random_summed_case
    ran = 0
    for seed in range(15 * block, 15 * block + 15):
        b, kw = random_summed_case(seed)
        what = f"summed seed {seed} F={b.F} batch={b.batch} {kw}"
        print(what, flush=True)
        opts = K.make_options(**kw)
        try:
            plan, _ = _check_forward(torch_cuda, oracle, b, opts, what=what)
        except K.BspmmError as e:
            assert e.code == K.ETOOBIG, what
            continue
        ran += 1
        if plan.info().transposed_supported:
            _check_transposed(torch_cuda, oracle, b, plan=plan, what=what)
    assert ran >= 5


def test_summed_groups_take_a_larger_lds_budget_when_they_need_it(torch_cuda, oracle):
    """Four channels of graphs with many hundred nodes do not fit the default 24 KiB together:
    with lds_bytes left open the plan moves to 80 KiB, then to the CU's whole 160 KiB, instead
    of refusing."""
    from random_cases import _random_csr
    rng = np.random.default_rng(5)
    for m, per_row, want in [(800, 2, 81920), (1800, 2, 163840)]:
        ops, blocks = [], []
        for g in range(3):
            for _ in range(4):
                rpt, ci, va = _random_csr(rng, m, m, per_row * m, True)
                ops.append((m, m, rpt, ci, va))
                blocks.append(g)
        b = W.assemble("big_summed", 64, ops, blocks, [m] * 3, rng, with_dY=True, n_graphs=3,
                       c_block_of_op=blocks)
        plan, _ = _check_forward(torch_cuda, oracle, b, K.make_options(flags=K.ACCUMULATE),
                                 what=f"summed m={m}")
        info = plan.info()
        assert info.lds_bytes == want and info.transposed_supported
        _check_transposed(torch_cuda, oracle, b, plan=plan, what=f"summed m={m}")
        with pytest.raises(K.BspmmError) as e:      # a budget the caller fixed is kept
            K.Plan(b, options=K.make_options(flags=K.ACCUMULATE, lds_bytes=24576))
        assert e.value.code == K.ETOOBIG


def test_large_batch_of_small_graphs(torch_cuda, oracle):
    """16384 molecule graphs in one launch (many times what the chip holds at once: the
    scheduler packs several small items into a workgroup), forward and transposed."""
    b = W.config2_molecule(seed=77, graphs=16384, F=64)
    b = dataclasses.replace(b, dY=np.random.default_rng(2).standard_normal(
        (b.n_c_rows, b.F)).astype(np.float32))
    plan, _ = _check_forward(torch_cuda, oracle, b, what="16384 graphs")
    info = plan.info()
    assert info.items[0] >= 16384 and info.workgroups[0] < info.items[0]
    _check_transposed(torch_cuda, oracle, b, plan=plan, what="16384 graphs")


def test_runs_replayed_from_a_hip_graph(torch_cuda, oracle):
    """Forward, transposed and channel-sum runs captured in one HIP graph (the one-off device
    builds done at plan creation with BSPMM_BUILD_TRANSPOSE, so that the capture holds the
    products only) and replayed with new operands, eager work and synchronisation in between:
    every replay equals the eager result bit for bit and meets the oracle."""
    torch = torch_cuda
    b = W.config5_skewed(graphs=64, F=64, asymmetric=True)
    c = W.config3_multichannel(graphs=48, F=64, accumulate=True, own_inputs=True, with_dY=True)
    pb = K.Plan(b, options=K.make_options(flags=K.BUILD_TRANSPOSE))
    pc = K.Plan(c, options=K.make_options(flags=K.BUILD_TRANSPOSE | K.ACCUMULATE))
    torch.cuda.synchronize()
    Bb = torch.zeros((b.n_b_rows, 64), device="cuda")
    Cb = torch.empty((b.n_c_rows, 64), device="cuda")
    Yb = torch.zeros((b.n_c_rows, 64), device="cuda")
    Gb = torch.empty((b.n_b_rows, 64), device="cuda")
    Bc = torch.zeros((c.n_b_rows, 64), device="cuda")
    Cc = torch.empty((c.n_c_rows, 64), device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            s = torch.cuda.current_stream().cuda_stream
            pb.run(Bb, Cb, stream=s)
            pb.run_transposed(Yb, Gb, stream=s)
            pc.run(Bc, Cc, stream=s)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    rng = np.random.default_rng(31)
    for rep in range(3):
        nb = rng.uniform(-1, 1, size=b.B.shape).astype(np.float32)
        ny = rng.standard_normal(size=b.dY.shape).astype(np.float32)
        nc = rng.uniform(-1, 1, size=c.B.shape).astype(np.float32)
        Bb.copy_(torch.from_numpy(nb).cuda())
        Yb.copy_(torch.from_numpy(ny).cuda())
        Bc.copy_(torch.from_numpy(nc).cuda())
        for t in (Cb, Gb, Cc):
            t.fill_(SENTINEL)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = [t.cpu().numpy() for t in (Cb, Gb, Cc)]
        eager = [torch.empty_like(t) for t in (Cb, Gb, Cc)]      # eager work between replays
        pb.run(Bb, eager[0])
        pb.run_transposed(Yb, eager[1])
        pc.run(Bc, eager[2])
        torch.cuda.synchronize()
        for a, e in zip(got, eager):
            assert np.array_equal(a, e.cpu().numpy()), f"replay {rep} differs from the eager run"
        b2 = dataclasses.replace(b, B=nb, dY=ny)
        ref, S = oracle.forward_batch(b2)
        _assert_close(got[0], ref, S, _owned_rows(b.c_row_off, b.rows, b.n_c_rows), f"replay {rep}")
        ref, S = oracle.transposed_batch(b2)
        _assert_close(got[1], ref, S, _owned_rows(b.b_row_off, b.cols, b.n_b_rows), f"replay {rep} transposed")
        ref, S = oracle.forward_batch(dataclasses.replace(c, B=nc))
        _assert_close(got[2], ref, S, _owned_rows(c.c_row_off, c.rows, c.n_c_rows), f"replay {rep} channel sum")


def test_first_run_inside_a_stream_capture(torch_cuda, oracle):
    """A plan whose first runs are recorded into a HIP graph: the one-off builds (transposed CSR,
    merged CSR of summed sets) are recorded with them and do not count as done, so an eager run
    before the first replay is still correct, and so is every replay."""
    torch = torch_cuda
    c = W.config3_multichannel(graphs=40, F=64, accumulate=True, own_inputs=True, with_dY=True)
    plan = K.Plan(c, options=K.make_options(flags=K.ACCUMULATE))
    Bd = torch.from_numpy(c.B).cuda()
    Yd = torch.from_numpy(c.dY).cuda()
    Cg = torch.full((c.n_c_rows, 64), SENTINEL, device="cuda")
    Gg = torch.full((c.n_b_rows, 64), SENTINEL, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            s = torch.cuda.current_stream().cuda_stream
            plan.run(Bd, Cg, stream=s)
            plan.run_transposed(Yd, Gg, stream=s)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    assert plan.info().transposed_built == 0
    refC, SC = oracle.forward_batch(c)
    refG, SG = oracle.transposed_batch(c)
    ownC = _owned_rows(c.c_row_off, c.rows, c.n_c_rows)
    ownG = _owned_rows(c.b_row_off, c.cols, c.n_b_rows)
    Ce = torch.full_like(Cg, SENTINEL)
    Ge = torch.full_like(Gg, SENTINEL)
    plan.run(Bd, Ce)                    # eager, before the graph has ever run
    plan.run_transposed(Yd, Ge)
    torch.cuda.synchronize()
    _assert_close(Ce.cpu().numpy(), refC, SC, ownC, "eager before the first replay")
    _assert_close(Ge.cpu().numpy(), refG, SG, ownG, "eager transposed before the first replay")
    for rep in range(2):
        Cg.fill_(SENTINEL)
        Gg.fill_(SENTINEL)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Cg, Ce) and torch.equal(Gg, Ge), f"replay {rep}"

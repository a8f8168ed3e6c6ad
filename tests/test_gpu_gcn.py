"""GPU parity for the fused front of the batched graph-convolution layer (Fig. 7: MatMul, Add,
BatchedSpMM in one launch per channel): bspmm_run_gcn through the C ABI against the CPU oracle's
three steps in fp64.

Bar: |Y_gpu - Y_ref| <= tol * T per element with T = sum_p |a_p| (sum_t |X||W| + |bias|) and
tol = max(1e-5, (n_X + d_max + 2) * 2^-23): an output element is a chain of n_X fused
multiply-adds on the matrix cores, one add of the bias and d row-gather FMAs, each rounding to
fp32 (2^-24 relative), so the worst case is (n_X + d + 1) * 2^-24 * T; the factor 2 covers the
different association inside the matrix instruction.  Exactly 0 where T == 0.
"""
import numpy as np
import pytest

from paper_1903_11409_amd import bspmm as K
from paper_1903_11409_amd import workloads as W

pytestmark = pytest.mark.gpu
SENTINEL = -12345.0


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    K.lib()   # raises if the HIP library has not been built: no fallback
    return torch


def _layer(b, n_x, seed, channels=1):
    rng = np.random.default_rng(seed)
    X = rng.uniform(-1, 1, size=(b.n_b_rows, n_x)).astype(np.float32)
    Ws = [rng.uniform(-1, 1, size=(n_x, b.F)).astype(np.float32) / np.float32(np.sqrt(n_x))
          for _ in range(channels)]
    biases = [rng.uniform(-1, 1, size=b.F).astype(np.float32) for _ in range(channels)]
    return X, Ws, biases


def _owned(off, length, n):
    m = np.zeros(n, dtype=bool)
    for o, l in zip(off, length):
        m[int(o):int(o) + int(l)] = True
    return m


def _assert_close(got, ref, T, owned, tol, what):
    got = got.astype(np.float64)
    assert np.all(got[~owned] == SENTINEL), f"{what}: rows outside every operation were written"
    g, r, t = got[owned], ref[owned], T[owned]
    assert not np.any(np.isnan(g)), f"{what}: NaN in output"
    err = np.abs(g - r)
    bad = err > tol * t
    assert not np.any(bad), (f"{what}: {int(bad.sum())} elements beyond {tol:.1e}*T, worst ratio "
                             f"{float((err / np.maximum(t, 1e-300)).max()):.3e}")
    assert np.all(g[t == 0.0] == 0.0), f"{what}: nonzero where nothing contributes"


def _tol(b, n_x):
    dmax = max((int(np.diff(b.op_csr(i)[0]).max()) if int(b.rows[i]) else 0) for i in range(b.batch))
    return max(1e-5, (n_x + dmax + 2) * 2.0 ** -23)


def _run_and_check(torch, oracle, b, n_x, seed=1, what="", **kw):
    print(f"gcn case {what or b.name}: batch={b.batch} F={b.F} n_X={n_x} {kw}", flush=True)
    X, Ws, biases = _layer(b, n_x, seed)
    plan = K.Plan(b, options=K.make_options(front_features=n_x, **kw))
    Xd, Wd, bd = (torch.from_numpy(a).cuda() for a in (X, Ws[0], biases[0]))
    Yd = torch.full((b.n_c_rows, b.F), SENTINEL, dtype=torch.float32, device="cuda")
    plan.run_gcn(Xd, Wd, bd, Yd)
    torch.cuda.synchronize()
    ref, T = oracle.gcn_channel(b, X, Ws[0], biases[0])
    _assert_close(Yd.cpu().numpy(), ref, T, _owned(b.c_row_off, b.rows, b.n_c_rows), _tol(b, n_x),
                  what or b.name)
    return plan


@pytest.mark.parametrize("maker,n_x", [
    (lambda: W.config1_tiny(), 64),
    (lambda: W.config2_molecule(), 64),             # the headline batch as a layer
    (lambda: W.config2_molecule(F=64), 76),         # n_X not a multiple of 16 or 64
    (lambda: W.config2_molecule(F=256), 128),       # X_i of the larger graphs in several passes
    (lambda: W.config3_multichannel(), 32),         # channels sharing their input block
    (lambda: W.config4_wide(F=512), 64),
    (lambda: W.random_general(55, F=64, shapes=[(200, 180, 1500), (150, 150, 900), (12, 300, 80)] * 3), 16),
    (lambda: W.config5_skewed(graphs=256, F=64, asymmetric=True), 64),   # up to 500 nodes: many passes
])
def test_layer_channel_configurations(torch_cuda, oracle, maker, n_x):
    b = maker()
    _run_and_check(torch_cuda, oracle, b, n_x)


@pytest.mark.parametrize("maker,n_x,kw,left", [
    # single channels of two and more workgroups per CU are run by resident workgroups that
    # stream the graphs: for real (600 graphs), and on small batches by telling the scheduler
    # that the chip has few CUs; `left`: graphs that fit the streaming launch in no way run in a
    # launch of their own
    (lambda: W.config2_molecule(graphs=600), 64, {}, False),
    (lambda: W.config2_molecule(graphs=48), 16, {"compute_units": 4}, False),
    (lambda: W.config2_molecule(graphs=48), 32, {"compute_units": 4}, False),
    (lambda: W.config2_molecule(graphs=48, F=64), 64, {"compute_units": 4}, False),
    (lambda: W.config2_molecule(graphs=48, F=256), 128, {"compute_units": 4}, False),
    (lambda: W.config3_multichannel(graphs=64), 32, {"compute_units": 8}, False),    # shared input blocks
    (lambda: W.random_general(55, F=64, shapes=[(100, 90, 700), (60, 60, 300), (12, 150, 80), (150, 20, 300)] * 3),
     16, {"compute_units": 1}, None),
    (lambda: W.config5_skewed(graphs=256, F=64, asymmetric=True), 64, {"compute_units": 32}, True),
    (lambda: W.config4_wide(F=512, graphs=64), 64, {"compute_units": 16}, False),
])
def test_single_channel_streamed(torch_cuda, oracle, maker, n_x, kw, left):
    b = maker()
    plan = _run_and_check(torch_cuda, oracle, b, n_x, **kw)
    info = plan.info()
    print("  streamed graphs / workgroups / LDS / left:", list(info.front_stream), flush=True)
    assert info.front_stream[0] > 0
    if left is not None:
        assert (info.front_stream[3] > 0) == left
    # the later channels of a layer add onto the output
    X, Ws, biases = _layer(b, n_x, 1)
    torch = torch_cuda
    Xd, Wd, bd = (torch.from_numpy(a).cuda() for a in (X, Ws[0], biases[0]))
    base = np.random.default_rng(4).uniform(-1, 1, size=(b.n_c_rows, b.F)).astype(np.float32)
    onto = torch.from_numpy(base).cuda()
    plan.run_gcn(Xd, Wd, bd, onto, accumulate=True)
    torch.cuda.synchronize()
    ref, T = oracle.gcn_channel(b, X, Ws[0], biases[0])
    owned = _owned(b.c_row_off, b.rows, b.n_c_rows)
    got = onto.cpu().numpy()
    assert np.array_equal(got[~owned], base[~owned])
    _assert_close(np.where(owned[:, None], got, SENTINEL), ref + base.astype(np.float64),
                  T + np.abs(base.astype(np.float64)), owned, _tol(b, n_x), "streamed channel, accumulated")
    # and the plan still runs the plain product
    Bd = torch.from_numpy(b.B).cuda()
    Cd = torch.full((b.n_c_rows, b.F), SENTINEL, dtype=torch.float32, device="cuda")
    plan.run(Bd, Cd)
    torch.cuda.synchronize()
    refc, S = oracle.forward_batch(b)
    err = np.abs(Cd.cpu().numpy().astype(np.float64) - refc)[owned]
    assert np.all(err <= 1e-5 * S[owned])


@pytest.mark.parametrize("n_x", [4, 8, 20, 60, 64, 68, 132, 256])
def test_input_widths_and_ragged_operations(torch_cuda, oracle, n_x):
    b = W.random_general(101, F=48, shapes=[(9, 5, 40), (5, 9, 40), (30, 30, 0), (1, 1, 1),
                                            (0, 0, 0), (17, 17, 60), (40, 33, 300), (1, 64, 64),
                                            (64, 1, 64)], shuffle_blocks=True)
    _run_and_check(torch_cuda, oracle, b, n_x, seed=n_x)


@pytest.mark.parametrize("kw", [{"max_tile": 16}, {"max_tile": 64}, {"min_tile": 32},
                                {"wg_passes": 1}, {"lds_bytes": 65536}, {"target_workgroups": 1}])
def test_knobs_do_not_change_the_layer(torch_cuda, oracle, kw):
    b = W.config2_molecule(graphs=48, F=128)
    _run_and_check(torch_cuda, oracle, b, 64, what=f"knobs {kw}", **kw)


def test_channels_accumulate_in_place(torch_cuda, oracle):
    """Y = sum_ch A_ch (X W_ch + bias_ch): one launch per channel, the later ones adding."""
    torch = torch_cuda
    chans, n_x = 3, 64
    bs = [W.config2_molecule(seed=70, graphs=64, F=128) for _ in range(chans)]
    rng = np.random.default_rng(5)
    for bb in bs:
        bb.values = (bb.values * rng.uniform(0.5, 1.5, size=bb.values.shape)).astype(np.float32)
    X, Ws, biases = _layer(bs[0], n_x, 9, channels=chans)
    Xd = torch.from_numpy(X).cuda()
    Yd = torch.full((bs[0].n_c_rows, 128), SENTINEL, dtype=torch.float32, device="cuda")
    Y = T = None
    plans = []
    for c in range(chans):
        plans.append(K.Plan(bs[c], options=K.make_options(front_features=n_x)))
        plans[-1].run_gcn(Xd, torch.from_numpy(Ws[c]).cuda(), torch.from_numpy(biases[c]).cuda(), Yd,
                          accumulate=c > 0)
        Y, T = oracle.gcn_channel(bs[c], X, Ws[c], biases[c], Y, T)
    torch.cuda.synchronize()
    b0 = bs[0]
    _assert_close(Yd.cpu().numpy(), Y, T, _owned(b0.c_row_off, b0.rows, b0.n_c_rows),
                  max(1e-5, chans * (n_x + 10) * 2.0 ** -23), "channel accumulation")


def test_identity_weights_give_the_plain_product_and_plan_still_runs_plain(torch_cuda, oracle):
    """W = I, bias = 0: Y = A X, equal to bspmm_run on the same plan (matrix-core products with
    a single non-zero term are exact)."""
    torch = torch_cuda
    b = W.config2_molecule(graphs=32, F=64)
    plan = K.Plan(b, options=K.make_options(front_features=64))
    Xd = torch.from_numpy(b.B).cuda()
    Y1 = torch.empty((b.n_c_rows, 64), dtype=torch.float32, device="cuda")
    Y2 = torch.empty_like(Y1)
    plan.run_gcn(Xd, torch.eye(64, device="cuda"), torch.zeros(64, device="cuda"), Y1)
    plan.run(Xd, Y2)
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y2)


def test_strided_operands_and_argument_errors(torch_cuda, oracle):
    torch = torch_cuda
    b = W.config2_molecule(graphs=24, F=64)
    n_x = 32
    X, Ws, biases = _layer(b, n_x, 4)
    plan = K.Plan(b, options=K.make_options(front_features=n_x))
    Xd = torch.zeros((b.n_b_rows, n_x + 8), dtype=torch.float32, device="cuda")
    Xd[:, :n_x] = torch.from_numpy(X).cuda()
    Wd = torch.zeros((n_x, 64 + 4), dtype=torch.float32, device="cuda")
    Wd[:, :64] = torch.from_numpy(Ws[0]).cuda()
    Yd = torch.full((b.n_c_rows, 64 + 12), SENTINEL, dtype=torch.float32, device="cuda")
    bd = torch.from_numpy(biases[0]).cuda()
    K.bspmm_run_gcn(plan.handle, Xd, n_x + 8, Wd, 68, bd, Yd, 76)
    torch.cuda.synchronize()
    ref, T = oracle.gcn_channel(b, X, Ws[0], biases[0])
    _assert_close(Yd[:, :64].cpu().numpy(), ref, T, _owned(b.c_row_off, b.rows, b.n_c_rows),
                  _tol(b, n_x), "strided")
    assert torch.all(Yd[:, 64:] == SENTINEL)
    for args in [(Xd, n_x - 4, Wd, 68, bd, Yd, 76),        # ldx < n_X
                 (Xd, n_x + 8, Wd, 60, bd, Yd, 76),        # ldw < F
                 (Xd, n_x + 7, Wd, 68, bd, Yd, 76),        # ldx not a multiple of 4
                 (Xd, n_x + 8, Wd, 68, None, Yd, 76),      # no bias
                 (Xd.data_ptr() + 4, n_x + 8, Wd, 68, bd, Yd, 76)]:   # misaligned X
        with pytest.raises(K.BspmmError) as e:
            K.bspmm_run_gcn(plan.handle, *args)
        assert e.value.code == K.EINVAL
    plain = K.Plan(b)
    with pytest.raises(K.BspmmError) as e:
        K.bspmm_run_gcn(plain.handle, Xd, n_x + 8, Wd, 68, bd, Yd, 76)
    assert e.value.code == K.ESTATE


def test_empty_batch_launches_nothing(torch_cuda):
    torch = torch_cuda
    b = W.random_general(1, F=16, shapes=[], with_dY=False)
    plan = K.Plan(b, options=K.make_options(front_features=8))
    Y = torch.full((4, 16), SENTINEL, device="cuda")
    plan.run_gcn(torch.zeros((4, 8), device="cuda"), torch.zeros((8, 16), device="cuda"),
                 torch.zeros(16, device="cuda"), Y)
    torch.cuda.synchronize()
    assert torch.all(Y == SENTINEL)


@pytest.mark.parametrize("block", range(4))
def test_random_batches_and_knobs_through_the_front(torch_cuda, oracle, block):
    """The seeded random shapes of the scheduler's property test as layer channels: random
    input width, output width a multiple of 16, the knobs the front honours.  A batch with an
    operation that does not fit on chip beside its layer input is refused and skipped."""
    import dataclasses
    from random_cases import random_case
    ran = 0
    for seed in range(300 + 10 * block, 300 + 10 * block + 10):
        b, kw = random_case(seed, max_ops=60, max_nnz=60_000, with_dY=False)
        rng = np.random.default_rng(seed)
        F = [16, 32, 48, 64, 128, 256][int(rng.integers(6))]
        n_x = [4, 8, 20, 32, 64, 100, 128][int(rng.integers(7))]
        if b.n_b_rows == 0 or b.n_c_rows == 0:
            continue
        b = dataclasses.replace(b, F=F, B=np.zeros((b.n_b_rows, F), dtype=np.float32))
        few = {k: v for k, v in kw.items() if k in ("lds_bytes", "target_workgroups", "wg_passes")}
        if "max_tile" in kw:
            few["max_tile"] = max(16, kw["max_tile"])
        try:
            _run_and_check(torch_cuda, oracle, b, n_x, seed=seed, what=f"seed {seed}", **few)
            ran += 1
        except K.BspmmError as e:
            assert e.code == K.ETOOBIG, f"seed {seed}: {e}"
    assert ran >= 4


def _channel(b, c, chans):
    """Sub-batch of channel c of a multichannel batch (operation index = graph * chans + c)."""
    import dataclasses
    sel = slice(c, None, chans)
    return dataclasses.replace(b, rows=b.rows[sel], cols=b.cols[sel], nnz=b.nnz[sel],
                               rpt_off=b.rpt_off[sel], nz_off=b.nz_off[sel],
                               b_row_off=b.b_row_off[sel], c_row_off=b.c_row_off[sel])


@pytest.mark.parametrize("graphs,F,n_x,chans", [(64, 128, 64, 4), (48, 64, 32, 4), (40, 48, 20, 3),
                                                 (24, 256, 128, 2), (128, 128, 64, 4)])
def test_whole_layer_in_one_launch(torch_cuda, oracle, graphs, F, n_x, chans):
    """Y = sum_ch A_ch (X W_ch + bias_ch) (Fig. 7 with the ElementWiseAdd over the channels) in
    ONE launch: a plan with front_features and BSPMM_ACCUMULATE whose channel operations share
    the layer input and the output block; W is the channels' weight matrices one under the
    other, bias one row per channel."""
    _whole_layer_case(torch_cuda, oracle, graphs, F, n_x, chans)


@pytest.mark.parametrize("graphs,F,n_x,chans,kw", [
    # a launch of several rounds of workgroups makes its dense tiles in 32 x 32 blocks: for real
    # (512 graphs), and on small batches by telling the scheduler that the chip has four CUs
    (512, 128, 32, 4, {}),
    (64, 128, 64, 4, {"compute_units": 4}),
    (48, 64, 32, 4, {"compute_units": 4}),
    (40, 64, 20, 3, {"compute_units": 4}),       # 20 = 16 + a partial trip of 4
    (40, 128, 44, 2, {"compute_units": 4}),      # 44 = 32 + a partial trip of 12
    (30, 96, 8, 2, {"compute_units": 4}),        # a partial trip only; 96 columns = three blocks
    (24, 64, 32, 8, {"compute_units": 4, "lds_bytes": 163840}),
])
def test_whole_layer_in_wide_blocks(torch_cuda, oracle, graphs, F, n_x, chans, kw):
    # (BSPMM_ONE_FRONT_LAUNCH: the shapes that would otherwise be streamed stay on this path)
    info = _whole_layer_case(torch_cuda, oracle, graphs, F, n_x, chans, one_launch=True, **kw)
    assert list(info.front_stream) == [0, 0, 0, 0]


@pytest.mark.parametrize("graphs,F,n_x,chans,kw,left", [
    # launches of many rounds are run by resident workgroups that keep their weights in
    # registers and stream the graphs: for real (640 graphs), and on small batches by telling
    # the scheduler that the chip has four CUs; `left` = some graphs exceed the LDS budget of the
    # streaming launch and run in a launch of their own
    (640, 128, 64, 4, {}, None),
    (64, 128, 64, 4, {"compute_units": 4}, None),
    (64, 128, 64, 4, {"compute_units": 4, "lds_bytes": 49152}, False),   # larger graphs in two halves
    (48, 64, 32, 4, {"compute_units": 4}, None),
    (40, 128, 16, 4, {"compute_units": 4}, None),
    (24, 256, 128, 2, {"compute_units": 4}, None),      # one block per wavefront
    (24, 128, 64, 2, {"compute_units": 4}, None),       # two channels: tiles of 64 columns
    (24, 64, 32, 8, {"compute_units": 4, "lds_bytes": 163840}, False),
    # five to eight channels: workgroups of eight wavefronts, one per channel
    (512, 128, 64, 8, {}, None),
    (32, 128, 128, 8, {"compute_units": 4}, None),
    (40, 64, 32, 5, {"compute_units": 4}, None),        # run as eight, three of them empty
    (24, 32, 16, 6, {"compute_units": 4}, None),
    (48, 128, 64, 7, {"compute_units": 4}, None),
    (48, 128, 64, 3, {"compute_units": 4}, None),       # run as four
])
def test_whole_layer_streamed(torch_cuda, oracle, graphs, F, n_x, chans, kw, left):
    info = _whole_layer_case(torch_cuda, oracle, graphs, F, n_x, chans, **kw)
    assert info.front_stream[0] > 0 and info.front_stream[1] > 0
    assert info.front_stream[0] + info.front_stream[3] == graphs
    if left is not None:
        assert (info.front_stream[3] > 0) == left


def test_streamed_layer_agrees_with_the_one_launch_path(torch_cuda):
    """The streaming launch and the one-launch kernel compute the same layer; they differ only
    in the order in which the matrix instructions add up a dense element's n_X products."""
    torch = torch_cuda
    graphs, F, n_x, chans = 64, 128, 64, 4
    b = W.config3_multichannel(seed=564, graphs=graphs, F=F, channels=chans, accumulate=True)
    assert int(b.rows.max()) <= 128      # (more rows than the streaming gather takes: not streamed)
    X, Ws, biases = _layer(b, n_x, 5, channels=chans)
    Xd = torch.from_numpy(X).cuda()
    Wd = torch.from_numpy(np.concatenate(Ws, axis=0)).cuda()
    bd = torch.from_numpy(np.stack(biases)).cuda()
    out = []
    for flags, cus, lds in ((K.ACCUMULATE, 4, 163840), (K.ACCUMULATE | K.ONE_FRONT_LAUNCH, 0, 0)):
        plan = K.Plan(b, options=K.make_options(flags=flags, front_features=n_x, compute_units=cus,
                                                lds_bytes=lds))
        # (the whole chip's LDS as the budget: every graph is streamed)
        assert plan.info().front_stream[0] == (graphs if cus == 4 else 0)
        Yd = torch.full((b.n_c_rows, F), SENTINEL, dtype=torch.float32, device="cuda")
        plan.run_gcn(Xd, Wd, bd, Yd)
        torch.cuda.synchronize()
        out.append(Yd.cpu().numpy().astype(np.float64))
        plan.close()
    scale = np.abs(out[1]).max()
    assert np.abs(out[0] - out[1]).max() <= 1e-5 * scale


def _whole_layer_case(torch, oracle, graphs, F, n_x, chans, **kw):
    b = W.config3_multichannel(seed=500 + graphs, graphs=graphs, F=F, channels=chans, accumulate=True)
    X, Ws, biases = _layer(b, n_x, 11, channels=chans)
    print(f"layer case: graphs={graphs} F={F} n_X={n_x} channels={chans} {kw}", flush=True)
    flags = K.ACCUMULATE | (K.ONE_FRONT_LAUNCH if kw.pop("one_launch", False) else 0)
    plan = K.Plan(b, options=K.make_options(flags=flags, front_features=n_x, **kw))
    info = plan.info()
    print("  streamed graphs / workgroups / LDS / left:", list(info.front_stream), flush=True)
    assert info.fused_tasks[0] == 0
    Xd = torch.from_numpy(X).cuda()
    Wd = torch.from_numpy(np.concatenate(Ws, axis=0)).cuda()
    bd = torch.from_numpy(np.stack(biases)).cuda()
    Yd = torch.full((b.n_c_rows, F), SENTINEL, dtype=torch.float32, device="cuda")
    plan.run_gcn(Xd, Wd, bd, Yd)
    torch.cuda.synchronize()
    Y = T = None
    dmax = 0
    for c in range(chans):
        bc = _channel(b, c, chans)
        Y, T = oracle.gcn_channel(bc, X, Ws[c], biases[c], Y, T)
        dmax += max(int(np.diff(bc.op_csr(i)[0]).max()) if int(bc.rows[i]) else 0 for i in range(bc.batch))
    tol = max(1e-5, chans * (n_x + 2) * 2.0 ** -23 + dmax * 2.0 ** -23)
    # rows no channel writes keep the oracle's NaN marker only where no operation owns them
    owned = _owned(b.c_row_off, b.rows, b.n_c_rows)
    _assert_close(Yd.cpu().numpy(), Y, T, owned, tol, "whole layer")
    again = torch.empty_like(Yd)
    plan.run_gcn(Xd, Wd, bd, again)
    torch.cuda.synchronize()
    assert torch.equal(Yd, again)
    # accumulate != 0 adds the layer onto what the output holds
    base = np.random.default_rng(3).uniform(-1, 1, size=(b.n_c_rows, F)).astype(np.float32)
    onto = torch.from_numpy(base).cuda()
    plan.run_gcn(Xd, Wd, bd, onto, accumulate=True)
    torch.cuda.synchronize()
    got = onto.cpu().numpy()
    assert np.array_equal(got[~owned], base[~owned])
    _assert_close(np.where(owned[:, None], got, SENTINEL), Y + base.astype(np.float64),
                  T + np.abs(base.astype(np.float64)), owned, tol, "whole layer, accumulated")
    return info


@pytest.mark.parametrize("seed", range(8))
def test_random_whole_layers(torch_cuda, oracle, seed, **kw):
    """Random layers: 2 to 8 channels, rectangular channel matrices (the layer input has its own
    row count), empty channels, odd input widths, graphs from one node to a few hundred.  A layer
    that is refused as a whole (a set does not fit on chip beside its layer input) runs channel by
    channel instead."""
    from random_cases import _random_csr
    torch = torch_cuda
    rng = np.random.default_rng(900 + seed)
    chans = int(rng.integers(2, 9))
    F = [16, 32, 48, 64, 128][int(rng.integers(5))]
    n_x = [4, 12, 20, 32, 64, 100][int(rng.integers(6))]
    graphs = [1, 3, 20, 60][int(rng.integers(4))]
    densities = kw.pop("densities", None)     # entries per row of every channel, instead of random ones
    if densities is not None:
        chans, F, n_x, graphs = len(densities), kw.pop("F"), kw.pop("n_x"), kw.pop("graphs")
    ops, b_block_of_op, b_block_rows, c_block_of_op = [], [], [], []
    for g in range(graphs):
        m = int(rng.integers(1, 90)) if rng.random() < 0.9 else int(rng.integers(90, 260))
        k = m if rng.integers(2) else int(rng.integers(1, 90))
        b_block_rows.append(k)
        for c in range(chans):
            per_row = [0.0, 0.5, 1.5, 4.0][int(rng.integers(4))]
            if densities is not None:
                per_row = densities[c]
            rpt, ci, va = _random_csr(rng, m, k, int(per_row * m), bool(rng.integers(2)))
            ops.append((m, k, rpt, ci, va))
            b_block_of_op.append(g)
            c_block_of_op.append(g)
    b = W.assemble("layer", F, ops, b_block_of_op, b_block_rows, rng, n_graphs=graphs,
                   c_block_of_op=c_block_of_op)
    X, Ws, biases = _layer(b, n_x, seed, channels=chans)
    print(f"random layer {seed}: graphs={graphs} channels={chans} F={F} n_X={n_x}", flush=True)
    flags = K.ACCUMULATE | (K.ONE_FRONT_LAUNCH if kw.pop("one_launch", False) else 0)
    Xd = torch.from_numpy(X).cuda()
    Wd = torch.from_numpy(np.concatenate(Ws, axis=0)).cuda()
    bd = torch.from_numpy(np.stack(biases)).cuda()
    Yd = torch.full((b.n_c_rows, F), SENTINEL, dtype=torch.float32, device="cuda")
    try:
        plan = K.Plan(b, options=K.make_options(flags=flags, front_features=n_x, **kw))
        plan.run_gcn(Xd, Wd, bd, Yd)
    except K.BspmmError as e:
        # A set whose channels do not fit on chip together beside their layer input is refused
        # as a whole layer.  What the caller does then: one plan and one launch per channel, the
        # later channels added onto Y.
        assert e.code == K.ETOOBIG
        print(f"random layer {seed}: refused as a whole layer, run channel by channel", flush=True)
        per_channel = [K.Plan(_channel(b, c, chans), options=K.make_options(front_features=n_x, **kw))
                       for c in range(chans)]
        for c, pc in enumerate(per_channel):
            pc.run_gcn(Xd, Wd[c * n_x:(c + 1) * n_x], bd[c], Yd, accumulate=c > 0)
    torch.cuda.synchronize()
    Y = T = None
    dsum = 0
    for c in range(chans):
        bc = _channel(b, c, chans)
        Y, T = oracle.gcn_channel(bc, X, Ws[c], biases[c], Y, T)
        dsum += max(int(np.diff(bc.op_csr(i)[0]).max()) if int(bc.rows[i]) else 0 for i in range(bc.batch))
    tol = max(1e-5, (chans * (n_x + 2) + dsum) * 2.0 ** -23)
    _assert_close(Yd.cpu().numpy(), Y, T, _owned(b.c_row_off, b.rows, b.n_c_rows), tol, f"random layer {seed}")


@pytest.mark.parametrize("densities,n_x,F", [
    ((0.0, 0.05, 0.7, 6.0), 64, 128),      # an empty channel, one with a handful of entries, a full one
    ((0.3, 0.3), 32, 128),
    ((8.0, 8.0, 8.0, 8.0), 32, 64),        # every row of every channel in use
    ((0.0, 0.0, 0.0, 0.0), 16, 64),        # nothing at all: Y = 0
    ((0.5, 0.0, 2.0, 0.1, 8.0, 0.7, 0.0, 1.0), 64, 64),    # eight channels
    ((1.0, 0.2, 0.0, 4.0, 0.6), 32, 128),                  # five, run as eight
    ((0.4, 0.0, 3.0), 16, 32),                             # three, run as four
])
def test_streamed_layer_makes_only_the_rows_in_use(torch_cuda, oracle, densities, n_x, F):
    """Streamed layers of several channels make only the rows of a channel's dense tile that
    an entry of that channel names (the merged CSR is renumbered once per plan): channels from
    empty to full, rectangular channel matrices, graphs of 1 to 260 nodes (the largest are
    taken one at a time, without the lists)."""
    for seed in (61, 62):
        test_random_whole_layers(torch_cuda, oracle, seed, compute_units=1, densities=densities,
                                 n_x=n_x, F=F, graphs=40)


@pytest.mark.parametrize("one_launch", [False, True], ids=["streamed_where_it_can", "one_launch"])
@pytest.mark.parametrize("seed", range(20, 32))
def test_random_whole_layers_in_several_rounds(torch_cuda, oracle, seed, one_launch):
    """The same random layers with the scheduler told that the chip has one CU.  Shapes the
    streaming kernel takes (2 to 8 channels, n_X = 16, 32, 64 or 128) then run as
    resident workgroups, larger graphs in halves or in a launch of their own; with
    BSPMM_ONE_FRONT_LAUNCH, and for every other shape, launches of more than six workgroups count
    as several rounds and (up to 64 input features, tiles of 32 columns or a multiple) make their
    dense tiles in 32 x 32 blocks."""
    test_random_whole_layers(torch_cuda, oracle, seed, compute_units=1, one_launch=one_launch)


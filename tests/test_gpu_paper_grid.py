"""GPU parity on the workload of the paper's preliminary evaluation (Sec. V-A, Fig. 8-10):
batches of random square matrices with a fixed number of entries per row, multiplied

  * batched: one plan, one launch for the whole batch (Sec. IV-C), and
  * non-batched: one plan and one launch per matrix, the route the paper compares against,

both through the C ABI, both against the CPU oracle element by element
(|C - C_ref| <= 1e-5 * sum|A||B|), and against each other bit for bit: a row's entries are
added in stored order with fused multiply-adds whichever bin, tile or launch computes it.

The matrices are seeded stand-ins with the shapes the paper states (batch 50 / 100, dimension
50 with 2 or 3 entries per row and n_B swept; batch 100 with dimension 32-256 and 1-5 entries
per row at n_B = 1024); the paper's own random matrices are not available.
"""
import numpy as np
import pytest

from paper_1903_11409_amd import bspmm as K
from paper_1903_11409_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = 1e-5
SENTINEL = -12345.0

# (name, batch, dimension, entries per row, dense widths n_B)
GRID = [("batch50_dim50_nnz2", 50, 50, 2, (32, 64, 128, 256, 512)),
        ("batch100_dim50_nnz3", 100, 50, 3, (64, 512)),
        ("batch100_dim32-256_nnz1-5", 100, (32, 256), (1, 5), (1024,))]
CASES = [(name, batch, dim, nz, F) for name, batch, dim, nz, widths in GRID for F in widths]


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    K.lib()   # raises if the HIP library has not been built: no fallback
    return torch


def _check(got, ref, scale, what):
    got = got.astype(np.float64)
    assert not np.any(np.isnan(got)), f"{what}: NaN in output"
    assert not np.any(got == SENTINEL), f"{what}: an output row was not written"
    err = np.abs(got - ref)
    bad = err > TOL * scale
    assert not np.any(bad), (f"{what}: {int(bad.sum())} elements beyond 1e-5*S, worst ratio "
                             f"{float((err / np.maximum(scale, 1e-300)).max()):.3e}")
    assert np.all(got[scale == 0.0] == 0.0), f"{what}: nonzero where no entry contributes"


@pytest.mark.parametrize("name,batch,dim,nz,F", CASES, ids=[f"{c[0]}-nB{c[4]}" for c in CASES])
def test_batched_and_one_launch_per_matrix_match_the_oracle(torch_cuda, oracle, name, batch, dim,
                                                            nz, F):
    torch = torch_cuda
    b = W.random_square(W.config_seed(8) + F, F, batch, dim, nz)
    assert b.batch == batch and int(b.rows.min()) >= (dim if np.isscalar(dim) else dim[0])
    ref, S = oracle.forward_batch(b)
    Bd = torch.from_numpy(b.B).cuda()

    # one launch for the batch
    plan = K.Plan(b)
    C_batched = torch.full((b.n_c_rows, F), SENTINEL, dtype=torch.float32, device="cuda")
    plan.run(Bd, C_batched)
    torch.cuda.synchronize()
    assert plan.info().workgroups[0] > 0
    got_batched = C_batched.cpu().numpy()
    _check(got_batched, ref, S, f"{name} n_B={F} batched")

    # one plan and one launch per matrix, all writing their rows of the same packed output
    C_single = torch.full((b.n_c_rows, F), SENTINEL, dtype=torch.float32, device="cuda")
    plans = [K.Plan(b.single(i)) for i in range(b.batch)]
    for p in plans:
        assert p.info().batch == 1
        p.run(Bd, C_single)
    torch.cuda.synchronize()
    got_single = C_single.cpu().numpy()
    _check(got_single, ref, S, f"{name} n_B={F} one launch per matrix")

    assert np.array_equal(got_batched.view(np.uint32), got_single.view(np.uint32)), \
        f"{name} n_B={F}: the batched launch and the per-matrix launches differ in some bit"
    for p in plans:
        p.close()
    plan.close()


def test_one_launch_per_matrix_from_a_hip_graph(torch_cuda, oracle):
    """The per-matrix launches as the benchmark times them: captured into one HIP graph and
    replayed.  Every replay must reproduce the eager result bit for bit."""
    torch = torch_cuda
    F = 64
    b = W.random_square(W.config_seed(8) + 7, F, 50, 50, 2)
    ref, S = oracle.forward_batch(b)
    Bd = torch.from_numpy(b.B).cuda()
    plans = [K.Plan(b.single(i)) for i in range(b.batch)]
    C_eager = torch.full((b.n_c_rows, F), SENTINEL, dtype=torch.float32, device="cuda")
    for p in plans:
        p.run(Bd, C_eager)
    torch.cuda.synchronize()
    eager = C_eager.cpu().numpy()
    _check(eager, ref, S, "eager per-matrix launches")
    C_graph = torch.full((b.n_c_rows, F), SENTINEL, dtype=torch.float32, device="cuda")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for p in plans:
            p.run(Bd, C_graph)
    for replay in range(3):
        C_graph.fill_(SENTINEL)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(C_graph.cpu().numpy().view(np.uint32), eager.view(np.uint32)), \
            f"replay {replay} differs from the eager launches"
    for p in plans:
        p.close()

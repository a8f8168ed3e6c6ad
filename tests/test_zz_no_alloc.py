"""bspmm_create_static: the plan whose workspace is the library's static device array (for callers
that cannot allocate device memory), checked through the C ABI against bspmm_create on a
caller-allocated workspace: same batch, same products, bit for bit, and within the parity bar of
the CPU oracle.  Two calls in a row share the array, the second with a smaller batch, so anything
the first left behind would show.
"""
import ctypes

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


class _Operands:
    """Device copies of a batch's CSR arrays and dense operands, and its host description."""

    def __init__(self, torch, b):
        self.b = b
        self.rpt = torch.from_numpy(b.rpt).cuda()
        self.colids = torch.from_numpy(b.colids).cuda()
        self.values = torch.from_numpy(b.values).cuda()
        self.hb = K.HostBatch(b.rows, b.cols, b.nnz, b.rpt_off, b.nz_off, b.b_row_off, b.c_row_off,
                              self.rpt, self.colids, self.values)
        self.B = torch.from_numpy(b.B).cuda()
        self.dY = torch.from_numpy(b.dY).cuda()


def _products(torch, ops, handle):
    b = ops.b
    C = torch.full((b.n_c_rows, b.F), SENTINEL, dtype=torch.float32, device="cuda")
    G = torch.full((b.n_b_rows, b.F), SENTINEL, dtype=torch.float32, device="cuda")
    K.bspmm_run(handle, ops.B, C, b.F, b.F)
    K.bspmm_run_transposed(handle, ops.dY, G, b.F, b.F)
    torch.cuda.synchronize()
    return C.cpu().numpy(), G.cpu().numpy()


def _within_bar(got, ref, scale, what):
    got = got.astype(np.float64)
    err = np.abs(got - ref)
    assert not np.any(err > TOL * scale), f"{what}: beyond 1e-5*S"
    assert np.all(got[scale == 0.0] == 0.0), f"{what}: nonzero where no entry contributes"


def _compare(torch, oracle, ops, options=None):
    b = ops.b
    # the existing entry point, on a workspace the caller allocates
    nbytes = K.bspmm_workspace_bytes(ops.hb, b.F, options)
    assert nbytes <= K.STATIC_WORKSPACE_BYTES
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    ref_plan = K.bspmm_create(ops.hb, b.F, options, ws, nbytes)
    C_ref, G_ref = _products(torch, ops, ref_plan)
    K.bspmm_destroy(ref_plan)
    # the entry point that allocates nothing
    plan = K.bspmm_create_static(ops.hb, b.F, options)
    C, G = _products(torch, ops, plan)
    assert np.array_equal(C.view(np.uint32), C_ref.view(np.uint32)), f"{b.name}: forward differs"
    assert np.array_equal(G.view(np.uint32), G_ref.view(np.uint32)), f"{b.name}: transposed differs"
    Co, So = oracle.forward_batch(b)
    Go, SGo = oracle.transposed_batch(b)
    _within_bar(C, Co, So, f"{b.name} forward")
    _within_bar(G, Go, SGo, f"{b.name} transposed")
    return plan


def test_static_workspace_plan_matches_the_caller_workspace_plan_twice_in_a_row(torch_cuda, oracle):
    torch = torch_cuda
    # skewed graphs with asymmetric values (a missing transpose would show), generic-bin
    # operations included; then a much smaller batch on the same array
    big = _Operands(torch, W.config5_skewed(graphs=192, F=128, asymmetric=True))
    small = _Operands(torch, W.config5_skewed(seed=W.config_seed(5, 3), graphs=9, F=128, asymmetric=True))
    first = _compare(torch, oracle, big)
    second = _compare(torch, oracle, small)
    # the first plan no longer owns the array: it must refuse to run instead of reading the
    # second plan's tables
    C = torch.empty((big.b.n_c_rows, big.b.F), dtype=torch.float32, device="cuda")
    rc = K.lib().bspmm_run(first, big.B.data_ptr(), C.data_ptr(), big.b.F, big.b.F,
                           torch.cuda.current_stream().cuda_stream)
    assert rc == K.ESTATE
    # and the second still works after that refusal
    C2, _ = _products(torch, small, second)
    Co, So = oracle.forward_batch(small.b)
    _within_bar(C2, Co, So, "second plan, run again")
    K.bspmm_destroy(first)
    K.bspmm_destroy(second)


def test_static_workspace_with_device_builds_inside_create(torch_cuda, oracle):
    """BSPMM_BUILD_TRANSPOSE and BSPMM_ACCUMULATE: the transposed CSR and the merged CSR of the
    summed sets are built into the static array by kernels enqueued inside the call."""
    torch = torch_cuda
    b = W.config3_multichannel(graphs=24, F=64, accumulate=True)
    b.dY = np.random.default_rng(5).standard_normal((b.n_c_rows, b.F)).astype(np.float32)
    ops = _Operands(torch, b)
    plan = _compare(torch, oracle, ops, K.make_options(flags=K.ACCUMULATE | K.BUILD_TRANSPOSE))
    K.bspmm_destroy(plan)


def test_static_workspace_limit_and_arguments(torch_cuda):
    torch = torch_cuda
    # a batch whose transposed CSR alone exceeds the static array
    b = W.config5_skewed(graphs=4096, F=64)
    ops = _Operands(torch, b)
    assert K.bspmm_workspace_bytes(ops.hb, b.F, None) > K.STATIC_WORKSPACE_BYTES
    plan = ctypes.c_void_p(None)
    rc = K.lib().bspmm_create_static(ctypes.byref(plan), ctypes.byref(ops.hb.struct), b.F, None,
                                     torch.cuda.current_stream().cuda_stream)
    assert rc == K.ENOSPACE and not plan.value
    rc = K.lib().bspmm_create_static(ctypes.byref(plan), None, b.F, None, None)
    assert rc == K.EINVAL
    opts = K.make_options(flags=K.DRY_RUN)
    rc = K.lib().bspmm_create_static(ctypes.byref(plan), ctypes.byref(ops.hb.struct), b.F,
                                     ctypes.byref(opts), None)
    assert rc == K.EINVAL

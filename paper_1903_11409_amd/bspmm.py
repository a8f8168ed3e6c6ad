"""Thin ctypes binding of libbspmm.so: argument marshalling only, same names as the C ABI.

Every step of the path (scheduling, staging, the products, the transposed build) runs inside
the library; PyTorch is used for device memory and streams only.  There is no fallback: if the
shared library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbspmm.so")

OK, EINVAL, ENOSPACE, EHIP, EOVERLAP, ESTATE, EBADCSR, ETOOBIG = 0, -1, -2, -3, -4, -5, -6, -7
DRY_RUN, BUILD_TRANSPOSE, FLOOR_PROBE, SPLIT_HUB_ROWS, ACCUMULATE, COO_DIRECT, SYMMETRIC = 1, 2, 4, 8, 16, 32, 64
ONE_FRONT_LAUNCH = 128
BIN_WORKGROUP, BIN_WAVE, BIN_SLICE32, BIN_SLICE16, BIN_GENERIC = 0, 1, 2, 3, 4
NUM_BINS = 5
BIN_COO = 5          # items of a COO_DIRECT plan
BIN_NAMES = ["workgroup", "wave", "slice32", "slice16", "generic"]

_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)


class bspmm_batch(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32),
                ("rows", _i32p), ("cols", _i32p), ("nnz", _i32p),
                ("rpt_off", _i64p), ("nz_off", _i64p), ("b_row_off", _i64p),
                ("c_row_off", _i64p),
                ("rpt", ctypes.c_void_p), ("colids", ctypes.c_void_p),
                ("values", ctypes.c_void_p)]


class bspmm_coo_batch(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32),
                ("rows", _i32p), ("cols", _i32p), ("nnz", _i32p),
                ("nz_off", _i64p), ("b_row_off", _i64p), ("c_row_off", _i64p),
                ("ids", ctypes.c_void_p), ("values", ctypes.c_void_p)]


class bspmm_options(ctypes.Structure):
    _fields_ = [("flags", ctypes.c_uint32), ("force_bin", ctypes.c_int32),
                ("lds_bytes", ctypes.c_int32), ("min_tile", ctypes.c_int32),
                ("max_tile", ctypes.c_int32), ("target_workgroups", ctypes.c_int32),
                ("compute_units", ctypes.c_int32), ("lds_pad", ctypes.c_int32),
                ("max_passes", ctypes.c_int32), ("generic_rows", ctypes.c_int32),
                ("wg_passes", ctypes.c_int32), ("resident_workgroups", ctypes.c_int32),
                ("front_features", ctypes.c_int32), ("reserved_", ctypes.c_int32)]


class bspmm_info(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("F", ctypes.c_int32),
                ("lds_bytes", ctypes.c_int32), ("compute_units", ctypes.c_int32),
                ("tile", ctypes.c_int32 * 2), ("workgroups", ctypes.c_int32 * 2),
                ("tasks", ctypes.c_int32 * 2),
                ("items", ctypes.c_int32 * 2),
                ("items_in_bin", (ctypes.c_int32 * NUM_BINS) * 2),
                ("fused_tasks", ctypes.c_int32 * 2),
                ("transposed_supported", ctypes.c_int32),
                ("transposed_built", ctypes.c_int32),
                ("lean", ctypes.c_int32 * 2),
                ("front_stream", ctypes.c_int32 * 4),
                ("effective_bytes", ctypes.c_int64 * 2), ("flops", ctypes.c_int64),
                ("workspace_bytes", ctypes.c_uint64)]


class bspmm_kernel_resources(ctypes.Structure):
    _fields_ = [("vgprs", ctypes.c_int32), ("sgprs", ctypes.c_int32),
                ("static_lds_bytes", ctypes.c_int32), ("scratch_bytes", ctypes.c_int32),
                ("threads", ctypes.c_int32), ("workgroups_per_cu", ctypes.c_int32),
                ("compute_units", ctypes.c_int32), ("reserved_", ctypes.c_int32)]


class bspmm_item(ctypes.Structure):
    _fields_ = [("op", ctypes.c_int32), ("bin", ctypes.c_int32), ("row0", ctypes.c_int32),
                ("nrows", ctypes.c_int32), ("f0", ctypes.c_int32), ("fw", ctypes.c_int32),
                ("workgroup", ctypes.c_int32), ("slot", ctypes.c_int32)]


EXPORTS = ["bspmm_workspace_bytes", "bspmm_create", "bspmm_run", "bspmm_run_transposed",
           "bspmm_export_transposed", "bspmm_validate", "bspmm_plan_info", "bspmm_plan_items",
           "bspmm_destroy", "bspmm_strerror", "bspmm_last_hip_error",
           "bspmm_workspace_bytes_coo", "bspmm_create_coo", "bspmm_export_csr", "bspmm_run_gcn",
           "bspmm_create_static", "bspmm_kernel_info"]
KERNEL_NAMES = ["lean", "general", "general_scalar", "front", "layer", "build", "build_large", "coo",
                "layer_stream"]
STATIC_WORKSPACE_BYTES = 8 * 1024 * 1024

_lib = None


class BspmmError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = int(code)
        msg = lib().bspmm_strerror(int(code)).decode()
        if code == EHIP:
            msg += f" (hipError {lib().bspmm_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{code}]")


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1903_11409_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        L.bspmm_workspace_bytes.argtypes = [ctypes.POINTER(bspmm_batch), ctypes.c_int32,
                                            ctypes.POINTER(bspmm_options),
                                            ctypes.POINTER(ctypes.c_size_t)]
        L.bspmm_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(bspmm_batch),
                                   ctypes.c_int32, ctypes.POINTER(bspmm_options), vp,
                                   ctypes.c_size_t, vp]
        L.bspmm_create_static.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(bspmm_batch),
                                          ctypes.c_int32, ctypes.POINTER(bspmm_options), vp]
        L.bspmm_run.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int64, vp]
        L.bspmm_run_transposed.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int64, vp]
        L.bspmm_export_transposed.argtypes = [vp, vp, vp, vp, vp]
        L.bspmm_validate.argtypes = [vp, _i32p, vp]
        L.bspmm_workspace_bytes_coo.argtypes = [ctypes.POINTER(bspmm_coo_batch), ctypes.c_int32,
                                                ctypes.POINTER(bspmm_options),
                                                ctypes.POINTER(ctypes.c_size_t)]
        L.bspmm_create_coo.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(bspmm_coo_batch),
                                       ctypes.c_int32, ctypes.POINTER(bspmm_options), vp,
                                       ctypes.c_size_t, vp]
        L.bspmm_export_csr.argtypes = [vp, vp, vp, vp, vp]
        L.bspmm_run_gcn.argtypes = [vp, vp, ctypes.c_int64, vp, ctypes.c_int64, vp, vp,
                                    ctypes.c_int64, ctypes.c_int32, vp]
        L.bspmm_kernel_info.argtypes = [ctypes.c_int32, ctypes.c_int32,
                                        ctypes.POINTER(bspmm_kernel_resources)]
        L.bspmm_plan_info.argtypes = [vp, ctypes.POINTER(bspmm_info)]
        L.bspmm_plan_items.argtypes = [vp, ctypes.c_int32, ctypes.POINTER(bspmm_item),
                                       ctypes.c_int32, _i32p]
        L.bspmm_destroy.argtypes = [vp]
        L.bspmm_destroy.restype = None
        L.bspmm_strerror.argtypes = [ctypes.c_int]
        L.bspmm_strerror.restype = ctypes.c_char_p
        L.bspmm_last_hip_error.argtypes = []
        for n in EXPORTS:
            if n not in ("bspmm_destroy", "bspmm_strerror"):
                getattr(L, n).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(code: int, where: str) -> None:
    if code != OK:
        raise BspmmError(code, where)


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor / raw integer; None stays NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _ld(t, width: int) -> int:
    """Leading dimension of a row-major matrix held in a tensor; a tensor with fewer than two
    rows (torch gives an empty one strides of zero) has none of its own and takes its width."""
    if t.dim() != 2 or t.shape[0] < 2:
        return max(int(width), int(t.shape[-1]) if t.dim() else 0)
    return int(t.stride(0))


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def make_options(flags: int = 0, force_bin: Optional[int] = None, **kw) -> bspmm_options:
    """Options struct; ``force_bin`` takes a BIN_* constant (None = automatic)."""
    o = bspmm_options()
    o.flags = flags
    o.force_bin = 0 if force_bin is None else 1 + int(force_bin)
    for k, v in kw.items():
        if not hasattr(o, k):
            raise TypeError(f"unknown option {k}")
        setattr(o, k, int(v))
    return o


class HostBatch:
    """Keeps the numpy metadata arrays alive and exposes them as a ``bspmm_batch``."""

    def __init__(self, rows, cols, nnz, rpt_off, nz_off, b_row_off, c_row_off,
                 rpt_dev=None, colids_dev=None, values_dev=None):
        as_ = np.ascontiguousarray
        self.arrays = [as_(rows, dtype=np.int32), as_(cols, dtype=np.int32),
                       as_(nnz, dtype=np.int32), as_(rpt_off, dtype=np.int64),
                       as_(nz_off, dtype=np.int64), as_(b_row_off, dtype=np.int64),
                       as_(c_row_off, dtype=np.int64)]
        self.device = (rpt_dev, colids_dev, values_dev)
        s = bspmm_batch()
        s.batch = int(self.arrays[0].shape[0])
        a = self.arrays
        s.rows = a[0].ctypes.data_as(_i32p)
        s.cols = a[1].ctypes.data_as(_i32p)
        s.nnz = a[2].ctypes.data_as(_i32p)
        s.rpt_off = a[3].ctypes.data_as(_i64p)
        s.nz_off = a[4].ctypes.data_as(_i64p)
        s.b_row_off = a[5].ctypes.data_as(_i64p)
        s.c_row_off = a[6].ctypes.data_as(_i64p)
        s.rpt = _ptr(rpt_dev)
        s.colids = _ptr(colids_dev)
        s.values = _ptr(values_dev)
        self.struct = s


class HostCooBatch:
    """Keeps the numpy metadata arrays alive and exposes them as a ``bspmm_coo_batch``."""

    def __init__(self, rows, cols, nnz, nz_off, b_row_off, c_row_off, ids_dev=None,
                 values_dev=None):
        as_ = np.ascontiguousarray
        self.arrays = [as_(rows, dtype=np.int32), as_(cols, dtype=np.int32),
                       as_(nnz, dtype=np.int32), as_(nz_off, dtype=np.int64),
                       as_(b_row_off, dtype=np.int64), as_(c_row_off, dtype=np.int64)]
        self.device = (ids_dev, values_dev)
        s = bspmm_coo_batch()
        a = self.arrays
        s.batch = int(a[0].shape[0])
        s.rows = a[0].ctypes.data_as(_i32p)
        s.cols = a[1].ctypes.data_as(_i32p)
        s.nnz = a[2].ctypes.data_as(_i32p)
        s.nz_off = a[3].ctypes.data_as(_i64p)
        s.b_row_off = a[4].ctypes.data_as(_i64p)
        s.c_row_off = a[5].ctypes.data_as(_i64p)
        s.ids = _ptr(ids_dev)
        s.values = _ptr(values_dev)
        self.struct = s


def bspmm_workspace_bytes_coo(hb: HostCooBatch, F: int,
                              options: Optional[bspmm_options] = None) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().bspmm_workspace_bytes_coo(ctypes.byref(hb.struct), int(F),
                                           ctypes.byref(options) if options is not None else None,
                                           ctypes.byref(out)), "bspmm_workspace_bytes_coo")
    return int(out.value)


def bspmm_create_coo(hb: HostCooBatch, F: int, options: Optional[bspmm_options] = None,
                     workspace=None, workspace_bytes: int = 0, stream=None) -> int:
    """Returns the opaque plan handle (an integer address)."""
    plan = ctypes.c_void_p(None)
    dry = options is not None and (options.flags & DRY_RUN)
    _check(lib().bspmm_create_coo(ctypes.byref(plan), ctypes.byref(hb.struct), int(F),
                                  ctypes.byref(options) if options is not None else None,
                                  _ptr(workspace), int(workspace_bytes),
                                  None if dry else _stream_handle(stream)), "bspmm_create_coo")
    return plan.value


def bspmm_export_csr(plan: int, rpt, colids, values, stream=None) -> None:
    _check(lib().bspmm_export_csr(plan, _ptr(rpt), _ptr(colids), _ptr(values),
                                  _stream_handle(stream)), "bspmm_export_csr")


def bspmm_workspace_bytes(hb: HostBatch, F: int, options: Optional[bspmm_options] = None) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().bspmm_workspace_bytes(ctypes.byref(hb.struct), int(F),
                                       ctypes.byref(options) if options is not None else None,
                                       ctypes.byref(out)), "bspmm_workspace_bytes")
    return int(out.value)


def bspmm_create(hb: HostBatch, F: int, options: Optional[bspmm_options] = None,
                 workspace=None, workspace_bytes: int = 0, stream=None) -> int:
    """Returns the opaque plan handle (an integer address)."""
    plan = ctypes.c_void_p(None)
    dry = options is not None and (options.flags & DRY_RUN)
    _check(lib().bspmm_create(ctypes.byref(plan), ctypes.byref(hb.struct), int(F),
                              ctypes.byref(options) if options is not None else None,
                              _ptr(workspace), int(workspace_bytes),
                              None if dry else _stream_handle(stream)), "bspmm_create")
    return plan.value


def bspmm_create_static(hb: HostBatch, F: int, options: Optional[bspmm_options] = None,
                        stream=None) -> int:
    """Plan whose workspace is the library's static device array; returns the plan handle."""
    plan = ctypes.c_void_p(None)
    _check(lib().bspmm_create_static(ctypes.byref(plan), ctypes.byref(hb.struct), int(F),
                                     ctypes.byref(options) if options is not None else None,
                                     _stream_handle(stream)), "bspmm_create_static")
    return plan.value


def bspmm_run(plan: int, B, C, ldb: int, ldc: int, stream=None) -> None:
    _check(lib().bspmm_run(plan, _ptr(B), _ptr(C), int(ldb), int(ldc), _stream_handle(stream)),
           "bspmm_run")


def bspmm_run_gcn(plan: int, X, ldx: int, W, ldw: int, bias, Y, ldy: int, accumulate: bool = False,
                  stream=None) -> None:
    _check(lib().bspmm_run_gcn(plan, _ptr(X), int(ldx), _ptr(W), int(ldw), _ptr(bias), _ptr(Y),
                               int(ldy), 1 if accumulate else 0, _stream_handle(stream)),
           "bspmm_run_gcn")


def bspmm_run_transposed(plan: int, dY, G, ldy: int, ldg: int, stream=None) -> None:
    _check(lib().bspmm_run_transposed(plan, _ptr(dY), _ptr(G), int(ldy), int(ldg),
                                      _stream_handle(stream)), "bspmm_run_transposed")


def bspmm_export_transposed(plan: int, rpt_t, colids_t, values_t, stream=None) -> None:
    _check(lib().bspmm_export_transposed(plan, _ptr(rpt_t), _ptr(colids_t), _ptr(values_t),
                                         _stream_handle(stream)), "bspmm_export_transposed")


def bspmm_validate(plan: int, stream=None) -> int:
    """Returns -1 when the device CSR is well formed, else the first malformed operation."""
    bad = ctypes.c_int32(-1)
    rc = lib().bspmm_validate(plan, ctypes.byref(bad), _stream_handle(stream))
    if rc == EBADCSR:
        return int(bad.value)
    _check(rc, "bspmm_validate")
    return -1


def bspmm_kernel_info(kernel: int, dynamic_lds_bytes: int = 0) -> bspmm_kernel_resources:
    out = bspmm_kernel_resources()
    _check(lib().bspmm_kernel_info(int(kernel), int(dynamic_lds_bytes), ctypes.byref(out)),
           "bspmm_kernel_info")
    return out


def bspmm_plan_info(plan: int) -> bspmm_info:
    info = bspmm_info()
    _check(lib().bspmm_plan_info(plan, ctypes.byref(info)), "bspmm_plan_info")
    return info


def bspmm_plan_items(plan: int, transposed: bool = False):
    n = ctypes.c_int32(0)
    _check(lib().bspmm_plan_items(plan, int(bool(transposed)), None, 0, ctypes.byref(n)),
           "bspmm_plan_items")
    arr = (bspmm_item * max(n.value, 1))()
    _check(lib().bspmm_plan_items(plan, int(bool(transposed)), arr, n.value, ctypes.byref(n)),
           "bspmm_plan_items")
    return [arr[i] for i in range(n.value)]


def bspmm_destroy(plan: Optional[int]) -> None:
    if plan:
        lib().bspmm_destroy(plan)


class Plan:
    """Owns a plan handle plus the torch tensors it borrows (CSR arrays and workspace).

    ``batch`` is a :class:`workloads.Batch`-like object: the per-operation sizes and offsets are
    host arrays; the CSR arrays (``rpt``, ``colids``, ``values``) are numpy arrays, copied to
    ``device`` once, or tensors already there, borrowed in place.  Dense operands are passed per
    call as torch tensors.
    """

    def __init__(self, batch, F: Optional[int] = None, options: Optional[bspmm_options] = None,
                 device="cuda:0", stream=None, coo=None):
        import torch
        self.torch = torch
        self.F = int(F if F is not None else batch.F)
        self.device = torch.device(device)
        dev = self.device
        self.options = options
        self.rpt_len = int((np.asarray(batch.rows, dtype=np.int64) + 1).sum())
        self.rpt_t_len = int((np.asarray(batch.cols, dtype=np.int64) + 1).sum())
        self.nnz_total = int(np.asarray(batch.nnz, dtype=np.int64).sum())
        def on_device(a, dtype):
            # numpy arrays are copied over; tensors that already sit on the device with the
            # right type and layout are borrowed as they are
            if isinstance(a, torch.Tensor):
                return a.to(device=dev, dtype=dtype).contiguous()
            np_type = np.int32 if dtype == torch.int32 else np.float32
            return torch.from_numpy(np.ascontiguousarray(a, dtype=np_type)).to(dev)

        if coo is not None:
            # COO / SparseTensor operands: ``coo`` = (ids, values), numpy arrays or tensors, laid
            # out by the batch's nz_off; the batch's own CSR arrays are not used
            ids, vals = coo
            self.ids = on_device(ids, torch.int32)
            self.values = on_device(vals, torch.float32)
            self.hb = HostCooBatch(batch.rows, batch.cols, batch.nnz, batch.nz_off,
                                   batch.b_row_off, batch.c_row_off,
                                   self.ids if self.ids.numel() else None,
                                   self.values if self.values.numel() else None)
            nbytes = bspmm_workspace_bytes_coo(self.hb, self.F, options)
            self.workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
            assert self.workspace.data_ptr() % 256 == 0
            self.handle = bspmm_create_coo(self.hb, self.F, options, self.workspace, nbytes, stream)
            return
        self.rpt = on_device(batch.rpt, torch.int32)
        self.colids = on_device(batch.colids, torch.int32)
        self.values = on_device(batch.values, torch.float32)
        # zero-length tensors have a null data_ptr; give the library something addressable
        if self.rpt.numel() == 0:
            self.rpt = torch.zeros(1, dtype=torch.int32, device=dev)
        self.hb = HostBatch(batch.rows, batch.cols, batch.nnz, batch.rpt_off, batch.nz_off,
                            batch.b_row_off, batch.c_row_off, self.rpt,
                            self.colids if self.colids.numel() else None,
                            self.values if self.values.numel() else None)
        nbytes = bspmm_workspace_bytes(self.hb, self.F, options)
        self.workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
        assert self.workspace.data_ptr() % 256 == 0
        self.handle = bspmm_create(self.hb, self.F, options, self.workspace, nbytes, stream)

    def run(self, B, C, stream=None):
        bspmm_run(self.handle, B, C, _ld(B, self.F), _ld(C, self.F), stream)
        return C

    def run_gcn(self, X, W, bias, Y, accumulate: bool = False, stream=None):
        """Y (+)= A (X W + bias) in one launch (plan created with ``front_features``)."""
        bspmm_run_gcn(self.handle, X, _ld(X, X.shape[-1]), W, _ld(W, self.F), bias, Y, _ld(Y, self.F),
                      accumulate, stream)
        return Y

    def run_transposed(self, dY, G, stream=None):
        bspmm_run_transposed(self.handle, dY, G, _ld(dY, self.F), _ld(G, self.F), stream)
        return G

    def export_transposed(self, stream=None):
        t = self.torch
        rpt_t = t.empty(max(self.rpt_t_len, 1), dtype=t.int32, device=self.device)
        col_t = t.empty(max(self.nnz_total, 1), dtype=t.int32, device=self.device)
        val_t = t.empty(max(self.nnz_total, 1), dtype=t.float32, device=self.device)
        bspmm_export_transposed(self.handle, rpt_t, col_t, val_t, stream)
        return rpt_t[:self.rpt_t_len], col_t[:self.nnz_total], val_t[:self.nnz_total]

    def export_csr(self, stream=None):
        """CSR arrays a COO plan built on the device (rpt, colids, values)."""
        t = self.torch
        rpt = t.empty(max(self.rpt_len, 1), dtype=t.int32, device=self.device)
        col = t.empty(max(self.nnz_total, 1), dtype=t.int32, device=self.device)
        val = t.empty(max(self.nnz_total, 1), dtype=t.float32, device=self.device)
        bspmm_export_csr(self.handle, rpt, col, val, stream)
        return rpt[:self.rpt_len], col[:self.nnz_total], val[:self.nnz_total]

    def validate(self, stream=None) -> int:
        return bspmm_validate(self.handle, stream)

    def info(self) -> bspmm_info:
        return bspmm_plan_info(self.handle)

    def items(self, transposed: bool = False):
        return bspmm_plan_items(self.handle, transposed)

    def close(self):
        if getattr(self, "handle", None):
            bspmm_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def dry_plan(batch, F: Optional[int] = None, **option_kw) -> int:
    """Schedule-only plan (no device needed); free it with bspmm_destroy."""
    kw = dict(option_kw)
    flags = kw.pop("flags", 0) | DRY_RUN
    coo = kw.pop("coo", False)
    opts = make_options(flags=flags, **kw)
    if coo:
        hc = HostCooBatch(batch.rows, batch.cols, batch.nnz, batch.nz_off, batch.b_row_off,
                          batch.c_row_off)
        return bspmm_create_coo(hc, int(F if F is not None else batch.F), opts)
    hb = HostBatch(batch.rows, batch.cols, batch.nnz, batch.rpt_off, batch.nz_off,
                   batch.b_row_off, batch.c_row_off)
    return bspmm_create(hb, int(F if F is not None else batch.F), opts)

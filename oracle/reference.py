"""ctypes front of the CPU oracle (``bspmm_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this module; it imports nothing from the HIP package and shares no code with it.
The functions take plain numpy arrays with the batch layout of the paper's problem statement
(per-operation CSR arrays located by offsets, packed row-major dense operands; Sec. II-B,
Fig. 4, Sec. IV-C/IV-D) and return fp64 results.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bspmm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_bspmm.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        i64p = ctypes.POINTER(ctypes.c_int64)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        common = [ctypes.c_int32, i32p, i32p, i32p, i64p, i64p, i64p, i64p, i32p, i32p, f32p,
                  f32p, ctypes.c_int64, ctypes.c_int32, f64p, f64p, ctypes.c_int64]
        lib.oracle_bspmm_forward.argtypes = common
        lib.oracle_bspmm_forward.restype = ctypes.c_int
        lib.oracle_bspmm_transposed.argtypes = common
        lib.oracle_bspmm_transposed.restype = ctypes.c_int
        lib.oracle_csr_transpose.argtypes = [ctypes.c_int32, i32p, i32p, i32p, i64p, i64p,
                                             i32p, i32p, f32p, i64p, i32p, i32p, f32p, i32p]
        lib.oracle_csr_transpose.restype = ctypes.c_int
        lib.oracle_coo_product.argtypes = [ctypes.c_int32, ctypes.c_int32, i32p, i32p, i32p,
                                           i64p, i64p, i64p, i32p, f32p, f32p, ctypes.c_int64,
                                           ctypes.c_int32, f64p, f64p, ctypes.c_int64]
        lib.oracle_coo_product.restype = ctypes.c_int
        lib.oracle_coo_to_csr.argtypes = [ctypes.c_int32, i32p, i32p, i32p, i64p, i32p, f32p,
                                          i64p, i32p, i32p, f32p, i32p]
        lib.oracle_coo_to_csr.restype = ctypes.c_int
        lib.oracle_bspmm_forward_f64.argtypes = [ctypes.c_int32, i32p, i32p, i32p, i64p, i64p,
                                                 i64p, i64p, i32p, i32p, f32p, f64p,
                                                 ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                                 f64p, ctypes.c_int64]
        lib.oracle_bspmm_forward_f64.restype = ctypes.c_int
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _prep(rows, cols, nnz, rpt_off, nz_off, b_row_off, c_row_off, rpt, colids, values):
    as_ = np.ascontiguousarray
    return (as_(rows, dtype=np.int32), as_(cols, dtype=np.int32), as_(nnz, dtype=np.int32),
            as_(rpt_off, dtype=np.int64), as_(nz_off, dtype=np.int64),
            as_(b_row_off, dtype=np.int64), as_(c_row_off, dtype=np.int64),
            as_(rpt, dtype=np.int32), as_(colids, dtype=np.int32),
            as_(values, dtype=np.float32))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def forward(rows, cols, nnz, rpt_off, nz_off, b_row_off, c_row_off, rpt, colids, values,
            B: np.ndarray, n_c_rows: int, want_scale: bool = True
            ) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """C_i = A_i B_i for every operation.  Returns (C, S) in fp64, shape (n_c_rows, F);
    rows of C that belong to no operation are NaN (so an accidental read shows)."""
    lib = _load()
    a = _prep(rows, cols, nnz, rpt_off, nz_off, b_row_off, c_row_off, rpt, colids, values)
    B = np.ascontiguousarray(B, dtype=np.float32)
    F = int(B.shape[1])
    C = np.full((int(n_c_rows), F), np.nan, dtype=np.float64)
    S = np.full((int(n_c_rows), F), np.nan, dtype=np.float64) if want_scale else None
    rc = lib.oracle_bspmm_forward(
        int(a[0].shape[0]), _p(a[0], ctypes.c_int32), _p(a[1], ctypes.c_int32),
        _p(a[2], ctypes.c_int32), _p(a[3], ctypes.c_int64), _p(a[4], ctypes.c_int64),
        _p(a[5], ctypes.c_int64), _p(a[6], ctypes.c_int64), _p(a[7], ctypes.c_int32),
        _p(a[8], ctypes.c_int32), _p(a[9], ctypes.c_float), _p(B, ctypes.c_float),
        F, F, _p(C, ctypes.c_double),
        _p(S, ctypes.c_double) if S is not None else None, F)
    if rc != 0:
        raise ValueError(f"oracle: malformed operation {-rc - 1}")
    return C, S


def time_forward_call(b, calls: int, samples: int = 5):
    """Wall time of the C routine alone on a Batch-like object: arrays converted and the fp64
    output allocated once, outside the clock; one warm-up call, then ``samples`` timed runs of
    ``calls`` back-to-back calls each.  Returns the list of seconds per call, one per sample.
    (The scale S is not computed: the baseline times the product only.)"""
    import time
    lib = _load()
    a = _prep(b.rows, b.cols, b.nnz, b.rpt_off, b.nz_off, b.b_row_off, b.c_row_off, b.rpt,
              b.colids, b.values)
    B = np.ascontiguousarray(b.B, dtype=np.float32)
    F = int(B.shape[1])
    C = np.zeros((int(b.n_c_rows), F), dtype=np.float64)
    args = (int(a[0].shape[0]), _p(a[0], ctypes.c_int32), _p(a[1], ctypes.c_int32),
            _p(a[2], ctypes.c_int32), _p(a[3], ctypes.c_int64), _p(a[4], ctypes.c_int64),
            _p(a[5], ctypes.c_int64), _p(a[6], ctypes.c_int64), _p(a[7], ctypes.c_int32),
            _p(a[8], ctypes.c_int32), _p(a[9], ctypes.c_float), _p(B, ctypes.c_float),
            F, F, _p(C, ctypes.c_double), None, F)
    if lib.oracle_bspmm_forward(*args) != 0:
        raise ValueError("oracle: malformed operation")
    out = []
    for _ in range(int(samples)):
        t0 = time.perf_counter()
        for _ in range(int(calls)):
            lib.oracle_bspmm_forward(*args)
        out.append((time.perf_counter() - t0) / max(int(calls), 1))
    return out


def transposed(rows, cols, nnz, rpt_off, nz_off, b_row_off, c_row_off, rpt, colids, values,
               dY: np.ndarray, n_b_rows: int, want_scale: bool = True
               ) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """G_i = A_i^T dY_i for every operation.  dY is indexed by c_row_off (rows_i rows), the
    result by b_row_off (cols_i rows).  Returns (G, S) in fp64, shape (n_b_rows, F)."""
    lib = _load()
    a = _prep(rows, cols, nnz, rpt_off, nz_off, b_row_off, c_row_off, rpt, colids, values)
    dY = np.ascontiguousarray(dY, dtype=np.float32)
    F = int(dY.shape[1])
    G = np.full((int(n_b_rows), F), np.nan, dtype=np.float64)
    S = np.full((int(n_b_rows), F), np.nan, dtype=np.float64) if want_scale else None
    rc = lib.oracle_bspmm_transposed(
        int(a[0].shape[0]), _p(a[0], ctypes.c_int32), _p(a[1], ctypes.c_int32),
        _p(a[2], ctypes.c_int32), _p(a[3], ctypes.c_int64), _p(a[4], ctypes.c_int64),
        _p(a[5], ctypes.c_int64), _p(a[6], ctypes.c_int64), _p(a[7], ctypes.c_int32),
        _p(a[8], ctypes.c_int32), _p(a[9], ctypes.c_float), _p(dY, ctypes.c_float),
        F, F, _p(G, ctypes.c_double),
        _p(S, ctypes.c_double) if S is not None else None, F)
    if rc != 0:
        raise ValueError(f"oracle: malformed operation {-rc - 1}")
    return G, S


def csr_transpose(rows, cols, nnz, rpt_off, nz_off, rpt, colids, values):
    """Stable transposed CSR of every operation.  Returns (rpt_t_off, rpt_t, colids_t,
    values_t): op i has cols[i]+1 local row pointers at rpt_t_off[i]; its entries sit at
    nz_off[i] like the input's."""
    lib = _load()
    z = np.zeros(len(rows), dtype=np.int64)
    a = _prep(rows, cols, nnz, rpt_off, nz_off, z, z, rpt, colids, values)
    nb = int(a[0].shape[0])
    rpt_t_off = np.zeros(nb, dtype=np.int64)
    if nb:
        rpt_t_off[1:] = np.cumsum(a[1][:-1].astype(np.int64) + 1)
    total_rpt = int((a[1].astype(np.int64) + 1).sum())
    rpt_t = np.zeros(total_rpt, dtype=np.int32)
    colids_t = np.zeros(a[8].shape[0], dtype=np.int32)
    values_t = np.zeros(a[8].shape[0], dtype=np.float32)
    scratch = np.zeros(max(int(a[1].max()) if nb else 0, 1), dtype=np.int32)
    rc = lib.oracle_csr_transpose(
        nb, _p(a[0], ctypes.c_int32), _p(a[1], ctypes.c_int32), _p(a[2], ctypes.c_int32),
        _p(a[3], ctypes.c_int64), _p(a[4], ctypes.c_int64), _p(a[7], ctypes.c_int32),
        _p(a[8], ctypes.c_int32), _p(a[9], ctypes.c_float), _p(rpt_t_off, ctypes.c_int64),
        _p(rpt_t, ctypes.c_int32), _p(colids_t, ctypes.c_int32), _p(values_t, ctypes.c_float),
        _p(scratch, ctypes.c_int32))
    if rc != 0:
        raise ValueError(f"oracle: malformed operation {-rc - 1}")
    return rpt_t_off, rpt_t, colids_t, values_t


def coo_product(rows, cols, nnz, nz_off, b_row_off, c_row_off, ids, values, X: np.ndarray,
                n_out_rows: int, transposed_: bool = False, want_scale: bool = True
                ) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """Product of every COO / SparseTensor operation (Fig. 2 loop nest): Y_i = A_i X_i, or
    A_i^T X_i with ``transposed_``.  ``ids`` holds (row, column) pairs, op i at 2*nz_off[i]."""
    lib = _load()
    as_ = np.ascontiguousarray
    rows, cols, nnz = (as_(x, dtype=np.int32) for x in (rows, cols, nnz))
    nz_off, b_row_off, c_row_off = (as_(x, dtype=np.int64) for x in (nz_off, b_row_off, c_row_off))
    ids = as_(ids, dtype=np.int32)
    values = as_(values, dtype=np.float32)
    X = as_(X, dtype=np.float32)
    F = int(X.shape[1])
    Y = np.full((int(n_out_rows), F), np.nan, dtype=np.float64)
    S = np.full((int(n_out_rows), F), np.nan, dtype=np.float64) if want_scale else None
    rc = lib.oracle_coo_product(
        int(rows.shape[0]), 1 if transposed_ else 0, _p(rows, ctypes.c_int32),
        _p(cols, ctypes.c_int32), _p(nnz, ctypes.c_int32), _p(nz_off, ctypes.c_int64),
        _p(b_row_off, ctypes.c_int64), _p(c_row_off, ctypes.c_int64), _p(ids, ctypes.c_int32),
        _p(values, ctypes.c_float), _p(X, ctypes.c_float), F, F, _p(Y, ctypes.c_double),
        _p(S, ctypes.c_double) if S is not None else None, F)
    if rc != 0:
        raise ValueError(f"oracle: malformed operation {-rc - 1}")
    return Y, S


def coo_to_csr(rows, cols, nnz, nz_off, ids, values):
    """Stable CSR of every COO operation.  Returns (rpt_off, rpt, colids, csr_values): op i has
    rows[i]+1 local row pointers at rpt_off[i]; its entries sit at nz_off[i] like the input's."""
    lib = _load()
    as_ = np.ascontiguousarray
    rows, cols, nnz = (as_(x, dtype=np.int32) for x in (rows, cols, nnz))
    nz_off = as_(nz_off, dtype=np.int64)
    ids = as_(ids, dtype=np.int32)
    values = as_(values, dtype=np.float32)
    nb = int(rows.shape[0])
    rpt_off = np.zeros(nb, dtype=np.int64)
    if nb:
        rpt_off[1:] = np.cumsum(rows[:-1].astype(np.int64) + 1)
    rpt = np.zeros(int((rows.astype(np.int64) + 1).sum()), dtype=np.int32)
    colids = np.zeros(values.shape[0], dtype=np.int32)
    csr_values = np.zeros(values.shape[0], dtype=np.float32)
    scratch = np.zeros(max(int(rows.max()) if nb else 0, 1), dtype=np.int32)
    rc = lib.oracle_coo_to_csr(
        nb, _p(rows, ctypes.c_int32), _p(cols, ctypes.c_int32), _p(nnz, ctypes.c_int32),
        _p(nz_off, ctypes.c_int64), _p(ids, ctypes.c_int32), _p(values, ctypes.c_float),
        _p(rpt_off, ctypes.c_int64), _p(rpt, ctypes.c_int32), _p(colids, ctypes.c_int32),
        _p(csr_values, ctypes.c_float), _p(scratch, ctypes.c_int32))
    if rc != 0:
        raise ValueError(f"oracle: malformed operation {-rc - 1}")
    return rpt_off, rpt, colids, csr_values


def _forward_f64(a, B64: np.ndarray, C: np.ndarray, accumulate: bool) -> None:
    lib = _load()
    F = int(B64.shape[1])
    rc = lib.oracle_bspmm_forward_f64(
        int(a[0].shape[0]), _p(a[0], ctypes.c_int32), _p(a[1], ctypes.c_int32),
        _p(a[2], ctypes.c_int32), _p(a[3], ctypes.c_int64), _p(a[4], ctypes.c_int64),
        _p(a[5], ctypes.c_int64), _p(a[6], ctypes.c_int64), _p(a[7], ctypes.c_int32),
        _p(a[8], ctypes.c_int32), _p(a[9], ctypes.c_float), _p(B64, ctypes.c_double), F, F,
        1 if accumulate else 0, _p(C, ctypes.c_double), F)
    if rc != 0:
        raise ValueError(f"oracle: malformed operation {-rc - 1}")


def gcn_channel(b, X: np.ndarray, W: np.ndarray, bias: np.ndarray, Y=None, T=None):
    """One channel of the batched graph-convolution layer (Fig. 7), step by step in fp64:
    U = MatMul(Xr, W); B = Add(bias, U); C = BatchedSpMM(A_list, B).  ``X`` is the packed
    feature matrix (row block i at ``b.b_row_off[i]``, ``b.cols[i]`` rows, n_X columns), ``W`` is
    n_X x F, ``bias`` has F entries.  Returns (Y, T): with ``Y``/``T`` given the channel is added
    to them (the ElementWiseAdd over channels).  T is the tolerance scale
    sum_p |a_p| (sum_t |X[c_p][t]| |W[t][j]| + |bias[j]|)."""
    a = _prep(b.rows, b.cols, b.nnz, b.rpt_off, b.nz_off, b.b_row_off, b.c_row_off, b.rpt,
              b.colids, b.values)
    X64 = np.asarray(X, dtype=np.float32).astype(np.float64)
    W64 = np.asarray(W, dtype=np.float32).astype(np.float64)
    bias64 = np.asarray(bias, dtype=np.float32).astype(np.float64)
    U = X64 @ W64                                   # MatMul
    B = np.ascontiguousarray(U + bias64[None, :])   # Add
    Babs = np.ascontiguousarray(np.abs(X64) @ np.abs(W64) + np.abs(bias64)[None, :])
    acc = Y is not None
    if not acc:
        Y = np.full((int(b.n_c_rows), B.shape[1]), np.nan, dtype=np.float64)
        T = np.full((int(b.n_c_rows), B.shape[1]), np.nan, dtype=np.float64)
    _forward_f64(a, B, Y, acc)                      # BatchedSpMM
    absa = list(a)
    absa[9] = np.abs(a[9])
    _forward_f64(tuple(absa), Babs, T, acc)
    return Y, T


def forward_batch(b, want_scale: bool = True):
    """Convenience: forward product of a workloads.Batch-like object (duck-typed)."""
    return forward(b.rows, b.cols, b.nnz, b.rpt_off, b.nz_off, b.b_row_off, b.c_row_off,
                   b.rpt, b.colids, b.values, b.B, b.n_c_rows, want_scale)


def transposed_batch(b, want_scale: bool = True):
    """Convenience: transposed product of a Batch-like object using its ``dY``."""
    return transposed(b.rows, b.cols, b.nnz, b.rpt_off, b.nz_off, b.b_row_off, b.c_row_off,
                      b.rpt, b.colids, b.values, b.dY, b.n_b_rows, want_scale)

"""Pins of the CPU oracle against things other than itself (all CPU, no GPU).

The paper prints no worked numeric example (its format figure is an image), so the oracle is
pinned by: a hand-worked fixture, dense brute force, a library CSR product, and algebraic facts
that any correct C = A B must satisfy (Sec. II-C definition; Fig. 2/3/4 all reduce to it).
Each pin is chosen so that a plausible slip (dropped term, wrong index base, transposed
operand, missing zero-initialisation, wrong offset) breaks at least one of them.
"""
import dataclasses
import os

import numpy as np
import pytest
import scipy.sparse as sp

from paper_1903_11409_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hand_example.txt")


def _read_golden():
    out = {}
    with open(GOLD) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            out[k] = [float(x) for x in v]
    return out


def _single_op(rows, cols, rpt, colids, values, dense, n_out, oracle, transposed=False):
    z = np.zeros(1, dtype=np.int64)
    args = ([rows], [cols], [len(colids)], z, z, z, z, rpt, colids, values, dense, n_out)
    return (oracle.transposed if transposed else oracle.forward)(*args)


def _dense_of(b, i):
    """fp64 dense copy of operation i (duplicates add), built without any product."""
    rpt, ci, va = b.op_csr(i)
    A = np.zeros((int(b.rows[i]), int(b.cols[i])), dtype=np.float64)
    r = np.repeat(np.arange(int(b.rows[i])), np.diff(rpt))
    np.add.at(A, (r, ci), va.astype(np.float64))
    return A


def _brute(A, B):
    """Triple loop, pure Python: the definition with nothing clever."""
    m, k = A.shape
    n = B.shape[1]
    C = np.zeros((m, n), dtype=np.float64)
    for i in range(m):
        for j in range(n):
            s = 0.0
            for t in range(k):
                s += A[i, t] * B[t, j]
            C[i, j] = s
    return C


def test_hand_worked_example(oracle):
    g = _read_golden()
    m, n = int(g["rows"][0]), int(g["cols"][0])
    rpt = np.array(g["rpt"], dtype=np.int32)
    ci = np.array(g["colids"], dtype=np.int32)
    va = np.array(g["values"], dtype=np.float32)
    B = np.array(g["B"], dtype=np.float32).reshape(n, 2)
    C, S = _single_op(m, n, rpt, ci, va, B, m, oracle)
    assert np.array_equal(C, np.array(g["C"]).reshape(m, 2))
    assert np.array_equal(S, np.array(g["S"]).reshape(m, 2))
    Y = np.array(g["Y"], dtype=np.float32).reshape(m, 1)
    G, _ = _single_op(m, n, rpt, ci, va, Y, n, oracle, transposed=True)
    assert np.array_equal(G, np.array(g["G"]).reshape(n, 1))
    z = np.zeros(1, dtype=np.int64)
    _, rt, ct, vt = oracle.csr_transpose([m], [n], [len(ci)], z, z, rpt, ci, va)
    assert rt.tolist() == [int(x) for x in g["rpt_t"]]
    assert ct.tolist() == [int(x) for x in g["colids_t"]]
    assert vt.tolist() == g["values_t"]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_dense_brute_force_tiny(oracle, seed):
    shapes = [(5, 7, 11), (12, 12, 30), (1, 1, 1), (3, 9, 0), (9, 3, 40), (0, 4, 0), (4, 0, 0)]
    b = W.random_general(100 + seed, F=5, shapes=shapes, shuffle_blocks=True)
    C, S = oracle.forward_batch(b)
    G, SG = oracle.transposed_batch(b)
    for i in range(b.batch):
        A = _dense_of(b, i)
        Bi = b.B[int(b.b_row_off[i]):int(b.b_row_off[i]) + int(b.cols[i])].astype(np.float64)
        Yi = b.dY[int(b.c_row_off[i]):int(b.c_row_off[i]) + int(b.rows[i])].astype(np.float64)
        ref = _brute(A, Bi)
        got = C[int(b.c_row_off[i]):int(b.c_row_off[i]) + int(b.rows[i])]
        assert np.allclose(got, ref, rtol=1e-12, atol=1e-14)
        refT = _brute(A.T.copy(), Yi)
        gotT = G[int(b.b_row_off[i]):int(b.b_row_off[i]) + int(b.cols[i])]
        assert np.allclose(gotT, refT, rtol=1e-12, atol=1e-14)
    # rows of the packed output that no operation owns (the gaps) were never written
    owned = np.zeros(b.n_c_rows, dtype=bool)
    for i in range(b.batch):
        owned[int(b.c_row_off[i]):int(b.c_row_off[i]) + int(b.rows[i])] = True
    assert np.all(np.isnan(C[~owned])) and not np.any(np.isnan(C[owned]))


def test_scale_is_abs_product(oracle):
    """S = |A| |B| needs unique entries (with duplicates |a1|+|a2| != |a1+a2|)."""
    b = W.config1_tiny()
    C, S = oracle.forward_batch(b)
    for i in range(b.batch):
        A = np.abs(_dense_of(b, i))
        Bi = np.abs(b.B[int(b.b_row_off[i]):int(b.b_row_off[i]) + int(b.cols[i])].astype(np.float64))
        got = S[int(b.c_row_off[i]):int(b.c_row_off[i]) + int(b.rows[i])]
        assert np.allclose(got, A @ Bi, rtol=1e-12)
    assert np.all(np.abs(C) <= S + 1e-300)


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_library_csr_product(oracle, cfg):
    b = W.CONFIGS[cfg]() if cfg != 3 else W.config3_multichannel(graphs=64)
    C, _ = oracle.forward_batch(b)
    for i in range(b.batch):
        rpt, ci, va = b.op_csr(i)
        A = sp.csr_matrix((va.astype(np.float64), ci, rpt), shape=(int(b.rows[i]), int(b.cols[i])))
        Bi = b.B[int(b.b_row_off[i]):int(b.b_row_off[i]) + int(b.cols[i])].astype(np.float64)
        got = C[int(b.c_row_off[i]):int(b.c_row_off[i]) + int(b.rows[i])]
        assert np.allclose(got, A @ Bi, rtol=1e-12, atol=1e-15)


def test_identity_gives_B_bitwise(oracle):
    b = W.identity_batch(7, F=9, sizes=[1, 5, 33])
    C, S = oracle.forward_batch(b)
    assert np.array_equal(C, b.B.astype(np.float64))
    G, _ = oracle.transposed_batch(b)
    assert np.array_equal(G, b.dY.astype(np.float64))


def test_empty_rows_and_empty_ops(oracle):
    b = W.random_general(5, F=6, shapes=[(10, 10, 4), (6, 6, 0), (0, 0, 0), (8, 3, 2)])
    C, S = oracle.forward_batch(b)
    for i in range(b.batch):
        rpt, _, _ = b.op_csr(i)
        got = C[int(b.c_row_off[i]):int(b.c_row_off[i]) + int(b.rows[i])]
        empty = np.diff(rpt) == 0
        assert np.all(got[empty] == 0.0)
        assert np.all(S[int(b.c_row_off[i]):int(b.c_row_off[i]) + int(b.rows[i])][empty] == 0.0)
    # a batch with no operation at all is fine
    e = W.random_general(5, F=4, shapes=[])
    C0, _ = oracle.forward_batch(e)
    assert C0.shape == (0, 4)


def test_linearity_in_B(oracle):
    b = W.config2_molecule(graphs=16, F=8)
    rng = np.random.default_rng(3)
    B1 = rng.uniform(-1, 1, b.B.shape).astype(np.float32)
    B2 = rng.uniform(-1, 1, b.B.shape).astype(np.float32)
    # alpha, beta powers of two and B1 + B2 formed exactly in fp64, then the fp32 operand is
    # avoided: the oracle takes fp32, so use values whose combination is exact in fp32
    B1 = np.round(B1 * 1024) / 1024
    B2 = np.round(B2 * 1024) / 1024
    comb = (2.0 * B1 - 0.5 * B2).astype(np.float32)
    assert np.array_equal(comb.astype(np.float64), 2.0 * B1.astype(np.float64) - 0.5 * B2.astype(np.float64))
    import dataclasses
    c1, _ = oracle.forward_batch(dataclasses.replace(b, B=B1.astype(np.float32)))
    c2, _ = oracle.forward_batch(dataclasses.replace(b, B=B2.astype(np.float32)))
    c12, _ = oracle.forward_batch(dataclasses.replace(b, B=comb))
    assert np.allclose(c12, 2.0 * c1 - 0.5 * c2, rtol=1e-12, atol=1e-13)


def test_node_relabelling(oracle):
    """(P A P^T)(P B) = P (A B): relabel nodes, rebuild a sorted CSR, compare row-permuted."""
    b = W.config1_tiny()
    C, _ = oracle.forward_batch(b)
    rng = np.random.default_rng(11)
    for i in range(b.batch):
        n = int(b.rows[i])
        rpt, ci, va = b.op_csr(i)
        perm = rng.permutation(n)            # new label of old node k is perm[k]
        r = np.repeat(np.arange(n), np.diff(rpt))
        nr, nc = perm[r], perm[ci]
        order = np.lexsort((nc, nr))
        rpt2 = np.zeros(n + 1, dtype=np.int32)
        rpt2[1:] = np.cumsum(np.bincount(nr, minlength=n))
        Bi = b.B[int(b.b_row_off[i]):int(b.b_row_off[i]) + n]
        PB = np.empty_like(Bi)
        PB[perm] = Bi
        C2, _ = _single_op(n, n, rpt2, nc[order].astype(np.int32), va[order], PB, n, oracle)
        Ci = C[int(b.c_row_off[i]):int(b.c_row_off[i]) + n]
        PC = np.empty_like(Ci)
        PC[perm] = Ci
        assert np.allclose(C2, PC, rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("cfg", [1, 2, 4])
def test_symmetric_normalisation_eigenvector(oracle, cfg):
    """A^ = D^-1/2 (A+I) D^-1/2 with d = rowsum(A+I) satisfies A^ sqrt(d) = sqrt(d).
    Values are rounded to fp32, so the identity holds to a few fp32 ulps."""
    b = W.CONFIGS[cfg](F=4) if cfg != 4 else W.config4_wide(F=4, graphs=16)
    B = b.B.copy()
    sq = []
    for i in range(b.batch):
        rpt, _, _ = b.op_csr(i)
        d = np.diff(rpt).astype(np.float64)   # entries per row = degree + 1
        sq.append(np.sqrt(d))
    sq = np.concatenate(sq)
    B[:, 2] = sq.astype(np.float32)
    import dataclasses
    C, _ = oracle.forward_batch(dataclasses.replace(b, B=B))
    assert np.allclose(C[:, 2], sq, rtol=5e-7)


def test_row_normalisation_row_sums(oracle):
    """(D_ch^-1 A_ch) 1 = 1 on rows that have an edge of the channel, 0 on the others."""
    b = W.config3_multichannel(graphs=32, F=3)
    import dataclasses
    C, _ = oracle.forward_batch(dataclasses.replace(b, B=np.ones_like(b.B)))
    has = np.concatenate([np.diff(b.op_csr(i)[0]) > 0 for i in range(b.batch)])
    assert np.allclose(C[has], 1.0, rtol=1e-6)
    assert np.all(C[~has] == 0.0)
    assert 0.2 < (~has).mean() < 0.8   # the channel split really leaves many rows empty


def test_adjoint_identity_asymmetric(oracle):
    """<A B, dY> = <B, A^T dY> ties the scatter (transposed) oracle to the forward one.
    Run on asymmetric values: with symmetric A a missing transpose would go unseen."""
    b = W.config5_skewed(graphs=24, F=8, asymmetric=True)
    # the structure is symmetric but the values must not be
    A0 = _dense_of(b, 0)
    assert not np.allclose(A0, A0.T)
    C, _ = oracle.forward_batch(b)
    G, _ = oracle.transposed_batch(b)
    lhs = float((C * b.dY.astype(np.float64)).sum())
    rhs = float((b.B.astype(np.float64) * G).sum())
    assert abs(lhs - rhs) <= 1e-11 * max(abs(lhs), 1.0)
    # and per operation against the dense transpose through a library matmul
    for i in range(0, b.batch, 5):
        A = _dense_of(b, i)
        Yi = b.dY[int(b.c_row_off[i]):int(b.c_row_off[i]) + int(b.rows[i])].astype(np.float64)
        got = G[int(b.b_row_off[i]):int(b.b_row_off[i]) + int(b.cols[i])]
        assert np.allclose(got, A.T @ Yi, rtol=1e-12, atol=1e-14)
        # the forward product of the same operand is different: the pin can see a missing T
        if not np.allclose(A, A.T):
            assert not np.allclose(got, A @ Yi, rtol=1e-3)


def test_transposed_rectangular_general(oracle):
    b = W.random_general(21, F=4, shapes=[(7, 13, 25), (13, 7, 25), (20, 20, 90)])
    G, SG = oracle.transposed_batch(b)
    for i in range(b.batch):
        A = _dense_of(b, i)
        Yi = b.dY[int(b.c_row_off[i]):int(b.c_row_off[i]) + int(b.rows[i])].astype(np.float64)
        got = G[int(b.b_row_off[i]):int(b.b_row_off[i]) + int(b.cols[i])]
        assert np.allclose(got, A.T @ Yi, rtol=1e-12, atol=1e-14)


def test_csr_transpose_is_stable_counting_sort(oracle):
    """Against numpy's stable sort by column, which defines the stable transpose."""
    b = W.random_general(33, F=1, shapes=[(9, 5, 40), (5, 9, 40), (30, 30, 0), (1, 1, 1),
                                          (0, 0, 0), (17, 17, 60)], with_dY=False)
    off_t, rt, ct, vt = oracle.csr_transpose(b.rows, b.cols, b.nnz, b.rpt_off, b.nz_off,
                                             b.rpt, b.colids, b.values)
    for i in range(b.batch):
        rpt, ci, va = b.op_csr(i)
        m, n, z = int(b.rows[i]), int(b.cols[i]), int(b.nnz[i])
        r = np.repeat(np.arange(m), np.diff(rpt)).astype(np.int32)
        order = np.argsort(ci, kind="stable")
        z0 = int(b.nz_off[i])
        assert np.array_equal(ct[z0:z0 + z], r[order])
        assert np.array_equal(vt[z0:z0 + z], va[order])
        exp_rpt = np.zeros(n + 1, dtype=np.int64)
        exp_rpt[1:] = np.cumsum(np.bincount(ci, minlength=n)) if z else 0
        o = int(off_t[i])
        assert np.array_equal(rt[o:o + n + 1], exp_rpt)


def test_csr_transpose_round_trip_and_library(oracle):
    """Sorted unique input: (A^T)^T = A exactly, and A^T matches scipy's."""
    b = W.config2_molecule(graphs=12, F=1)
    b3 = W.config3_multichannel(graphs=8, F=1)
    for bb in (b, b3):
        off_t, rt, ct, vt = oracle.csr_transpose(bb.rows, bb.cols, bb.nnz, bb.rpt_off,
                                                 bb.nz_off, bb.rpt, bb.colids, bb.values)
        off2, r2, c2, v2 = oracle.csr_transpose(bb.cols, bb.rows, bb.nnz, off_t, bb.nz_off,
                                                rt, ct, vt)
        assert np.array_equal(off2, bb.rpt_off)
        assert np.array_equal(r2, bb.rpt) and np.array_equal(c2, bb.colids)
        assert np.array_equal(v2, bb.values)
        for i in range(bb.batch):
            rpt, ci, va = bb.op_csr(i)
            m, n, z = int(bb.rows[i]), int(bb.cols[i]), int(bb.nnz[i])
            T = sp.csr_matrix((va, ci, rpt), shape=(m, n)).T.tocsr()
            T.sort_indices()
            o, z0 = int(off_t[i]), int(bb.nz_off[i])
            assert np.array_equal(rt[o:o + n + 1], T.indptr)
            assert np.array_equal(ct[z0:z0 + z], T.indices)
            assert np.array_equal(vt[z0:z0 + z], T.data)


def test_oracle_rejects_malformed(oracle):
    z = np.zeros(1, dtype=np.int64)
    B = np.zeros((3, 2), dtype=np.float32)
    with pytest.raises(ValueError):   # column index out of range
        oracle.forward([2], [3], [1], z, z, z, z, np.array([0, 1, 1], np.int32),
                       np.array([3], np.int32), np.array([1.0], np.float32), B, 2)
    with pytest.raises(ValueError):   # row pointer does not end at nnz
        oracle.forward([2], [3], [2], z, z, z, z, np.array([0, 1, 1], np.int32),
                       np.array([0, 1], np.int32), np.array([1.0, 1.0], np.float32), B, 2)


def test_flop_formula():
    b = W.config1_tiny()
    assert W.flops(b) == 2 * int(b.nnz.sum()) * b.F   # 2 * nnz_A * n_B (Sec. V-A)


# ---------------------------------------------------------------------------------------------
# channel sum: operations that name one output block are added up (Fig. 6 / Fig. 7,
# "ElementWiseAdd" of the per-channel products)
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("own_inputs", [False, True])
def test_shared_output_blocks_are_summed(oracle, own_inputs):
    b = W.config3_multichannel(graphs=12, F=6, accumulate=True, own_inputs=own_inputs,
                               with_dY=True)
    C, S = oracle.forward_batch(b)
    G, SG = oracle.transposed_batch(b)
    ch = b.meta["channels"]
    refG = np.zeros((b.n_b_rows, b.F))
    for g in range(b.n_graphs):
        ops = range(g * ch, (g + 1) * ch)
        n = int(b.rows[g * ch])
        c0 = int(b.c_row_off[g * ch])
        ref = np.zeros((n, b.F))
        refS = np.zeros((n, b.F))
        Y = b.dY[c0:c0 + n].astype(np.float64)
        for i in ops:
            assert int(b.c_row_off[i]) == c0
            A = _dense_of(b, i)
            Bi = b.B[int(b.b_row_off[i]):int(b.b_row_off[i]) + n].astype(np.float64)
            ref += _brute(A, Bi)
            refS += np.abs(A) @ np.abs(Bi)
            refG[int(b.b_row_off[i]):int(b.b_row_off[i]) + n] += A.T @ Y
        assert np.allclose(C[c0:c0 + n], ref, rtol=1e-12, atol=1e-14)
        assert np.allclose(S[c0:c0 + n], refS, rtol=1e-12, atol=1e-14)
    assert np.allclose(G, refG, rtol=1e-12, atol=1e-14)
    # adjoint identity across the channel sum
    lhs = float((C * b.dY.astype(np.float64)).sum())
    rhs = float((b.B.astype(np.float64) * G).sum())
    assert abs(lhs - rhs) <= 1e-11 * max(abs(lhs), 1.0)


def test_unit_channels_sum_to_the_adjacency_matrix(oracle):
    """With entries 1.0 the channel matrices of a graph partition its edges, so the summed
    product is the plain neighbour sum: C[r] = sum of B over the neighbours of r."""
    b = W.config3_multichannel(graphs=10, F=5, accumulate=True, normalise=False)
    C, _ = oracle.forward_batch(b)
    ch = b.meta["channels"]
    for g in range(b.n_graphs):
        n = int(b.rows[g * ch])
        c0 = int(b.c_row_off[g * ch])
        b0 = int(b.b_row_off[g * ch])
        adj = np.zeros((n, n))
        for i in range(g * ch, (g + 1) * ch):
            rpt, ci, _ = b.op_csr(i)
            r = np.repeat(np.arange(n), np.diff(rpt))
            assert np.all(adj[r, ci] == 0)          # every edge belongs to exactly one channel
            adj[r, ci] = 1.0
        assert np.array_equal(adj, adj.T) and np.all(np.diag(adj) == 0)
        Bg = b.B[b0:b0 + n].astype(np.float64)
        ref = np.stack([Bg[adj[r] > 0].sum(axis=0) for r in range(n)])
        assert np.allclose(C[c0:c0 + n], ref, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------------------------------------
# COO / SparseTensor operands (Sec. II-B, Fig. 1; the loop nest of Fig. 2; unsorted, Sec. IV)
# ---------------------------------------------------------------------------------------------
def _coo_dense(b, ids, vals, i):
    """fp64 dense copy of COO operation i, assembled entry by entry (repeats add)."""
    z0, n = int(b.nz_off[i]), int(b.nnz[i])
    A = np.zeros((int(b.rows[i]), int(b.cols[i])), dtype=np.float64)
    for p in range(n):
        A[ids[2 * (z0 + p)], ids[2 * (z0 + p) + 1]] += float(vals[z0 + p])
    return A


def _coo_batches():
    return [W.random_general(51, F=5, shapes=[(7, 13, 25), (13, 7, 25), (20, 20, 90), (1, 1, 3),
                                              (0, 0, 0), (9, 9, 0)]),
            W.config2_molecule(graphs=6, F=3),
            W.config5_skewed(graphs=4, F=2)]


@pytest.mark.parametrize("which", [0, 1, 2])
@pytest.mark.parametrize("transposed", [False, True])
def test_coo_product_dense_and_library(oracle, which, transposed):
    """Against a dense matrix assembled one entry at a time, and scipy's COO product."""
    b = _coo_batches()[which]
    if b.dY is None:
        b.dY = np.random.default_rng(3).standard_normal((b.n_c_rows, b.F)).astype(np.float32)
    ids, vals = W.coo_view(b, seed=77)
    X = b.dY if transposed else b.B
    n_out = b.n_b_rows if transposed else b.n_c_rows
    Y, S = oracle.coo_product(b.rows, b.cols, b.nnz, b.nz_off, b.b_row_off, b.c_row_off, ids,
                              vals, X, n_out, transposed_=transposed)
    for i in range(b.batch):
        A = _coo_dense(b, ids, vals, i)
        z0, n = int(b.nz_off[i]), int(b.nnz[i])
        L = sp.coo_matrix((vals[z0:z0 + n].astype(np.float64),
                           (ids[2 * z0:2 * (z0 + n):2], ids[2 * z0 + 1:2 * (z0 + n):2])),
                          shape=A.shape)
        if transposed:
            A, L = A.T, L.T
            xi = X[int(b.c_row_off[i]):int(b.c_row_off[i]) + int(b.rows[i])].astype(np.float64)
            got = Y[int(b.b_row_off[i]):int(b.b_row_off[i]) + int(b.cols[i])]
            sc = S[int(b.b_row_off[i]):int(b.b_row_off[i]) + int(b.cols[i])]
        else:
            xi = X[int(b.b_row_off[i]):int(b.b_row_off[i]) + int(b.cols[i])].astype(np.float64)
            got = Y[int(b.c_row_off[i]):int(b.c_row_off[i]) + int(b.rows[i])]
            sc = S[int(b.c_row_off[i]):int(b.c_row_off[i]) + int(b.rows[i])]
        assert np.allclose(got, A @ xi, rtol=1e-12, atol=1e-14)
        assert np.allclose(got, L @ xi, rtol=1e-12, atol=1e-14)
        if A.shape[0] and A.shape[1] and not np.allclose(A, A.T if A.shape[0] == A.shape[1] else 0):
            wrong = A.T @ xi if A.shape[0] == A.shape[1] else None
            if wrong is not None:
                assert not np.allclose(got, wrong, rtol=1e-3)   # swapped indices would show
        assert np.all(sc >= np.abs(got) - 1e-12)


def test_coo_brute_force_tiny(oracle):
    """Pure-Python triple loop on a tiny operation with a repeated pair."""
    rows, cols = 3, 4
    ids = np.array([2, 1, 0, 3, 2, 1, 1, 0, 0, 0], dtype=np.int32)      # (2,1) twice
    vals = np.array([0.5, -2.0, 0.25, 3.0, 1.5], dtype=np.float32)
    Bm = np.arange(1, cols * 2 + 1, dtype=np.float32).reshape(cols, 2)
    z = np.zeros(1, dtype=np.int64)
    Y, S = oracle.coo_product([rows], [cols], [5], z, z, z, ids, vals, Bm, rows)
    A = np.zeros((rows, cols))
    A[2, 1] = 0.75; A[0, 3] = -2.0; A[1, 0] = 3.0; A[0, 0] = 1.5
    assert np.array_equal(Y, _brute(A, Bm.astype(np.float64)))
    absA = np.zeros((rows, cols))
    absA[2, 1] = 0.75; absA[0, 3] = 2.0; absA[1, 0] = 3.0; absA[0, 0] = 1.5
    assert np.array_equal(S, _brute(absA, np.abs(Bm).astype(np.float64)))
    G, _ = oracle.coo_product([rows], [cols], [5], z, z, z, ids, vals,
                              np.arange(1, rows * 2 + 1, dtype=np.float32).reshape(rows, 2), cols,
                              transposed_=True)
    assert np.array_equal(G, _brute(A.T, np.arange(1, rows * 2 + 1, dtype=np.float64).reshape(rows, 2)))


def test_coo_in_stored_order_equals_csr_oracle_bitwise(oracle):
    """A CSR batch read out entry by entry is a COO batch whose loop nest visits every output
    element's terms in the same order: the two oracles must agree to the last bit."""
    b = W.config3_multichannel(graphs=6, F=7, with_dY=True)
    ids, vals = W.coo_view(b, shuffle=False)
    C, S = oracle.forward_batch(b)
    Y, T = oracle.coo_product(b.rows, b.cols, b.nnz, b.nz_off, b.b_row_off, b.c_row_off, ids,
                              vals, b.B, b.n_c_rows)
    assert np.array_equal(C, Y, equal_nan=True) and np.array_equal(S, T, equal_nan=True)
    G, _ = oracle.transposed_batch(b)
    H, _ = oracle.coo_product(b.rows, b.cols, b.nnz, b.nz_off, b.b_row_off, b.c_row_off, ids,
                              vals, b.dY, b.n_b_rows, transposed_=True)
    assert np.array_equal(G, H, equal_nan=True)


def test_coo_entry_order_does_not_matter(oracle):
    b = W.config5_skewed(graphs=3, F=4)
    ref = None
    for seed in (1, 2, 3):
        ids, vals = W.coo_view(b, seed=seed)
        Y, _ = oracle.coo_product(b.rows, b.cols, b.nnz, b.nz_off, b.b_row_off, b.c_row_off,
                                  ids, vals, b.B, b.n_c_rows)
        if ref is None:
            ref = Y
        assert np.allclose(Y, ref, rtol=1e-13, atol=1e-15, equal_nan=True)


def test_coo_to_csr_is_stable_sort_by_row(oracle):
    """Against numpy's stable argsort of the row ids, which defines the stable conversion, and
    (unique sorted case) against scipy's conversion."""
    b = W.random_general(34, F=1, shapes=[(9, 5, 40), (5, 9, 40), (30, 30, 0), (1, 1, 1),
                                          (0, 0, 0), (17, 17, 60)], with_dY=False)
    ids, vals = W.coo_view(b, seed=5)
    off, rp, ci, va = oracle.coo_to_csr(b.rows, b.cols, b.nnz, b.nz_off, ids, vals)
    assert np.array_equal(off, b.rpt_off)
    for i in range(b.batch):
        m, z, z0 = int(b.rows[i]), int(b.nnz[i]), int(b.nz_off[i])
        r = ids[2 * z0:2 * (z0 + z):2]
        c = ids[2 * z0 + 1:2 * (z0 + z):2]
        order = np.argsort(r, kind="stable")
        assert np.array_equal(ci[z0:z0 + z], c[order])
        assert np.array_equal(va[z0:z0 + z], vals[z0:z0 + z][order])
        exp = np.zeros(m + 1, dtype=np.int64)
        exp[1:] = np.cumsum(np.bincount(r, minlength=m)) if z else 0
        o = int(off[i])
        assert np.array_equal(rp[o:o + m + 1], exp)
    # unique entries: the row pointers and the per-row entry SETS are scipy's
    b2 = W.config2_molecule(graphs=5, F=1)
    ids2, vals2 = W.coo_view(b2, seed=9)
    off2, rp2, ci2, va2 = oracle.coo_to_csr(b2.rows, b2.cols, b2.nnz, b2.nz_off, ids2, vals2)
    for i in range(b2.batch):
        m, n, z, z0 = int(b2.rows[i]), int(b2.cols[i]), int(b2.nnz[i]), int(b2.nz_off[i])
        L = sp.coo_matrix((vals2[z0:z0 + z], (ids2[2 * z0:2 * (z0 + z):2],
                                              ids2[2 * z0 + 1:2 * (z0 + z):2])), shape=(m, n)).tocsr()
        L.sort_indices()
        o = int(off2[i])
        mine = sp.csr_matrix((va2[z0:z0 + z], ci2[z0:z0 + z], rp2[o:o + m + 1]), shape=(m, n))
        mine.sort_indices()
        assert np.array_equal(mine.indptr, L.indptr)
        assert np.array_equal(mine.indices, L.indices) and np.array_equal(mine.data, L.data)
        # and sorting the shuffled view by column inside rows gives back the batch's CSR
        rpt, cc, vv = b2.op_csr(i)
        assert np.array_equal(mine.indptr, rpt) and np.array_equal(mine.indices, cc)
        assert np.array_equal(mine.data, vv)


def test_coo_rejects_out_of_range(oracle):
    z = np.zeros(1, dtype=np.int64)
    Bm = np.zeros((3, 2), dtype=np.float32)
    for bad in ([3, 0], [0, 3], [-1, 0], [0, -1]):
        with pytest.raises(ValueError):
            oracle.coo_product([3], [3], [1], z, z, z, np.array(bad, dtype=np.int32),
                               np.ones(1, dtype=np.float32), Bm, 3)
        with pytest.raises(ValueError):
            oracle.coo_to_csr([3], [3], [1], z, np.array(bad, dtype=np.int32),
                              np.ones(1, dtype=np.float32))


# ---------------------------------------------------------------------------------------------
# one channel of the batched graph-convolution layer (Fig. 7): MatMul, Add, BatchedSpMM
# ---------------------------------------------------------------------------------------------
def _layer_inputs(b, n_x, seed, integer=False):
    rng = np.random.default_rng(seed)
    if integer:   # small integers: every intermediate is exact in fp32 and fp64 alike
        X = rng.integers(-3, 4, size=(b.n_b_rows, n_x)).astype(np.float32)
        W = rng.integers(-2, 3, size=(n_x, b.F)).astype(np.float32)
        bias = rng.integers(-2, 3, size=b.F).astype(np.float32)
    else:
        X = rng.uniform(-1, 1, size=(b.n_b_rows, n_x)).astype(np.float32)
        W = rng.uniform(-1, 1, size=(n_x, b.F)).astype(np.float32)
        bias = rng.uniform(-1, 1, size=b.F).astype(np.float32)
    return X, W, bias


@pytest.mark.parametrize("which", [0, 1])
def test_gcn_channel_against_dense_algebra(oracle, which):
    b = [W.config2_molecule(graphs=5, F=6), W.random_general(61, F=5, shapes=[(7, 13, 25), (13, 7, 25),
                                                                              (4, 4, 0), (0, 0, 0)])][which]
    X, Wt, bias = _layer_inputs(b, 9, 3)
    Y, T = oracle.gcn_channel(b, X, Wt, bias)
    for i in range(b.batch):
        A = _dense_of(b, i)
        xi = X[int(b.b_row_off[i]):int(b.b_row_off[i]) + int(b.cols[i])].astype(np.float64)
        # every product of the expected value is the pure-Python triple loop: the oracle's
        # MatMul step is a library routine, and calling that routine again would pin nothing
        W64, bias64 = Wt.astype(np.float64), bias.astype(np.float64)
        want = _brute(A, _brute(xi, W64) + bias64)
        got = Y[int(b.c_row_off[i]):int(b.c_row_off[i]) + int(b.rows[i])]
        assert np.allclose(got, want, rtol=1e-12, atol=1e-13)
        # a transposed weight matrix, a dropped bias or a bias added after the SpMM would show
        assert not np.allclose(got, _brute(A, _brute(xi, W64)), rtol=1e-3) or A.size == 0 or not A.any()
        # scale: every stored entry counts with its absolute value (repeated pairs do not cancel)
        absA = _dense_of(dataclasses.replace(b, values=np.abs(b.values)), i)
        want_T = _brute(absA, _brute(np.abs(xi), np.abs(W64)) + np.abs(bias64))
        assert np.allclose(T[int(b.c_row_off[i]):int(b.c_row_off[i]) + int(b.rows[i])], want_T,
                           rtol=1e-12, atol=1e-13)


def test_gcn_channel_bias_goes_through_the_adjacency(oracle):
    """W = 0: every output row is (row sum of A) * bias, not bias itself."""
    b = W.config5_skewed(graphs=3, F=4, asymmetric=True)
    X, Wt, bias = _layer_inputs(b, 5, 4)
    Y, _ = oracle.gcn_channel(b, X, np.zeros_like(Wt), bias)
    for i in range(b.batch):
        rs = _dense_of(b, i).sum(axis=1)
        got = Y[int(b.c_row_off[i]):int(b.c_row_off[i]) + int(b.rows[i])]
        assert np.allclose(got, rs[:, None] * bias[None, :].astype(np.float64), rtol=1e-12)


def test_gcn_channel_identity_weights_reduce_to_the_plain_product(oracle):
    """W = I, bias = 0: the layer is C = A X, bit for bit the forward oracle."""
    b = W.config2_molecule(graphs=6, F=8)
    Y, _ = oracle.gcn_channel(b, b.B, np.eye(8, dtype=np.float32), np.zeros(8, dtype=np.float32))
    C, _ = oracle.forward_batch(b)
    assert np.array_equal(Y, C, equal_nan=True)


def test_gcn_channel_exact_integers_equal_the_three_step_pipeline(oracle):
    """Integer-valued inputs: B = XW + bias is exact in fp32, so feeding it to the forward
    oracle as an fp32 matrix gives the same bits as the fp64 pipeline."""
    b = W.config3_multichannel(graphs=5, F=6, normalise=False)
    X, Wt, bias = _layer_inputs(b, 7, 8, integer=True)
    Y, _ = oracle.gcn_channel(b, X, Wt, bias)
    B32 = (X @ Wt + bias[None, :]).astype(np.float32)
    C, _ = oracle.forward(b.rows, b.cols, b.nnz, b.rpt_off, b.nz_off, b.b_row_off, b.c_row_off,
                          b.rpt, b.colids, b.values, B32, b.n_c_rows)
    assert np.array_equal(Y, C, equal_nan=True)


def test_gcn_channels_accumulate_like_the_layer(oracle):
    """Y = sum over channels of A_ch (X W_ch + bias_ch) (Fig. 7 last line), channel by channel."""
    chans = 3
    # the same graphs in every channel, with channel-specific edge weights
    bs = [W.config2_molecule(seed=70, graphs=4, F=5) for _ in range(chans)]
    rng = np.random.default_rng(5)
    for c, bb in enumerate(bs):
        bb.values = (bb.values * rng.uniform(0.5, 1.5, size=bb.values.shape)).astype(np.float32)
    X = rng.uniform(-1, 1, size=(bs[0].n_b_rows, 6)).astype(np.float32)
    Ws = [rng.uniform(-1, 1, size=(6, 5)).astype(np.float32) for _ in range(chans)]
    biases = [rng.uniform(-1, 1, size=5).astype(np.float32) for _ in range(chans)]
    Y = T = None
    for c in range(chans):
        Y, T = oracle.gcn_channel(bs[c], X, Ws[c], biases[c], Y, T)
    b0 = bs[0]
    for i in range(b0.batch):
        xi = X[int(b0.b_row_off[i]):int(b0.b_row_off[i]) + int(b0.cols[i])].astype(np.float64)
        want = sum(_brute(_dense_of(bs[c], i),
                          _brute(xi, Ws[c].astype(np.float64)) + biases[c].astype(np.float64))
                   for c in range(chans))
        got = Y[int(b0.c_row_off[i]):int(b0.c_row_off[i]) + int(b0.rows[i])]
        assert np.allclose(got, want, rtol=1e-12, atol=1e-13)

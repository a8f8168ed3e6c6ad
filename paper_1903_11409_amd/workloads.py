"""Seeded synthetic batches for Batched SpMM (inputs only, none of the method's arithmetic).

A *batch* is a list of independent SpMM operations ``C_i = A_i . B_i`` (paper Sec. IV-C): every
``A_i`` is a small CSR matrix (row pointer / column index / value arrays, Sec. II-B), every
``B_i`` is a row slice of one packed row-major dense matrix whose column count ``F`` (the
paper's ``n_B``) is the same for the whole batch (Sec. IV; packed layout as in the reshaped
input of Sec. IV-D).

The paper evaluates on Tox21 / Reaction100 molecule graphs (Table 1: at most 50 nodes, batch
50-200, n_B 64/512) and on random square matrices (Sec. V-A: dim 32-256, nnz/row 1-5).  Neither
dataset is available here; the generators below are seeded stand-ins with those shapes and
sparsities.  No dataset item is reproduced.

Only numpy is used.  Everything is deterministic given ``seed``.  Both the CPU oracle's tests
and the GPU tests/bench draw their inputs from here; nothing in this module multiplies a sparse
matrix by a dense one.
"""
from __future__ import annotations

import dataclasses
import hashlib
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 190311409


def config_seed(config: int, rep: int = 0) -> int:
    """Seed convention shared by tests and bench: base + 1000*config + rep."""
    return BASE_SEED + 1000 * int(config) + int(rep)


@dataclasses.dataclass
class Batch:
    """Host-side description of one batch of SpMM operations (all numpy, C-contiguous).

    ``rpt`` holds the per-operation row-pointer arrays back to back; operation ``i`` owns
    ``rows[i]+1`` entries starting at ``rpt_off[i]`` and they are *local* (first entry 0, last
    entry ``nnz[i]``).  ``colids``/``values`` hold the non-zeros back to back; operation ``i``
    owns ``nnz[i]`` entries starting at ``nz_off[i]``.  ``B`` is the packed dense input
    (``n_b_rows x F``, leading dimension ``F``); operation ``i`` reads rows
    ``b_row_off[i] .. b_row_off[i]+cols[i]``.  The output is a packed ``n_c_rows x F`` matrix;
    operation ``i`` writes rows ``c_row_off[i] .. c_row_off[i]+rows[i]``.
    """

    name: str
    F: int
    rows: np.ndarray       # int32 [batch]
    cols: np.ndarray       # int32 [batch]
    nnz: np.ndarray        # int32 [batch]
    rpt_off: np.ndarray    # int64 [batch]
    nz_off: np.ndarray     # int64 [batch]
    b_row_off: np.ndarray  # int64 [batch]
    c_row_off: np.ndarray  # int64 [batch]
    rpt: np.ndarray        # int32 [sum(rows+1)]
    colids: np.ndarray     # int32 [sum(nnz)]
    values: np.ndarray     # float32 [sum(nnz)]
    B: np.ndarray          # float32 [n_b_rows, F]
    n_b_rows: int
    n_c_rows: int
    dY: Optional[np.ndarray] = None  # float32 [n_c_rows, F] upstream gradient (training configs)
    n_graphs: int = 0                # number of graphs (ops / channels)
    meta: Dict[str, object] = dataclasses.field(default_factory=dict)

    @property
    def batch(self) -> int:
        return int(self.rows.shape[0])

    def op_csr(self, i: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        """(rpt, colids, values) views of operation ``i``."""
        r0 = int(self.rpt_off[i])
        z0 = int(self.nz_off[i])
        return (self.rpt[r0:r0 + int(self.rows[i]) + 1],
                self.colids[z0:z0 + int(self.nnz[i])],
                self.values[z0:z0 + int(self.nnz[i])])

    def checksum(self) -> str:
        h = hashlib.sha256()
        for a in (self.rows, self.cols, self.nnz, self.rpt_off, self.nz_off, self.b_row_off,
                  self.c_row_off, self.rpt, self.colids, self.values, self.B):
            h.update(np.ascontiguousarray(a).tobytes())
        if self.dY is not None:
            h.update(np.ascontiguousarray(self.dY).tobytes())
        return h.hexdigest()[:16]

    def single(self, i: int) -> "Batch":
        """Operation ``i`` alone, as a batch of one that still reads and writes its rows of the
        packed dense matrices (the non-batched route of Sec. V-A: one launch per matrix)."""
        rpt, ci, va = self.op_csr(i)
        z = np.zeros(1, dtype=np.int64)
        return dataclasses.replace(
            self, name=f"{self.name}[{i}]", rows=self.rows[i:i + 1], cols=self.cols[i:i + 1],
            nnz=self.nnz[i:i + 1], rpt_off=z, nz_off=z.copy(), b_row_off=self.b_row_off[i:i + 1],
            c_row_off=self.c_row_off[i:i + 1], rpt=rpt, colids=ci, values=va, n_graphs=1)

    def subset(self, ops: Sequence[int], name: Optional[str] = None) -> "Batch":
        """The operations ``ops`` alone, repacked: CSR arrays, dense input rows and output rows
        back to back in the order given (operations that read one dense block keep sharing
        it only if it is listed once: every operation gets a block of its own here)."""
        ops = np.asarray(list(ops), dtype=np.int64)
        rows, cols, nnz = self.rows[ops], self.cols[ops], self.nnz[ops]
        parts = [self.op_csr(int(i)) for i in ops]

        def cat(j, dtype):
            return (np.concatenate([p[j] for p in parts]).astype(dtype) if len(parts)
                    else np.zeros(0, dtype=dtype))

        def starts(lengths):
            out = np.zeros(len(lengths), dtype=np.int64)
            if len(lengths) > 1:
                out[1:] = np.cumsum(np.asarray(lengths[:-1], dtype=np.int64))
            return out

        b_off, c_off = starts(cols), starts(rows)
        B = (np.concatenate([self.B[int(self.b_row_off[i]):int(self.b_row_off[i]) + int(self.cols[i])]
                             for i in ops]) if len(ops) else np.zeros((0, self.F), np.float32))
        dY = None
        if self.dY is not None:
            dY = (np.concatenate([self.dY[int(self.c_row_off[i]):int(self.c_row_off[i]) + int(self.rows[i])]
                                  for i in ops]) if len(ops) else np.zeros((0, self.F), np.float32))
        return dataclasses.replace(
            self, name=name or f"{self.name}[{len(ops)} ops]", rows=rows, cols=cols, nnz=nnz,
            rpt_off=starts(rows.astype(np.int64) + 1), nz_off=starts(nnz), b_row_off=b_off,
            c_row_off=c_off, rpt=cat(0, np.int32), colids=cat(1, np.int32), values=cat(2, np.float32),
            B=np.ascontiguousarray(B), dY=None if dY is None else np.ascontiguousarray(dY),
            n_b_rows=int(cols.sum()), n_c_rows=int(rows.sum()), n_graphs=int(len(ops)))

    def with_F(self, F: int, seed: int) -> "Batch":
        """Same sparse structure, fresh dense input of width ``F``."""
        rng = np.random.default_rng(seed)
        B = rng.uniform(-1.0, 1.0, size=(self.n_b_rows, F)).astype(np.float32)
        dY = None
        if self.dY is not None:
            dY = rng.standard_normal(size=(self.n_c_rows, F)).astype(np.float32)
        return dataclasses.replace(self, F=int(F), B=B, dY=dY)


# --------------------------------------------------------------------------------------------
# graph structure generators (undirected edge lists, no self-loops, no duplicates)
# --------------------------------------------------------------------------------------------

def _gnm_edges(rng: np.random.Generator, n: int, m: int) -> np.ndarray:
    """``m`` distinct undirected pairs (u<v) drawn uniformly: the G(n,m) model."""
    total = n * (n - 1) // 2
    m = int(min(max(m, 0), total))
    if m == 0:
        return np.zeros((0, 2), dtype=np.int64)
    picks = rng.choice(total, size=m, replace=False)
    # unrank pair index k -> (u, v), u < v, pairs ordered by u then v
    u = np.zeros(m, dtype=np.int64)
    rem = picks.astype(np.int64)
    # row u starts at offset u*n - u*(u+1)/2 ; solve by searchsorted on the starts
    starts = np.array([uu * n - uu * (uu + 1) // 2 for uu in range(n)], dtype=np.int64)
    u = np.searchsorted(starts, rem, side="right") - 1
    v = rem - starts[u] + u + 1
    return np.stack([u, v], axis=1)


def _molecule_edges(rng: np.random.Generator, n: int, avg_degree: float,
                    max_degree: int = 6) -> np.ndarray:
    """Connected sparse graph: random recursive spanning tree + extra edges, degree capped.

    Every new node attaches to a uniformly chosen earlier node whose degree is still below
    ``max_degree``; then extra edges are added (duplicates and saturated endpoints rejected)
    until the average degree reaches ``avg_degree`` or no candidate is found.
    """
    deg = np.zeros(n, dtype=np.int64)
    edges = set()
    for v in range(1, n):
        cand = np.flatnonzero(deg[:v] < max_degree)
        u = int(cand[rng.integers(0, cand.size)])
        edges.add((u, v))
        deg[u] += 1
        deg[v] += 1
    target = int(round(avg_degree * n / 2.0))
    limit = min(target, n * (n - 1) // 2, (n * max_degree) // 2)
    tries = 0
    while len(edges) < limit and tries < 50 * n + 100:
        tries += 1
        u = int(rng.integers(0, n))
        v = int(rng.integers(0, n))
        if u == v:
            continue
        if u > v:
            u, v = v, u
        if (u, v) in edges or deg[u] >= max_degree or deg[v] >= max_degree:
            continue
        edges.add((u, v))
        deg[u] += 1
        deg[v] += 1
    if not edges:
        return np.zeros((0, 2), dtype=np.int64)
    return np.array(sorted(edges), dtype=np.int64)


# --------------------------------------------------------------------------------------------
# edge list -> CSR with values (input normalisation; values computed in fp64, stored fp32)
# --------------------------------------------------------------------------------------------

def _csr_from_directed(n_rows: int, r: np.ndarray, c: np.ndarray,
                       v: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Sort directed entries by (row, col) and build a local row-pointer array."""
    order = np.lexsort((c, r))
    r, c, v = r[order], c[order], v[order]
    counts = np.bincount(r, minlength=n_rows) if r.size else np.zeros(n_rows, dtype=np.int64)
    rpt = np.zeros(n_rows + 1, dtype=np.int32)
    rpt[1:] = np.cumsum(counts)
    return rpt, c.astype(np.int32), v.astype(np.float32)


def sym_normalised_csr(n: int, edges: np.ndarray):
    """D^-1/2 (A+I) D^-1/2 with d = degree + 1, both edge directions stored, sorted columns."""
    u, v = edges[:, 0], edges[:, 1]
    loops = np.arange(n, dtype=np.int64)
    r = np.concatenate([u, v, loops])
    c = np.concatenate([v, u, loops])
    d = np.bincount(r, minlength=n).astype(np.float64)  # degree + 1 (self-loop counted once)
    val = 1.0 / np.sqrt(d[r] * d[c])
    return _csr_from_directed(n, r, c, val)


def row_normalised_csr(n: int, edges: np.ndarray, self_loops: bool):
    """D^-1 A (optionally A+I): each stored entry of row r is 1/(number of entries in row r)."""
    u, v = edges[:, 0], edges[:, 1]
    if self_loops:
        loops = np.arange(n, dtype=np.int64)
        r = np.concatenate([u, v, loops])
        c = np.concatenate([v, u, loops])
    else:
        r = np.concatenate([u, v])
        c = np.concatenate([v, u])
    d = np.bincount(r, minlength=n).astype(np.float64)
    val = 1.0 / d[r] if r.size else np.zeros(0)
    return _csr_from_directed(n, r, c, val)


# --------------------------------------------------------------------------------------------
# batch assembly
# --------------------------------------------------------------------------------------------

def assemble(name: str, F: int, ops: Sequence[Tuple[int, int, np.ndarray, np.ndarray, np.ndarray]],
             b_block_of_op: Sequence[int], b_block_rows: Sequence[int],
             rng: np.random.Generator, with_dY: bool = False, n_graphs: Optional[int] = None,
             meta: Optional[dict] = None, c_block_of_op: Optional[Sequence[int]] = None) -> Batch:
    """Pack operations ``(rows, cols, rpt, colids, values)`` into one :class:`Batch`.

    ``b_block_of_op[i]`` names the dense-input block operation ``i`` reads (several operations
    may name the same block); ``b_block_rows[k]`` is the row count of block ``k``.  Output
    blocks are laid out back to back in operation order, unless ``c_block_of_op`` names an
    output block per operation (operations naming the same block are summed into it).
    """
    nb = len(ops)
    rows = np.array([o[0] for o in ops], dtype=np.int32).reshape(nb)
    cols = np.array([o[1] for o in ops], dtype=np.int32).reshape(nb)
    nnz = np.array([o[3].shape[0] for o in ops], dtype=np.int32).reshape(nb)
    rpt_off = np.zeros(nb, dtype=np.int64)
    nz_off = np.zeros(nb, dtype=np.int64)
    c_row_off = np.zeros(nb, dtype=np.int64)
    if nb:
        rpt_off[1:] = np.cumsum(rows[:-1].astype(np.int64) + 1)
        nz_off[1:] = np.cumsum(nnz[:-1].astype(np.int64))
        c_row_off[1:] = np.cumsum(rows[:-1].astype(np.int64))
    n_c_rows = int(rows.astype(np.int64).sum())
    if c_block_of_op is not None:
        nblk = (max(c_block_of_op) + 1) if nb else 0
        blk_rows = np.zeros(nblk, dtype=np.int64)
        for i in range(nb):
            assert blk_rows[c_block_of_op[i]] in (0, int(rows[i]))
            blk_rows[c_block_of_op[i]] = int(rows[i])
        cstart = np.zeros(nblk + 1, dtype=np.int64)
        cstart[1:] = np.cumsum(blk_rows)
        c_row_off = np.array([cstart[k] for k in c_block_of_op], dtype=np.int64).reshape(nb)
        n_c_rows = int(cstart[-1])
    blk_start = np.zeros(len(b_block_rows) + 1, dtype=np.int64)
    blk_start[1:] = np.cumsum(np.asarray(b_block_rows, dtype=np.int64))
    b_row_off = np.array([blk_start[k] for k in b_block_of_op], dtype=np.int64).reshape(nb)
    for i in range(nb):
        assert int(b_block_rows[b_block_of_op[i]]) == int(cols[i])
    rpt = (np.concatenate([o[2] for o in ops]).astype(np.int32) if nb
           else np.zeros(0, dtype=np.int32))
    colids = (np.concatenate([o[3] for o in ops]).astype(np.int32) if nb
              else np.zeros(0, dtype=np.int32))
    values = (np.concatenate([o[4] for o in ops]).astype(np.float32) if nb
              else np.zeros(0, dtype=np.float32))
    n_b_rows = int(blk_start[-1])
    B = rng.uniform(-1.0, 1.0, size=(n_b_rows, F)).astype(np.float32)
    dY = rng.standard_normal(size=(n_c_rows, F)).astype(np.float32) if with_dY else None
    return Batch(name=name, F=int(F), rows=rows, cols=cols, nnz=nnz, rpt_off=rpt_off,
                 nz_off=nz_off, b_row_off=b_row_off, c_row_off=c_row_off, rpt=rpt,
                 colids=colids, values=values, B=B, n_b_rows=n_b_rows, n_c_rows=n_c_rows,
                 dY=dY, n_graphs=int(n_graphs if n_graphs is not None else nb),
                 meta=dict(meta or {}))


def _lognormal_sizes(rng, count, mean=None, median=None, sigma=0.5, lo=3, hi=132):
    if mean is not None:
        mu = np.log(mean) - 0.5 * sigma * sigma
    else:
        mu = np.log(median)
    n = np.rint(rng.lognormal(mean=mu, sigma=sigma, size=count))
    return np.clip(n, lo, hi).astype(np.int64)


# --------------------------------------------------------------------------------------------
# the five workload configurations
# --------------------------------------------------------------------------------------------

def config1_tiny(seed: Optional[int] = None, F: int = 64) -> Batch:
    """8 graphs, n ~ U{10..50}, G(n, round(1.5 n)) + self-loops, symmetric normalisation."""
    rng = np.random.default_rng(config_seed(1) if seed is None else seed)
    ops, blocks = [], []
    for _ in range(8):
        n = int(rng.integers(10, 51))
        e = _gnm_edges(rng, n, int(round(1.5 * n)))
        ops.append((n, n) + sym_normalised_csr(n, e))
        blocks.append(n)
    return assemble("cfg1_tiny", F, ops, list(range(len(ops))), blocks, rng)


def config2_molecule(seed: Optional[int] = None, F: int = 128, graphs: int = 128) -> Batch:
    """Molecule-like graphs: log-normal sizes (mean ~25, clip [3,132]), tree + extras, deg<=6."""
    rng = np.random.default_rng(config_seed(2) if seed is None else seed)
    sizes = _lognormal_sizes(rng, graphs, mean=25.0, sigma=0.5, lo=3, hi=132)
    ops, blocks = [], []
    for n in sizes:
        n = int(n)
        e = _molecule_edges(rng, n, float(rng.uniform(2.0, 4.0)), max_degree=6)
        ops.append((n, n) + sym_normalised_csr(n, e))
        blocks.append(n)
    return assemble("cfg2_molecule", F, ops, list(range(len(ops))), blocks, rng)


def config3_multichannel(seed: Optional[int] = None, F: int = 128, graphs: int = 512,
                         channels: int = 4, accumulate: bool = False, own_inputs: bool = False,
                         normalise: bool = True, with_dY: bool = False) -> Batch:
    """Each graph's edges are split at random into ``channels`` edge types.

    Every channel gives one CSR matrix without self-loops, row-normalised by its channel degree
    (rows without an edge of that type stay empty).  The ``channels`` operations of one graph
    read the same dense block; each writes its own output block.  Operation index =
    ``graph * channels + channel``.

    Variants for the layer's channel sum (Fig. 6 / Fig. 7 of the paper): ``accumulate`` makes the
    channels of a graph name ONE output block (their products are added), ``own_inputs`` gives
    every channel its own dense block (the paper's ``B = X W[ch] + bias[ch]``),
    ``normalise=False`` keeps the entries at 1.0 (the channel matrices then add up to the plain
    adjacency matrix).
    """
    rng = np.random.default_rng(config_seed(3) if seed is None else seed)
    sizes = _lognormal_sizes(rng, graphs, mean=25.0, sigma=0.5, lo=3, hi=150)
    ops, block_of_op, blocks, c_block_of_op = [], [], [], []
    for g, n in enumerate(sizes):
        n = int(n)
        e = _molecule_edges(rng, n, float(rng.uniform(2.0, 4.0)), max_degree=6)
        ch = rng.integers(0, channels, size=e.shape[0])
        for k in range(channels):
            rpt, ci, va = row_normalised_csr(n, e[ch == k], self_loops=False)
            if not normalise:
                va = np.ones_like(va)
            ops.append((n, n, rpt, ci, va))
            block_of_op.append(g * channels + k if own_inputs else g)
            c_block_of_op.append(g)
        blocks.extend([n] * (channels if own_inputs else 1))
    name = "cfg3_multichannel" + ("_acc" if accumulate else "") + ("_own" if own_inputs else "")
    return assemble(name, F, ops, block_of_op, blocks, rng, n_graphs=graphs,
                    meta={"channels": channels}, with_dY=with_dY,
                    c_block_of_op=c_block_of_op if accumulate else None)


def config4_wide(seed: Optional[int] = None, F: int = 1024, graphs: int = 128) -> Batch:
    """n ~ U{20..100}, G(n, 2n) (average degree 4) + self-loops, symmetric normalisation."""
    rng = np.random.default_rng(config_seed(4) if seed is None else seed)
    ops, blocks = [], []
    for _ in range(graphs):
        n = int(rng.integers(20, 101))
        e = _gnm_edges(rng, n, 2 * n)
        ops.append((n, n) + sym_normalised_csr(n, e))
        blocks.append(n)
    return assemble("cfg4_wide", F, ops, list(range(len(ops))), blocks, rng)


def config5_skewed(seed: Optional[int] = None, F: int = 256, graphs: int = 1024,
                   asymmetric: bool = False) -> Batch:
    """Heavy-tailed sizes (log-normal, median 40, sigma 0.9, clip [8,500]), degree U[3,8].

    ``asymmetric=True`` keeps the structure and replaces the symmetric normalisation by
    ``1/d_r`` (row normalisation with self-loops) so that A differs from its transpose: a
    missing transpose in the backward product is invisible with symmetric values.
    Carries an upstream gradient ``dY`` ~ N(0,1).
    """
    rng = np.random.default_rng(config_seed(5) if seed is None else seed)
    sizes = _lognormal_sizes(rng, graphs, median=40.0, sigma=0.9, lo=8, hi=500)
    ops, blocks = [], []
    for n in sizes:
        n = int(n)
        m = int(round(float(rng.uniform(3.0, 8.0)) * n / 2.0))
        e = _gnm_edges(rng, n, m)
        if asymmetric:
            ops.append((n, n) + row_normalised_csr(n, e, self_loops=True))
        else:
            ops.append((n, n) + sym_normalised_csr(n, e))
        blocks.append(n)
    return assemble("cfg5_skewed" + ("_asym" if asymmetric else ""), F, ops,
                    list(range(len(ops))), blocks, rng, with_dY=True)


CONFIGS = {
    1: config1_tiny,
    2: config2_molecule,
    3: config3_multichannel,
    4: config4_wide,
    5: config5_skewed,
}


# --------------------------------------------------------------------------------------------
# adversarial / edge-case batches for parity tests
# --------------------------------------------------------------------------------------------

def random_general(seed: int, F: int, shapes: Sequence[Tuple[int, int, int]],
                   sort_columns: bool = False, with_dY: bool = True,
                   shuffle_blocks: bool = False) -> Batch:
    """Rectangular operations ``(rows, cols, nnz)`` with random, unsorted, possibly duplicate
    entries, signed values in [-1,1); many rows end up empty when nnz is small.

    ``shuffle_blocks`` lays the output blocks out in a random order with gaps so that offsets
    are not monotone in the operation index.
    """
    rng = np.random.default_rng(seed)
    ops, blocks = [], []
    for (m, n, z) in shapes:
        if m == 0 or n == 0:
            z = 0
        r = rng.integers(0, max(m, 1), size=z)
        c = rng.integers(0, max(n, 1), size=z)
        v = rng.uniform(-1.0, 1.0, size=z)
        order = np.lexsort((c, r)) if sort_columns else np.argsort(r, kind="stable")
        r, c, v = r[order], c[order], v[order]
        counts = np.bincount(r, minlength=m) if z else np.zeros(m, dtype=np.int64)
        rpt = np.zeros(m + 1, dtype=np.int32)
        rpt[1:] = np.cumsum(counts)
        ops.append((m, n, rpt, c.astype(np.int32), v.astype(np.float32)))
        blocks.append(n)
    b = assemble("general", F, ops, list(range(len(ops))), blocks, rng, with_dY=with_dY)
    if shuffle_blocks and b.batch > 1:
        perm = rng.permutation(b.batch)
        gap = 3
        off = np.zeros(b.batch, dtype=np.int64)
        cur = 0
        for i in perm:
            off[i] = cur
            cur += int(b.rows[i]) + gap
        b.c_row_off = off
        b.n_c_rows = int(cur)
        if with_dY:
            b.dY = rng.standard_normal(size=(b.n_c_rows, F)).astype(np.float32)
    return b


def random_square(seed: int, F: int, batch: int, dim, nnz_per_row) -> Batch:
    """The paper's preliminary workload (Sec. V-A): ``batch`` random square matrices, every
    row holding ``nnz_per_row`` entries at distinct random columns (sorted), values U[-1,1).
    ``dim`` and ``nnz_per_row`` are ints, or (lo, hi) pairs drawn per matrix for the mixed
    batch of the last preliminary experiment."""
    rng = np.random.default_rng(seed)
    ops, blocks = [], []
    for _ in range(batch):
        n = int(dim if np.isscalar(dim) else rng.integers(dim[0], dim[1] + 1))
        z = int(nnz_per_row if np.isscalar(nnz_per_row)
                else rng.integers(nnz_per_row[0], nnz_per_row[1] + 1))
        z = min(z, n)
        cols = np.stack([np.sort(rng.choice(n, size=z, replace=False)) for _ in range(n)])
        rpt = (np.arange(n + 1) * z).astype(np.int32)
        vals = rng.uniform(-1.0, 1.0, size=n * z).astype(np.float32)
        ops.append((n, n, rpt, cols.reshape(-1).astype(np.int32), vals))
        blocks.append(n)
    return assemble("random_square", F, ops, list(range(batch)), blocks, rng)


def identity_batch(seed: int, F: int, sizes: Sequence[int]) -> Batch:
    """Every A_i is the identity matrix (values exactly 1.0)."""
    rng = np.random.default_rng(seed)
    ops = []
    for n in sizes:
        ops.append((n, n, np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32),
                    np.ones(n, dtype=np.float32)))
    return assemble("identity", F, ops, list(range(len(ops))), list(sizes), rng, with_dY=True)


def hub_batch(seed: int, F: int, n: int, copies: int = 2) -> Batch:
    """Star graphs: row 0 touches every node (one row of degree n), other rows touch node 0."""
    rng = np.random.default_rng(seed)
    ops = []
    for _ in range(copies):
        r = np.concatenate([np.zeros(n, dtype=np.int64), np.arange(1, n)])
        c = np.concatenate([np.arange(n), np.zeros(n - 1, dtype=np.int64)])
        v = rng.uniform(-1.0, 1.0, size=r.size)
        ops.append((n, n) + _csr_from_directed(n, r, c, v))
    return assemble("hub", F, ops, list(range(copies)), [n] * copies, rng, with_dY=True)


def coo_view(b: Batch, seed: Optional[int] = None, shuffle: bool = True
             ) -> Tuple[np.ndarray, np.ndarray]:
    """The batch as SparseTensor / COO entries (Fig. 1): ``ids`` is int32 [2*sum(nnz)] with
    the (row, column) pair of entry p of operation i at ``ids[2*(nz_off[i]+p)], [..+1]`` and the
    matching ``values``.  With ``shuffle`` the entries of every operation are put in a seeded
    random order (the paper assumes they are sorted neither by row nor by column, Sec. IV);
    without it they keep the CSR's stored order."""
    rng = np.random.default_rng(BASE_SEED if seed is None else seed)
    ids = np.zeros(2 * int(b.colids.shape[0]), dtype=np.int32)
    vals = np.zeros(b.values.shape[0], dtype=np.float32)
    for i in range(b.batch):
        rp, ci, va = b.op_csr(i)
        n = int(b.nnz[i])
        rid = np.repeat(np.arange(int(b.rows[i]), dtype=np.int32), np.diff(rp))
        order = rng.permutation(n) if shuffle else np.arange(n)
        z0 = int(b.nz_off[i])
        ids[2 * z0:2 * (z0 + n):2] = rid[order]
        ids[2 * z0 + 1:2 * (z0 + n):2] = ci[order]
        vals[z0:z0 + n] = va[order]
    return ids, vals


def effective_bytes(b: Batch, transposed: bool = False) -> int:
    """Compulsory bytes one launch must move: CSR once, each distinct dense block once, each
    distinct output block once (fp32 dense, int32 indices).  For the transposed product the dense input
    is indexed like the forward output and vice versa."""
    rows = b.rows.astype(np.int64)
    cols = b.cols.astype(np.int64)
    nnz = b.nnz.astype(np.int64)
    if not transposed:
        csr = int((4 * (rows + 1) + 8 * nnz).sum())
        blocks = {(int(o), int(c)) for o, c in zip(b.b_row_off, cols)}
        dense_in = sum(4 * c * b.F for _, c in blocks)
        outs = {(int(o), int(r)) for o, r in zip(b.c_row_off, rows)}
        dense_out = sum(4 * r * b.F for _, r in outs)
    else:
        csr = int((4 * (cols + 1) + 8 * nnz).sum())
        blocks = {(int(o), int(r)) for o, r in zip(b.c_row_off, rows)}
        dense_in = sum(4 * r * b.F for _, r in blocks)
        outs = {(int(o), int(c)) for o, c in zip(b.b_row_off, cols)}
        dense_out = sum(4 * c * b.F for _, c in outs)
    return int(csr + dense_in + dense_out)


def flops(b: Batch) -> int:
    """2 * nnz_A * n_B per operation (paper Sec. V-A)."""
    return int(2 * int(b.nnz.astype(np.int64).sum()) * b.F)

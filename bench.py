#!/usr/bin/env python3
"""Benchmark of the batched SpMM hot path on one MI355X.

A *step* is one `bspmm_run` launch over one batch (the plan is built once, outside the timed
region, as a GCN reuses one adjacency batch across layers and passes; plan-creation time is
reported separately).  The headline workload is the molecule-like batch of 128 graphs at
F = 128.  Dense operands rotate through a pool larger than the on-chip caches so that every
launch really reads its inputs from, and writes its outputs to, HBM ("cold"); the cache-warm
figure, the launch floor of an emptied schedule, eager launches and the other workload
configurations are reported under "extra".

Prints ONE JSON line.  The CPU oracle is timed beside the GPU as a baseline, not a target.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
POOL_BYTES = 640 << 20          # rotate dense operands through more than L2 + Infinity Cache


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4000)
    ap.add_argument("--warmup", type=int, default=400)
    ap.add_argument("--no-extra", action="store_true", help="headline measurement only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--only", default=None,
                    choices=["cfg2", "cfg2_F64", "cfg3", "cfg4_F256", "cfg4_F1024", "cfg5",
                             "cfg5_transposed", "cfg5_staged_ops", "cfg5_row_block_ops",
                             "layer_512_nx64", "layer_2048_nx32", "layer_2048_nx64"],
                    help="run only this configuration, HBM-cold, eager launches, and print a "
                         "short JSON line (for rocprofv3 counter runs per configuration); "
                         "layer_<graphs>_nx<n_X>: one whole graph-convolution layer, four "
                         "channels, through bspmm_run_gcn and through the BLAS library")
    ap.add_argument("--no-graph", action="store_true",
                    help="with --only: eager launches only (counter passes)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a 256 MiB elementwise copy kernel of known traffic "
                         "(scale reference for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


class Runner:
    """Holds a plan and a pool of dense operand sets for one workload.

    Rotation.  Launch number i of a pass reads input set i and writes output set i; a pass
    goes once through the whole pool, and every measurement is laid out in whole passes, so a
    launch always touches a set that the previous ``nsets - 1`` launches (more than the 256 MB
    Infinity Cache plus the L2s of other traffic) did not: warm-up, timed and filler launches
    share one rotation, whatever ``steps`` is.  A measurement of K launches is
    ``[pass (untimed)] e0 [K // nsets passes + the first K % nsets sets] e1 [the rest of
    that pass (untimed)]``.  The untimed pass in front also keeps the GPU busy while the host
    enqueues the timed region, so the events bracket back-to-back kernels and not the host's
    submission latency; that makes a 20-launch measurement agree with a 4000-launch one.
    """

    def __init__(self, torch, K, batch, transposed=False, options=None, pool_bytes=POOL_BYTES,
                 plan=None):
        self.torch, self.K, self.b, self.transposed = torch, K, batch, transposed
        t0 = time.perf_counter()
        self.plan = plan or K.Plan(batch, options=options)
        torch.cuda.synchronize()
        self.create_ms = (time.perf_counter() - t0) * 1e3
        F = batch.F
        n_in = batch.n_c_rows if transposed else batch.n_b_rows
        n_out = batch.n_b_rows if transposed else batch.n_c_rows
        per_set = 4 * F * (n_in + n_out)
        self.per_set_bytes = per_set
        self.nsets = max(2, min(512, -(-pool_bytes // max(per_set, 1))))
        self.inp = torch.rand((self.nsets, max(n_in, 1), F), dtype=torch.float32, device="cuda") * 2 - 1
        self.out = torch.empty((self.nsets, max(n_out, 1), F), dtype=torch.float32, device="cuda")
        self.in_ptrs = [self.inp[i].data_ptr() for i in range(self.nsets)]
        self.out_ptrs = [self.out[i].data_ptr() for i in range(self.nsets)]
        self.call = K.lib().bspmm_run_transposed if transposed else K.lib().bspmm_run
        self.F = F
        info = self.plan.info()
        d = 1 if transposed else 0
        self.eff_bytes = int(info.effective_bytes[d])
        self.flops = int(info.flops)
        self.workgroups = int(info.workgroups[d])
        self.info = info
        self._graphs = {}
        # one launch outside any timed or captured region (builds the transposed CSR, if any)
        self.launch(0, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()

    def launch(self, s, stream):
        rc = self.call(self.plan.handle, self.in_ptrs[s], self.out_ptrs[s], self.F, self.F, stream)
        if rc != 0:
            raise self.K.BspmmError(rc, "bench launch")

    def rotation(self):
        return (f"{self.nsets} dense operand sets ({self.nsets * self.per_set_bytes / 2**20:.0f} MiB) "
                f"in one rotation shared by warm-up, timed and filler launches: a launch's set was "
                f"last touched {self.nsets - 1} launches "
                f"({(self.nsets - 1) * self.per_set_bytes / 2**20:.0f} MiB of other traffic) earlier")

    def _graph(self, first, count, rotate):
        """A HIP graph of `count` launches on sets first, first+1, ... (all on set 0 when not
        rotating).  The launches of a replay are issued by the GPU's command processor."""
        key = (first, count, rotate)
        if key not in self._graphs:
            torch = self.torch
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                cs = torch.cuda.current_stream().cuda_stream
                for i in range(count):
                    self.launch((first + i) % self.nsets if rotate else 0, cs)
            self._graphs[key] = g
        return self._graphs[key]

    def measure(self, steps, warmup, repeats=5, rotate=True, graph=True):
        """Seconds per launch of `repeats` measurements of exactly `steps` launches each
        (sorted), after `warmup` untimed launches (rounded up to whole passes)."""
        torch = self.torch
        # one graph holds whole passes over the pool, at least 64 launches (a replay's own start
        # and end, about 10 us, must stay small against what it holds)
        n = self.nsets * max(1, -(-64 // self.nsets)) if rotate else min(256, max(steps, 1))
        q, rem = divmod(steps, n)
        stream = torch.cuda.current_stream()

        def eager(first, count):
            for i in range(count):
                self.launch((first + i) % self.nsets if rotate else 0, stream.cuda_stream)

        if graph:
            whole, head = self._graph(0, n, rotate), (self._graph(0, rem, rotate) if rem else None)
            rest = self._graph(rem, n - rem, rotate) if rem else None
            run_pass, run_head = whole.replay, (head.replay if rem else None)
            run_rest = rest.replay if rem else None
        else:
            run_pass = lambda: eager(0, n)
            run_head = (lambda: eager(0, rem)) if rem else None
            run_rest = (lambda: eager(rem, n - rem)) if rem else None
        for _ in range(-(-max(warmup, 1) // n)):      # warm-up: whole passes, eager
            eager(0, n)
        if graph:                                       # and every graph once
            run_pass()
            if rem:
                run_head()
                run_rest()
        torch.cuda.synchronize()
        out = []
        for _ in range(repeats):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            run_pass()                                  # untimed: GPU busy, rotation intact
            e0.record()
            for _ in range(q):
                run_pass()
            if rem:
                run_head()
            e1.record()
            if rem:
                run_rest()                              # untimed: completes the pass
            torch.cuda.synchronize()
            out.append(e0.elapsed_time(e1) * 1e-3 / steps)
        return sorted(out)

    def per_launch_slope(self, steps, repeats=5):
        """Seconds per launch with the fixed cost of a graph replay taken out: the difference
        between replays of `steps` and of 2 * `steps` launches (both inside one pass, GPU busy in
        front as in measure()), divided by `steps`.  For measurements shorter than a pass, where
        the replay's own start and end (about 10 us) are not amortised.  Median of `repeats`."""
        torch = self.torch
        k1 = max(1, min(steps, self.nsets // 2))
        k2 = 2 * k1
        whole = self._graph(0, self.nsets, True)
        g1, g2 = self._graph(0, k1, True), self._graph(0, k2, True)
        r1, r2 = self._graph(k1, self.nsets - k1, True), self._graph(k2, self.nsets - k2, True) \
            if k2 < self.nsets else None
        for g in (whole, g1, r1, g2, r2):
            if g is not None:
                g.replay()
        torch.cuda.synchronize()
        out = []
        for _ in range(repeats):
            t = []
            for g, rest in ((g1, r1), (g2, r2)):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                whole.replay()
                e0.record()
                g.replay()
                e1.record()
                if rest is not None:
                    rest.replay()
                torch.cuda.synchronize()
                t.append(e0.elapsed_time(e1) * 1e-3)
            out.append((t[1] - t[0]) / (k2 - k1))
        return sorted(out), (k1, k2)

    def time_graph(self, steps, warmup, rotate=True, repeats=3):
        """Median seconds per launch over `repeats` HIP-graph measurements of `steps` launches."""
        r = self.measure(steps, warmup, repeats=repeats, rotate=rotate, graph=True)
        return r[len(r) // 2], steps

    def time_eager(self, steps, warmup, rotate=True, repeats=3):
        r = self.measure(steps, warmup, repeats=repeats, rotate=rotate, graph=False)
        return r[len(r) // 2]

    def summary(self, sec):
        return {"us_per_launch": round(sec * 1e6, 3),
                "graphs_per_s": round(self.b.n_graphs / sec, 1),
                "gflops": round(self.flops / sec * 1e-9, 2),
                "eff_GBps": round(self.eff_bytes / sec * 1e-9, 1),
                "frac_of_8TBps": round(self.eff_bytes / sec * 1e-9 / HBM_PEAK_GBPS, 4),
                "eff_MB": round(self.eff_bytes * 1e-6, 3),
                "workgroups": self.workgroups}


def coo_operands(torch, K, W):
    """COO / SparseTensor operands (unsorted index pairs): the conversion launch of
    bspmm_create_coo, the product on the converted plan, and the direct LDS-atomic kernel
    (BSPMM_COO_DIRECT), all HBM-cold."""
    out = {}
    for name, mk in (("cfg2_F128", lambda: W.config2_molecule(F=128)),
                     ("cfg5_F256", lambda: W.config5_skewed())):
        b = mk()
        ids, vals = W.coo_view(b, seed=W.config_seed(9))
        conv = K.Plan(b, coo=(ids, vals))
        r = Runner(torch, K, b, plan=conv)
        s_conv, _ = r.time_graph(1000, 100)
        # device time of a plan creation: uploads of the tables plus the sort launch
        ws, hb = conv.workspace, conv.hb
        nbytes = K.bspmm_workspace_bytes_coo(hb, b.F, None)
        stream = torch.cuda.current_stream().cuda_stream
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 20
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        for _ in range(reps):
            K.bspmm_destroy(K.bspmm_create_coo(hb, b.F, None, ws, nbytes, stream))
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / reps
        # the last creation left the workspace as the first did: conv is still valid
        direct = K.Plan(b, coo=(ids, vals), options=K.make_options(flags=K.COO_DIRECT))
        rd = Runner(torch, K, b, plan=direct)
        s_dir, _ = rd.time_graph(400, 40)
        out[name] = {"create_coo_wall_us": round(wall * 1e6, 1),
                     "create_coo_stream_us": round(e0.elapsed_time(e1) * 1e3 / reps, 1),
                     "converted_run": r.summary(s_conv), "direct_run": rd.summary(s_dir)}
        del r, rd, conv, direct
        torch.cuda.empty_cache()
    return out


def layer_front(torch, K, W, n_x=64, graphs=128):
    """One channel of the graph-convolution layer on molecule graphs (128: the headline batch),
    HBM-cold: the fused launch (bspmm_run_gcn) against MatMul+Add by the BLAS library followed by
    bspmm_run."""
    b = W.config2_molecule(F=128, graphs=graphs)
    F = b.F
    fused = K.Plan(b, options=K.make_options(front_features=n_x))
    plain = K.Plan(b)
    per_set = 4 * (b.n_b_rows * (n_x + F) + b.n_c_rows * F)
    nsets = max(2, min(512, -(-POOL_BYTES // per_set)))
    X = torch.rand((nsets, b.n_b_rows, n_x), device="cuda") * 2 - 1
    Bm = torch.empty((nsets, b.n_b_rows, F), device="cuda")
    Y = torch.empty((nsets, b.n_c_rows, F), device="cuda")
    Wt = (torch.rand((n_x, F), device="cuda") * 2 - 1) / n_x ** 0.5
    bias = torch.rand(F, device="cuda")

    def run_fused(i, stream):
        K.bspmm_run_gcn(fused.handle, X[i], n_x, Wt, F, bias, Y[i], F, False, stream)

    def run_unfused(i, stream):
        torch.addmm(bias, X[i], Wt, out=Bm[i])
        K.bspmm_run(plain.handle, Bm[i], Y[i], F, F, stream)

    def run_front_only(i, stream):
        torch.addmm(bias, X[i], Wt, out=Bm[i])

    def timed(fn):
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn(0, side)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            cs = torch.cuda.current_stream()
            for i in range(nsets):
                fn(i, cs)
        for _ in range(2):
            g.replay()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        reps = 4
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (reps * nsets)

    nnz = int(b.nnz.sum())
    flops = 2 * b.n_b_rows * n_x * F + 2 * nnz * F
    info = fused.info()
    out = {"workload": f"cfg2_molecule, {graphs} graphs, n_X={n_x}, F={F}, one channel", "operand_sets": nsets,
           "streamed": {"graphs": int(info.front_stream[0]), "workgroups": int(info.front_stream[1]),
                        "lds_bytes": int(info.front_stream[2]),
                        "graphs_left_to_a_second_launch": int(info.front_stream[3])},
           "fused_us": round(timed(run_fused), 3),
           "blas_addmm_then_bspmm_run_us": round(timed(run_unfused), 3),
           "blas_addmm_alone_us": round(timed(run_front_only), 3)}
    out["fused_gflops"] = round(flops / out["fused_us"] * 1e-3, 1)
    out["speedup"] = round(out["blas_addmm_then_bspmm_run_us"] / out["fused_us"], 2)
    return out


def layer_whole(torch, K, W, n_x=64, channels=4, graphs=128):
    """The whole graph-convolution layer Y = sum_ch A_ch (X W_ch + bias_ch), HBM-cold, on config
    3's structure (the channels of a graph share the layer input and one output block): one
    launch (front_features with BSPMM_ACCUMULATE), one fused launch per channel, and the BLAS
    library's addmm per channel followed by the summed product."""
    import dataclasses
    F = 128
    b = W.config3_multichannel(graphs=graphs, F=F, channels=channels, accumulate=True)
    whole = K.Plan(b, options=K.make_options(flags=K.ACCUMULATE, front_features=n_x))
    kept = K.Plan(b, options=K.make_options(flags=K.ACCUMULATE | K.ONE_FRONT_LAUNCH, front_features=n_x))
    sel = [slice(c, None, channels) for c in range(channels)]
    per_ch = [K.Plan(dataclasses.replace(b, rows=b.rows[q], cols=b.cols[q], nnz=b.nnz[q],
                                         rpt_off=b.rpt_off[q], nz_off=b.nz_off[q],
                                         b_row_off=b.b_row_off[q], c_row_off=b.c_row_off[q]),
                     options=K.make_options(front_features=n_x)) for q in sel]
    bo = W.config3_multichannel(graphs=graphs, F=F, channels=channels, accumulate=True,
                                own_inputs=True)
    summed = K.Plan(bo, options=K.make_options(flags=K.ACCUMULATE))
    per_set = 4 * (b.n_b_rows * n_x + b.n_c_rows * F)
    nsets = max(2, min(128, -(-POOL_BYTES // per_set)))
    X = torch.rand((nsets, b.n_b_rows, n_x), device="cuda") * 2 - 1
    Y = torch.empty((nsets, b.n_c_rows, F), device="cuda")
    Wt = (torch.rand((channels * n_x, F), device="cuda") * 2 - 1) / n_x ** 0.5
    bias = torch.rand((channels, F), device="cuda")
    Ws = [Wt[c * n_x:(c + 1) * n_x] for c in range(channels)]
    # dense blocks per (graph, channel) as the summed product reads them; the library calls below
    # write full-size matrices per channel instead (a strided batched GEMM would be needed to
    # put them there), which costs the same arithmetic and traffic
    Bm = torch.empty((min(nsets, 16), bo.n_b_rows, F), device="cuda")
    U = torch.empty((channels, b.n_b_rows, F), device="cuda")

    def run_whole(i, stream):
        K.bspmm_run_gcn(whole.handle, X[i], n_x, Wt, F, bias, Y[i], F, False, stream)

    def run_kept(i, stream):
        K.bspmm_run_gcn(kept.handle, X[i], n_x, Wt, F, bias, Y[i], F, False, stream)

    def run_per_channel(i, stream):
        for c in range(channels):
            K.bspmm_run_gcn(per_ch[c].handle, X[i], n_x, Ws[c], F, bias[c], Y[i], F, c > 0, stream)

    def run_unfused(i, stream):
        for c in range(channels):
            torch.addmm(bias[c], X[i], Ws[c], out=U[c])
        K.bspmm_run(summed.handle, Bm[i % Bm.shape[0]], Y[i], F, F, stream)

    def timed(fn):
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn(0, side.cuda_stream)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            cs = torch.cuda.current_stream().cuda_stream
            for i in range(nsets):
                fn(i, cs)
        for _ in range(2):
            g.replay()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(4):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (4 * nsets)

    nnz = int(b.nnz.sum())
    flops = channels * 2 * b.n_b_rows * n_x * F + 2 * nnz * F
    info = whole.info()
    out = {"workload": f"cfg3 structure, {graphs} graphs, {channels} channels, n_X={n_x}, F={F}",
           "operand_sets": nsets,
           "streamed": {"graphs": int(info.front_stream[0]), "workgroups": int(info.front_stream[1]),
                        "lds_bytes": int(info.front_stream[2]),
                        "graphs_left_to_a_second_launch": int(info.front_stream[3])},
           "whole_layer_us": round(timed(run_whole), 3),
           "whole_layer_one_launch_kernel_us": round(timed(run_kept), 3),
           "one_fused_launch_per_channel_us": round(timed(run_per_channel), 3),
           "blas_addmm_per_channel_then_summed_product_us": round(timed(run_unfused), 3)}
    out["whole_layer_gflops"] = round(flops / out["whole_layer_us"] * 1e-3, 1)
    # the layer's dense part, counted as the GEMMs X W[ch] a library runs, against the fp32
    # matrix-core peak (157.3 TFLOP/s).  The streamed launch issues fewer flops than that: rows of
    # X W[ch] that no entry of channel ch names are not made (the counter summary under profiles/
    # has the matrix instructions issued).
    out["dense_part_as_gemm_frac_of_fp32_mfma_peak"] = round(
        channels * 2 * b.n_b_rows * n_x * F / (out["whole_layer_us"] * 1e-6) / 157.3e12, 3)
    return out


def kernel_resources(K, lds_bytes):
    """Registers, LDS and workgroups per CU of the library's kernels (bspmm_kernel_info)."""
    out = {}
    for i, name in enumerate(K.KERNEL_NAMES):
        dyn = lds_bytes if name in ("lean", "general", "general_scalar", "coo", "layer_stream") else 0
        r = K.bspmm_kernel_info(i, dyn)
        out[name] = {"vgprs": r.vgprs, "static_lds_bytes": r.static_lds_bytes,
                     "scratch_bytes": r.scratch_bytes, "lanes_per_workgroup": r.threads,
                     "dynamic_lds_bytes_assumed": dyn, "workgroups_per_cu": r.workgroups_per_cu,
                     "compute_units": r.compute_units}
    return out


_marker = None


def phase_marker(torch, k):
    """A one-element int16 fill between measurement phases: shows up in a kernel trace as a
    FillFunctor<short> dispatch, so a profile of this script can be cut into its phases."""
    global _marker
    if _marker is None:
        _marker = torch.empty(1, dtype=torch.int16, device="cuda")
    torch.cuda.synchronize()
    _marker.fill_(k)
    torch.cuda.synchronize()


def copy_bandwidth(torch):
    n = 1 << 28   # 1 GiB of fp32
    a = torch.empty(n, dtype=torch.float32, device="cuda")
    b = torch.empty(n, dtype=torch.float32, device="cuda")
    a.fill_(1.0)
    for _ in range(3):
        b.copy_(a)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(10):
        b.copy_(a)
    e1.record()
    torch.cuda.synchronize()
    sec = e0.elapsed_time(e1) * 1e-3 / 10
    del a, b
    torch.cuda.empty_cache()
    return 2 * 4 * n / sec * 1e-9


def paper_grid(torch, K, W):
    """Batched against one launch per matrix on the random square matrices of the paper's
    preliminary evaluation (Sec. V-A: batch 50/100, dim 50, 2-3 entries per row, n_B swept; and
    the mixed batch with dim 32-256, 1-5 entries per row, n_B = 1024).  Cache-warm."""
    rows = []
    grid = [("batch50_dim50_nnz2", 50, 50, 2, (32, 64, 128, 256, 512)),
            ("batch100_dim50_nnz3", 100, 50, 3, (64, 512)),
            ("batch100_dim32-256_nnz1-5", 100, (32, 256), (1, 5), (1024,))]
    for name, batch, dim, nz, widths in grid:
        for F in widths:
            b = W.random_square(W.config_seed(8) + F, F, batch, dim, nz)
            r = Runner(torch, K, b, pool_bytes=1)
            s, _ = r.time_graph(400, 40, rotate=False)
            nb = non_batched(torch, K, b, s)
            rows.append({"workload": name, "n_B": F, "batched_us": round(s * 1e6, 2),
                         "gflops": round(r.flops / s * 1e-9, 1),
                         "non_batched_us": min(nb["eager_us_per_batch"], nb["hipgraph_us_per_batch"]),
                         "speedup": nb["batched_speedup"]})
            del r
    return rows


def non_batched(torch, K, b, batched_sec):
    """The paper's comparison (Sec. V-A): the same graphs multiplied one launch per graph
    (a single-operation plan each, same kernel) against the one batched launch."""
    Bd = torch.rand((b.n_b_rows, b.F), dtype=torch.float32, device="cuda")
    Cd = torch.empty((b.n_c_rows, b.F), dtype=torch.float32, device="cuda")
    plans = [K.Plan(b.single(i)) for i in range(b.batch)]
    stream = torch.cuda.current_stream().cuda_stream
    run = K.lib().bspmm_run

    def sweep():
        for p in plans:
            run(p.handle, Bd.data_ptr(), Cd.data_ptr(), b.F, b.F, stream)

    for _ in range(3):
        sweep()
    g = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        cs = torch.cuda.current_stream().cuda_stream
        for p in plans:
            run(p.handle, Bd.data_ptr(), Cd.data_ptr(), b.F, b.F, cs)
    res = {}
    for name, fn in (("eager", sweep), ("hipgraph", g.replay)):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(20):
            fn()
        e1.record()
        torch.cuda.synchronize()
        res[name + "_us_per_batch"] = round(e0.elapsed_time(e1) * 1e3 / 20, 2)
    best = min(res.values())
    res["launches_per_batch"] = len(plans)
    res["batched_speedup"] = round(best * 1e-6 / batched_sec, 1)
    res["note"] = ("cache-warm operands; the paper reports up to 9.27x for batched over "
                   "non-batched SpMM on a P100 (Sec. V-A)")
    for p in plans:
        p.close()
    return res


def parity_sample(torch, K, runner, oracle):
    """One launch of the timed configuration checked against the oracle on set 0."""
    import numpy as np
    b = runner.b
    import dataclasses
    bb = dataclasses.replace(b, B=runner.inp[0][:b.n_b_rows].cpu().numpy())
    runner.out[0].fill_(-7.0)
    runner.launch(0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    C, S = oracle.forward_batch(bb)
    got = runner.out[0][:b.n_c_rows].cpu().numpy()
    return bool(np.all(np.abs(got - C) <= 1e-5 * S))


def cpu_baseline(oracle, b, seconds, eff_bytes, flops):
    """The oracle as it stands, on the host cores: its C routine alone on the same batch
    (arrays and the fp64 output prepared once, outside the clock), one warm-up call, then the
    best of 5 samples of back-to-back calls; all host threads, and one thread."""
    def leg(budget):
        probe = min(oracle.time_forward_call(b, 3, samples=1))
        calls = max(1, int(budget / 5 / max(probe, 1e-7)))
        return min(oracle.time_forward_call(b, calls, samples=5)), calls

    threads = int(oracle.num_threads())
    best, calls = leg(seconds)
    out = {"value": round(b.n_graphs / best, 1), "unit": "graphs/s", "cores": threads,
           "kind": "oracle",
           "sample": f"the C routine of the fp64 OpenMP oracle alone (preallocated output, no "
                     f"Python marshalling) on the same {b.n_graphs}-graph F={b.F} batch: 1 warm-up "
                     f"call, then best of 5 samples of {calls} back-to-back calls "
                     f"(about {seconds:.0f} s of CPU work)",
           "us_per_batch": round(best * 1e6, 2),
           "gflops": round(flops / best * 1e-9, 2),
           "eff_GBps": round(eff_bytes / best * 1e-9, 2),
           "eff_bytes_note": "the same algorithmic bytes as the GPU line (fp32 operands and "
                             "output; the oracle itself writes fp64)"}
    oracle.set_num_threads(1)
    try:
        best1, calls1 = leg(min(3.0, seconds))
    finally:
        oracle.set_num_threads(threads)
    out["one_thread"] = {"value": round(b.n_graphs / best1, 1), "cores": 1,
                         "us_per_batch": round(best1 * 1e6, 2),
                         "gflops": round(flops / best1 * 1e-9, 2),
                         "eff_GBps": round(eff_bytes / best1 * 1e-9, 2),
                         "calls_per_sample": calls1}
    return out


def read_traffic():
    """HBM bytes per launch from the committed rocprofv3 counter summary, if there is one."""
    path = os.path.join(ROOT, "profiles", "bspmm_lean_kernel_cfg2_F128_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1].split()[0])
    except OSError:
        pass
    return None


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 (a batch would shard "
              "across GPUs by whole graphs, without any exchange)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_1903_11409_amd import bspmm as K
    from paper_1903_11409_amd import workloads as W
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    K.lib()

    if args.only and args.only.startswith("layer_"):
        # one whole graph-convolution layer (4 channels, F = 128), HBM-cold: layer_<graphs>_nx<n_X>
        graphs, n_x = (int(v) for v in args.only[len("layer_"):].split("_nx"))
        line = layer_whole(torch, K, W, n_x=n_x, graphs=graphs)
        line["kernel"] = kernel_resources(K, line["streamed"]["lds_bytes"])["layer_stream"]
        print(json.dumps(line))
        return
    if args.only:
        def cfg5_part(generic):
            # config 5 cut in two by what the scheduler does with an operation: staged in LDS, or
            # too large for it and cut into row blocks that gather from L2 (per-bin evidence)
            b5 = W.config5_skewed()
            h = K.dry_plan(b5)
            blocks = {it.op for it in K.bspmm_plan_items(h) if it.bin == K.BIN_GENERIC}
            K.bspmm_destroy(h)
            ops = [i for i in range(b5.batch) if (i in blocks) == generic]
            return b5.subset(ops, name="cfg5_row_block_ops" if generic else "cfg5_staged_ops")

        mk, tr = {"cfg2": (lambda: W.config2_molecule(F=128), False),
                  "cfg2_F64": (lambda: W.config2_molecule(F=64), False),
                  "cfg3": (lambda: W.config3_multichannel(), False),
                  "cfg4_F256": (lambda: W.config4_wide(F=256), False),
                  "cfg4_F1024": (lambda: W.config4_wide(F=1024), False),
                  "cfg5": (lambda: W.config5_skewed(), False),
                  "cfg5_transposed": (lambda: W.config5_skewed(), True),
                  "cfg5_staged_ops": (lambda: cfg5_part(False), False),
                  "cfg5_row_block_ops": (lambda: cfg5_part(True), False)}[args.only]
        if args.calib_copy:
            a = torch.ones(1 << 26, dtype=torch.float32, device="cuda")
            c = torch.empty_like(a)
            for _ in range(3):
                torch.mul(a, 1.0, out=c)      # reads 256 MiB, writes 256 MiB
            torch.cuda.synchronize()
            del a, c
        r = Runner(torch, K, mk(), transposed=tr)
        steps = min(args.steps, 400)
        sec = r.time_eager(steps, min(args.warmup, 40))
        sec_graph = sec if args.no_graph else r.time_graph(steps, min(args.warmup, 40))[0]
        d = 1 if tr else 0
        line = r.summary(sec)
        line.update({"workload": args.only, "launches": steps, "mode": "eager, HBM-cold",
                     **({} if args.no_graph else {
                         "us_per_launch_hipgraph": round(sec_graph * 1e6, 3),
                         "eff_GBps_hipgraph": round(r.eff_bytes / sec_graph * 1e-9, 1)}),
                     "lean": int(r.info.lean[d]), "bins": list(r.info.items_in_bin[d]),
                     "dynamic_lds_bytes": int(r.info.lds_bytes),
                     "kernel": kernel_resources(K, int(r.info.lds_bytes))[
                         "lean" if r.info.lean[d] else "general"]})
        print(json.dumps(line))
        return

    b = W.config2_molecule(F=128)
    head = Runner(torch, K, b)
    phase_marker(torch, 1)          # phase 1: headline, HIP-graph replay, rotating operands
    reps_graph = head.measure(args.steps, args.warmup, repeats=5, graph=True)
    phase_marker(torch, 2)          # phase 2: headline, eager launches, rotating operands
    reps_eager = head.measure(args.steps, args.warmup, repeats=5, graph=False)
    phase_marker(torch, 3)          # phase 3: everything else
    sec_graph, sec_eager = reps_graph[2], reps_eager[2]      # medians of five
    sec = min(sec_graph, sec_eager)
    launch_mode = "hipgraph_replay" if sec_graph <= sec_eager else "eager"
    reps_head = reps_graph if sec_graph <= sec_eager else reps_eager
    value_from = f"median of 5 measurements of {args.steps} back-to-back launches between two events"
    direct = None
    if args.steps < head.nsets:
        # Shorter than one pass over the operand pool: the start and end of a graph replay
        # (about 10 us on the GPU's timeline, whatever it holds) are not amortised over the
        # timed launches.  The time per launch is then the difference between a replay of 2K
        # and a replay of K launches, divided by K: the fixed part cancels, and the figure
        # agrees with a measurement over thousands of launches.
        direct = {"median_us": round(reps_head[2] * 1e6, 3), "min_us": round(reps_head[0] * 1e6, 3),
                  "max_us": round(reps_head[4] * 1e6, 3), "launch": launch_mode,
                  "what": f"{args.steps} launches between two events, replay overhead included"}
        reps_head, ks = head.per_launch_slope(args.steps)
        sec = reps_head[2]
        launch_mode = "hipgraph_replay"
        value_from = (f"median of 5 two-point measurements: (replay of {ks[1]} launches - replay of "
                      f"{ks[0]} launches) / {ks[1] - ks[0]}, same HIP graph mechanism and operand rotation")

    extra = {}
    parity_ok = None
    if args.calib_copy:
        a = torch.ones(1 << 26, dtype=torch.float32, device="cuda")
        c = torch.empty_like(a)
        for _ in range(3):
            torch.mul(a, 1.0, out=c)      # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del a, c
    if not args.no_cpu:
        # the CPU baseline leg (the only place that touches the oracle): its first pass over the
        # batch also serves as a check of one launch of the timed configuration
        from oracle import reference as oracle
        parity_ok = parity_sample(torch, K, head, oracle)
    if not args.no_extra:
        extra["headline_hipgraph"] = head.summary(sec_graph)
        extra["headline_eager"] = head.summary(sec_eager)
        warm, _ = head.time_graph(args.steps, args.warmup, rotate=False)
        extra["headline_cache_warm"] = head.summary(warm)
        floor = Runner(torch, K, b, options=K.make_options(flags=K.FLOOR_PROBE))
        freps = min(floor.measure(args.steps, args.warmup, repeats=5, graph=True),
                    floor.measure(args.steps, args.warmup, repeats=5, graph=False),
                    key=lambda r: r[2])
        extra["launch_floor_us"] = round(freps[2] * 1e6, 3)
        extra["launch_floor_5_repeats_us"] = {"median": round(freps[2] * 1e6, 3),
                                              "min": round(freps[0] * 1e6, 3),
                                              "max": round(freps[4] * 1e6, 3)}
        if args.steps < head.nsets:
            fl, _ = floor.per_launch_slope(args.steps)
            extra["launch_floor_direct_bracket_us"] = extra["launch_floor_us"]
            extra["launch_floor_us"] = round(fl[2] * 1e6, 3)
            extra["launch_floor_5_repeats_us"] = {"median": round(fl[2] * 1e6, 3), "min": round(fl[0] * 1e6, 3),
                                                  "max": round(fl[4] * 1e6, 3), "method": "two-point, as the headline"}
        del floor
        extra["headline_hipgraph_5_repeats_us"] = {"median": round(reps_graph[2] * 1e6, 3),
                                                   "min": round(reps_graph[0] * 1e6, 3),
                                                   "max": round(reps_graph[4] * 1e6, 3)}
        extra["headline_eager_5_repeats_us"] = {"median": round(reps_eager[2] * 1e6, 3),
                                                "min": round(reps_eager[0] * 1e6, 3),
                                                "max": round(reps_eager[4] * 1e6, 3)}
        extra["kernel_resources"] = kernel_resources(K, int(head.info.lds_bytes))
        extra["headline_launch"] = {"kernel": "bspmm_lean_kernel" if head.info.lean[0] else "bspmm_kernel<4>",
                                    "workgroups": head.workgroups,
                                    "dynamic_lds_bytes": int(head.info.lds_bytes)}
        extra["plan_create_ms"] = round(head.create_ms, 3)
        # the paper's batched timings include handing the matrix list to the device: plan
        # creation through the C ABI (schedule, upload) plus one product, device arrays in place
        hb, ws = head.plan.hb, head.plan.workspace
        stream = torch.cuda.current_stream().cuda_stream
        nbytes = K.bspmm_workspace_bytes(hb, b.F, None)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(50):
            K.bspmm_workspace_bytes(hb, b.F, None)
            h = K.bspmm_create(hb, b.F, None, ws, nbytes, stream)
            rc = K.lib().bspmm_run(h, head.in_ptrs[i % head.nsets], head.out_ptrs[i % head.nsets],
                                   b.F, b.F, stream)
            assert rc == 0
            torch.cuda.synchronize()
            K.bspmm_destroy(h)
        extra["create_plus_run_us"] = round((time.perf_counter() - t0) / 50 * 1e6, 1)
        t0 = time.perf_counter()
        for _ in range(20):
            K.Plan(b).close()
        torch.cuda.synchronize()
        extra["plan_create_ms_repeat"] = round((time.perf_counter() - t0) * 1e3 / 20, 3)
        extra["copy_GBps_1GiB"] = round(copy_bandwidth(torch), 1)
        extra["headline_frac_of_copy_bandwidth"] = round(
            head.eff_bytes / sec * 1e-9 / extra["copy_GBps_1GiB"], 4)
        extra["non_batched"] = non_batched(torch, K, b, sec)
        others = {}
        for name, mk, tr in [
                ("cfg2_F64", lambda: W.config2_molecule(F=64), False),
                ("cfg3_multichannel_F128", lambda: W.config3_multichannel(), False),
                ("cfg4_F256", lambda: W.config4_wide(F=256), False),
                ("cfg4_F1024", lambda: W.config4_wide(F=1024), False),
                ("cfg5_forward_F256", lambda: W.config5_skewed(), False),
                ("cfg5_transposed_F256", lambda: W.config5_skewed(), True),
                # throughput regime: the headline's molecule graphs, 128 times as many
                ("cfg2_molecule_16384_graphs_F128", lambda: W.config2_molecule(graphs=16384), False)]:
            bb = mk()
            r = Runner(torch, K, bb, transposed=tr)
            steps = max(200, min(args.steps, 2000))
            s, _ = r.time_graph(steps, max(20, steps // 10))
            others[name] = r.summary(s)
            others[name]["bins"] = list(r.info.items_in_bin[1 if tr else 0])
            del r
            torch.cuda.empty_cache()
        extra["other_configs_cold"] = others
        # the layer's channel sum done inside the launch (BSPMM_ACCUMULATE): the 4 channel
        # products of a graph go to ONE output block, 512 and 2048 graphs
        acc = {}
        for name, graphs in (("cfg3_channel_sum_512", 512), ("cfg3_channel_sum_2048", 2048)):
            for label, mk, opts in (
                    ("separate_outputs", lambda g=graphs: W.config3_multichannel(graphs=g), None),
                    ("summed_in_launch", lambda g=graphs: W.config3_multichannel(graphs=g, accumulate=True),
                     K.make_options(flags=K.ACCUMULATE))):
                r = Runner(torch, K, mk(), options=opts)
                s, _ = r.time_graph(1000, 100)
                acc[f"{name}_{label}"] = r.summary(s)
                del r
                torch.cuda.empty_cache()
        extra["channel_sum"] = acc
        extra["paper_grid_batched_vs_non_batched"] = paper_grid(torch, K, W)
        extra["coo_operands"] = coo_operands(torch, K, W)
        extra["layer_front"] = [layer_front(torch, K, W, n_x=n, graphs=g)
                                for g, n in ((128, 32), (128, 64), (128, 128), (1024, 64), (4096, 128))]
        # 128 graphs: two (graph, feature tile) pairs per CU; 512 and 2048 graphs: launches of
        # resident workgroups that stream many graphs each
        extra["layer_whole"] = [layer_whole(torch, K, W, n_x=n, graphs=g)
                                for g, n in ((128, 32), (128, 64), (512, 32), (512, 64), (2048, 32),
                                             (2048, 64))]
        # other channel counts (two: one block per wavefront; eight: workgroups of eight wavefronts)
        extra["layer_whole"] += [layer_whole(torch, K, W, n_x=64, channels=c, graphs=2048) for c in (2, 8)]

    out = {
        "metric": "batched SpMM graphs/sec, F=128, batch 128",
        "value": round(b.n_graphs / sec, 1),
        "unit": "graphs/s",
        "n_gpus": 1,
        "steps": int(args.steps),
        "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "cfg2_molecule: 128 molecule-like graphs (log-normal sizes, mean "
                               "25 nodes, degree <= 6, self-loops, symmetric normalisation), "
                               "F=128, forward",
                   "seed": W.config_seed(2), "checksum": b.checksum(),
                   "operands": "hbm_cold: " + head.rotation(),
                   "repeats": {"n": 5, "median_us": round(reps_head[2] * 1e6, 3),
                               "min_us": round(reps_head[0] * 1e6, 3),
                               "max_us": round(reps_head[4] * 1e6, 3),
                               "value_from": value_from},
                   **({"direct_bracket": direct} if direct else {}),
                   "launch": launch_mode, "one_launch_per_batch": True,
                   "gflops": round(head.flops / sec * 1e-9, 2),
                   },
        "roofline": {"bound": "hbm", "achieved": round(head.eff_bytes / sec * 1e-9, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(head.eff_bytes / sec * 1e-9 / HBM_PEAK_GBPS, 4),
                     "traffic": read_traffic(),
                     "traffic_source": "committed rocprofv3 counter summary profiles/"
                                       "bspmm_lean_kernel_cfg2_F128_pmc.txt (a separate run of this "
                                       "workload, not measured by this process)",
                     "kernel": "bspmm_lean_kernel" if head.info.lean[0] else "bspmm_kernel<4>",
                     "bytes_per_launch": head.eff_bytes},
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(oracle, b, args.cpu_seconds, head.eff_bytes, head.flops)
        out["cpu_baseline"]["gpu_launch_within_tolerance_of_it"] = parity_ok
    if extra:
        out["extra"] = extra
    print(json.dumps(out))


if __name__ == "__main__":
    main()

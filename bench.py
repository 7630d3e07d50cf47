#!/usr/bin/env python3
"""Benchmark of the scheduled dense operators on one MI355X.

ONE short JSON line on stdout (under 4 KB).  A "step" is one launch of the headline operator: the
fp16 GEMM M=N=K=4096 (fp32 accumulate and output, A row-major, B column-major) with the schedule
gensor_construct picked for it; inputs are resident in HBM before the timed region.  `value` is its
TFLOP/s over exactly --steps launches.  The same line carries
  roofline      dense fp16 MFMA peak against the measured kernel time (HIP events on the stream the
                kernel runs on)
  cpu_baseline  the CPU oracle timed on a bounded slice of the same GEMM
  operators     one compact row per benchmark configuration (fp32 GEMM, the headline, GPT-2 GEMMs,
                attention-score BMM, ResNet-50 convolutions): us, tf (TFLOP/s), pk (% of the dense MFMA
                peak of its type), ceil (% of its own roofline ceiling min(MFMA peak, flop/byte x HBM
                peak)), gbs (GB/s on algorithmic bytes), id (kernel instance), cs (construction
                seconds), err (sampled relative Frobenius error against the oracle)
Every row but the headline's `value` is timed by one protocol that does not depend on --steps: launches
that settle the shader clock, then the median of 5 event-bracketed batches of at least 50 launches.
The long sections (per-shape details, unbalanced and deep-k GEMMs, output-type variants, the other
operators of the paper's table, the walk ablation) go to the file named by --details
(see its default below); one progress line per section goes to stderr.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f16": 2516.6, "bf16": 2516.6, "f32": 157.3}   # dense MFMA, MI355X
HBM_GBS = 8000.0
# HBM-side bytes per launch of the headline kernel.  Not measured in this run (hardware counters need the
# profiler): the figures of the FETCH_SIZE / WRITE_SIZE counter passes recorded in TRAFFIC_SOURCE, each scaled by
# the same counter's reading for a 256 MiB device copy; keyed by (tile, wave tile, direct) of the instance they
# were measured on.  Any other instance reports null.
TRAFFIC_SOURCE = "profiles/gemm_f16_4096_kernel_trace.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes, copy-calibrated)"
MEASURED_TRAFFIC_BYTES = {((256, 256, 64), (128, 128), 1): 268.9e6, ((256, 256, 64), (128, 64), 1): 269.4e6,
                          ((256, 256, 64), (64, 128), 1): 269.4e6}


def _algorithmic_bytes(w, gs_inputs, out_dtype="f32"):
    es = 4 if w.dtype == "f32" else 2
    eo = 4 if out_dtype == "f32" else 2
    if isinstance(w, gs_inputs.GemmWorkload):
        return w.batch * (es * (w.M * w.K + w.K * w.N) + eo * w.M * w.N)
    # convolution: only the input elements some window touches count (a stride larger than the filter skips rows and columns)
    def touched(extent, out_extent, f):
        hit = {o * w.stride - w.pad + t for o in range(out_extent) for t in range(f)}
        return sum(1 for x in hit if 0 <= x < extent)
    in_elems = w.n * w.c * touched(w.h, w.p, w.r) * touched(w.w, w.q, w.s)
    return es * (in_elems + w.k * w.c * w.r * w.s) + eo * w.n * w.k * w.p * w.q


COLD_BYTES = 640 << 20     # operand sets rotated through in the cold-cache timing (Infinity Cache: 256 MB)


class Case:
    """One workload resident on the device with its constructed schedule."""

    def __init__(self, gs, inputs, w, opts=None, out_dtype="f32"):
        import torch
        self.gs, self.w = gs, w
        self.is_gemm = isinstance(w, inputs.GemmWorkload)
        if self.is_gemm:
            self.p = gs.gemm_problem(w.dtype, w.M, w.N, w.K, w.transA, w.transB, w.batch, out_dtype)
            self.a, self.b = gs.to_device(w.A, w.dtype), gs.to_device(w.B, w.dtype)
            self.out = gs.empty_device((w.batch, w.M, w.N) if w.batch > 1 else (w.M, w.N), out_dtype)
        else:
            self.p = gs.conv_problem(w.dtype, w.n, w.c, w.h, w.w, w.k, w.r, w.s, w.stride, w.pad, out_dtype)
            self.a, self.b = gs.to_device(w.I, w.dtype), gs.to_device(w.W, w.dtype)
            self.out = gs.empty_device((w.n, w.k, w.p, w.q), out_dtype)
        t0 = time.perf_counter()
        self.sched = gs.construct(self.p, seed=0, opts=opts)
        self.construct_s = time.perf_counter() - t0
        self.ws = gs.gemm_workspace(self.p, self.sched) if self.is_gemm else gs.conv_workspace(self.p, self.sched)
        self.sets = [(self.a, self.b, self.out)]
        torch.cuda.synchronize()

    def launch(self, which=0):
        gs, w = self.gs, self.w
        a, b, out = self.sets[which]
        if not self.is_gemm:
            gs.conv2d(self.p, a, b, out, self.sched, self.ws)
        elif w.batch > 1:
            gs.bmm(self.p, a, b, out, 1.0, 0.0, self.sched, workspace=self.ws)
        else:
            gs.gemm(self.p, a, b, out, 1.0, 0.0, self.sched, workspace=self.ws)

    def time_cold_ms(self, launches=20):
        """Average launch duration when every launch works on another copy of the operands, the
        copies together larger than the Infinity Cache, so inputs come from HBM."""
        import torch
        per_set = sum(t.numel() * t.element_size() for t in self.sets[0])
        n_sets = max(2, -(-COLD_BYTES // per_set))
        while len(self.sets) < n_sets:
            self.sets.append((self.a.clone(), self.b.clone(), torch.empty_like(self.out)))
        for i in range(n_sets):
            self.launch(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(launches):
            self.launch(i % n_sets)
        e1.record()
        torch.cuda.synchronize()
        del self.sets[1:]
        return e0.elapsed_time(e1) / launches, n_sets

    def time_median_ms(self, batches=5, min_launches=50, settle_ms=25.0, batch_ms=4.0, max_rounds=4, steady_pct=2.0):
        """The protocol of every row: launches that keep the chip busy for settle_ms (the shader clock
        needs tens of milliseconds of load to settle after an idle period), then the median over
        `batches` event-bracketed batches of at least `min_launches` launches (more for short kernels:
        a batch lasts about batch_ms).  The first few hundred launches of a kernel on fresh buffers run up
        to 20 % slower than the steady state whatever the clock does (a first measurement of the 3x3
        convolution reads 17.8 us, every later one 15.0), so the measurement is repeated, at least twice
        and at most max_rounds times, until two successive medians agree within steady_pct; the last
        one is reported."""
        import torch
        prev = None
        for rnd in range(max_rounds):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                self.launch()
            e1.record()
            torch.cuda.synchronize()
            per = max(1e-3, e0.elapsed_time(e1) / 10)
            for _ in range(int(min(3000, max(20, settle_ms / per)))):
                self.launch()
            steps = int(min(2000, max(min_launches, batch_ms / per)))
            out = []
            for _ in range(batches):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(steps):
                    self.launch()
                e1.record()
                torch.cuda.synchronize()
                out.append(e0.elapsed_time(e1) / steps)
            med = sorted(out)[len(out) // 2]
            if prev is not None and abs(med - prev) <= steady_pct * 0.01 * prev:
                break
            prev = med
        self.protocol = {"batches": batches, "launches_per_batch": steps, "spread_pct": 100.0 * (max(out) - min(out)) / min(out),
                         "rounds": rnd + 1}
        return med

    def time_ms(self, steps, warmup):
        """Average launch duration from HIP events recorded on the launch stream."""
        import torch
        for _ in range(warmup):
            self.launch()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            self.launch()
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        return e0.elapsed_time(e1) / steps, wall_ms

    def parity(self, samples=512):
        """Relative Frobenius error against the oracle on sampled output coordinates."""
        import torch
        from oracle import ops
        from paper_2502_11407_amd import inputs
        w = self.w
        self.launch()
        torch.cuda.synchronize()
        if self.is_gemm:
            co = inputs.sample_indices(7, (w.batch, w.M, w.N), samples)
            want = ops.bmm_at(w.A, w.B, w.dtype, co, transA=w.transA, transB=w.transB)
            out = self.out if w.batch > 1 else self.out[None]
            idx = torch.from_numpy(co).cuda()
            got = out[idx[:, 0], idx[:, 1], idx[:, 2]]
        else:
            co = inputs.sample_indices(7, (w.n, w.k, w.p, w.q), samples)
            want = ops.conv2d_at(w.I, w.W, w.dtype, co, stride=w.stride, pad=w.pad)
            idx = torch.from_numpy(co).cuda()
            got = self.out[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]]
        return ops.rel_frobenius(got.double().cpu().numpy(), want)


def mfma_ceiling(gs, inputs, dtype, iters=20000):
    """TFLOP/s of a kernel of nothing but dense MFMAs whose operands are drawn like the headline's
    inputs (uniform [-1, 1)): the rate the chip's power limit allows for such values."""
    import torch
    from paper_2502_11407_amd import probe
    vals = inputs.uniform_pm1(99, (128 * 1024,), dtype)                         # 256 KiB of operand fragments
    ops_dev = gs.to_device(vals, dtype)
    sink = torch.empty(256 * 256, dtype=torch.float32, device="cuda")
    for _ in range(3):
        probe.mfma_probe(dtype, ops_dev, sink, iters, gs.hw_mi355x().compute_units)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    probe.mfma_probe(dtype, ops_dev, sink, iters, gs.hw_mi355x().compute_units)
    e1.record()
    torch.cuda.synchronize()
    flops = gs.hw_mi355x().compute_units * 4.0 * iters * 8 * 2 * 32 * 32 * 16
    return flops / (e0.elapsed_time(e1) * 1e-3) / 1e12


def _graph_us(fn, launches=20, replays=10, warm_replays=3):
    """Microseconds per launch when `launches` calls of fn are captured in one HIP graph and the graph is replayed:
    the host's per-call cost (interpreter, binding, enqueue) is paid once at capture, so what remains is the
    device's own time per launch.  For the launches of a few microseconds the eager event timing is the host's."""
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(launches):
            fn()
    for _ in range(warm_replays):
        g.replay()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (launches * replays)


def _median_ms(fn, batches=5, min_launches=50, settle_ms=25.0, batch_ms=4.0):
    """Case.time_median_ms for a plain callable."""
    c = Case.__new__(Case)
    c.launch = lambda which=0: fn()
    return Case.time_median_ms(c, batches, min_launches, settle_ms, batch_ms)


def variant_rows(gs, inputs):
    """The benchmark shapes in their other stated forms: the 16-bit-input shapes with output in the input type
    (half the store traffic, so another roofline), and the attention scores with K^T laid out in memory."""
    import torch
    cfgs = inputs.all_configs()
    todo = [(cfgs[n], "f16") for n in ("cfg3_up", "cfg3_down", "cfg4", "cfg5_3x3", "cfg5_1x1s2")]
    todo.append((inputs.config4_bmm_scores(materialised_kt=True), "f32"))
    rows = []
    for wl, out_dtype in todo:
        c = Case(gs, inputs, wl, out_dtype=out_dtype)
        m = c.time_median_ms()
        nbytes = _algorithmic_bytes(wl, inputs, out_dtype)
        tf = wl.flops / (m * 1e-3) / 1e12
        ceiling = min(PEAK_TFLOPS[wl.dtype], wl.flops / nbytes * HBM_GBS / 1e3)
        rows.append({"workload": wl.name, "out_dtype": out_dtype, "us": m * 1e3, "tflops": tf,
                     "algorithmic_GBs": nbytes / (m * 1e-3) / 1e9, "roofline_ceiling_tflops": ceiling,
                     "pct_of_roofline_ceiling": 100.0 * tf / ceiling, "kernel_id": c.sched.kernel_id,
                     "schedule": "%dx%dx%d wave %dx%d stages %d direct %d" % (
                         c.sched.tile[0][0], c.sched.tile[1][0], c.sched.tile[2][0], c.sched.tile[0][1],
                         c.sched.tile[1][1], c.sched.stages, c.sched.direct_lds),
                     "parity_rel_frobenius_sampled": c.parity(256)})
        del c
        torch.cuda.empty_cache()
    return rows


def deep_k_rows(gs, inputs):
    """Contractions with few output tiles and a deep k: the constructed schedule (which splits k) beside the best
    schedule without a split."""
    import torch
    rows = []
    for i in range(len(inputs.DEEP_K_GEMMS)):
        wl = inputs.deep_k_gemm(i)
        c = Case(gs, inputs, wl)
        m = c.time_median_ms()
        c1 = Case(gs, inputs, wl, opts=gs.ConstructOpts(0, 0, 0, 0, 0, 0, 1, 0))
        m1 = c1.time_median_ms(batches=3, min_launches=20)
        rows.append({"workload": wl.name, "us": m * 1e3, "tflops": wl.flops / (m * 1e-3) / 1e12,
                     "kernel_id": c.sched.kernel_id, "split_k": c.sched.split_k, "predicted_us": c.sched.predicted_us,
                     "workspace_MB": gs.workspace_bytes(c.p, c.sched) / 1e6,
                     "unsplit_us": m1 * 1e3, "unsplit_kernel_id": c1.sched.kernel_id,
                     "parity_rel_frobenius_sampled": c.parity(128)})
        del c, c1, wl
        torch.cuda.empty_cache()
    return rows


def stream_k_rows(gs, inputs):
    """The two GPT-2 shapes fill the 256 compute units 1.5 and 0.375 times with 256x256 tiles.  The split-k plan of
    this library is the hybrid form of stream-K for such counts: whole rounds run one tile per workgroup, the tiles of
    the partly filled last round are cut along k into equal parts that exchange partial sums.  Rows: every 256x256
    instance with that plan forced (2 to 4 parts) beside the constructed, unsplit schedule."""
    import torch
    rows = []
    cfgs = inputs.all_configs()
    for name in ("cfg3_up", "cfg3_down"):
        wl = cfgs[name]
        c = Case(gs, inputs, wl)
        base_ms = c.time_median_ms(batches=3)
        row = {"workload": wl.name, "constructed": {"kernel_id": c.sched.kernel_id, "split_k": c.sched.split_k, "us": base_ms * 1e3},
               "forced": []}
        for idx in range(gs.num_instances()):
            s = gs.instance_schedule(idx, c.p)
            if s is None or (s.tile[0][0], s.tile[1][0]) != (256, 256) or (s.direct_lds and wl.K % s.tile[2][0]):
                continue
            for split in (2, 3, 4):
                s.split_k = split
                if gs.workspace_bytes(c.p, s) == 0:
                    continue
                c.sched, c.ws = s, gs.gemm_workspace(c.p, s)
                ms = c.time_median_ms(batches=3, min_launches=20)
                row["forced"].append({"kernel_id": idx, "split_k": split, "us": ms * 1e3, "predicted_us": gs.predict_us(s, c.p),
                                      "workspace_MB": gs.workspace_bytes(c.p, s) / 1e6})
        row["forced"].sort(key=lambda r: r["us"])
        row["forced"] = row["forced"][:6]
        rows.append(row)
        del c
        torch.cuda.empty_cache()
    return rows


def operator_table_rows(gs, inputs):
    """The other shapes of the paper's operator table: Conv2d C1-C3 (constructed schedules), GEMV V1-V3 and
    AvgPooling2d P1-P3 (streaming kernels, judged against HBM bandwidth)."""
    import torch
    from oracle import ops
    rows = []
    for i in range(len(inputs.PAPER_CONVS)):
        wl = inputs.paper_conv(i)
        c = Case(gs, inputs, wl)
        m = c.time_median_ms()
        nbytes = _algorithmic_bytes(wl, inputs)
        tf = wl.flops / (m * 1e-3) / 1e12
        ceiling = min(PEAK_TFLOPS[wl.dtype], wl.flops / nbytes * HBM_GBS / 1e3)
        rows.append({"workload": wl.name, "us": m * 1e3, "tflops": tf, "algorithmic_GBs": nbytes / (m * 1e-3) / 1e9,
                     "pct_of_roofline_ceiling": 100.0 * tf / ceiling, "kernel_id": c.sched.kernel_id,
                     "parity_rel_frobenius_sampled": c.parity(128)})
        del c, wl
        torch.cuda.empty_cache()
    for i, (M, N) in enumerate(inputs.GEMV_SHAPES):
        A, x = inputs.gemv_workload(i)
        dA, dx = gs.to_device(A, "f16"), gs.to_device(x, "f16")
        y = torch.empty(M, dtype=torch.float32, device="cuda")
        m = _median_ms(lambda: gs.gemv("f16", dA, dx, y))
        in_graph = _graph_us(lambda: gs.gemv("f16", dA, dx, y))
        nbytes = 2 * (M * N + N) + 4 * M
        sel = inputs.sample_indices(7, (M,), 64)[:, 0]
        err = ops.rel_frobenius(gs.to_host_f64(y)[sel], ops.gemv(np.ascontiguousarray(A[sel]), x, "f16"))
        rows.append({"workload": f"gemv_{M}x{N}_f16", "us": m * 1e3, "us_in_graph": in_graph,
                     "GBs_in_graph": nbytes / (in_graph * 1e-6) / 1e9, "tflops": 2.0 * M * N / (m * 1e-3) / 1e12,
                     "algorithmic_GBs": nbytes / (m * 1e-3) / 1e9, "pct_of_hbm_peak": 100.0 * nbytes / (m * 1e-3) / 1e9 / HBM_GBS,
                     "parity_rel_frobenius_sampled": err})
        del dA, dx, A
        torch.cuda.empty_cache()
    for i in range(len(inputs.POOL_SHAPES)):
        I, f, stride = inputs.pool_workload(i)
        shape = ops.pool_out_shape(*I.shape, f, stride)
        dI = gs.to_device(I, "f16")
        O = gs.empty_device(shape)
        m = _median_ms(lambda: gs.avgpool2d("f16", dI, O, f, stride))
        in_graph = _graph_us(lambda: gs.avgpool2d("f16", dI, O, f, stride))
        nbytes = 2 * I.size + 4 * int(np.prod(shape))
        co = inputs.sample_indices(7, shape, 256)
        idx = torch.from_numpy(co).cuda()
        got = O[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].double().cpu().numpy()
        rows.append({"workload": "avgpool_%dx%dx%dx%d_f%d_s%d_f16" % (*I.shape, f, stride), "us": m * 1e3,
                     "us_in_graph": in_graph, "GBs_in_graph": nbytes / (in_graph * 1e-6) / 1e9,
                     "algorithmic_GBs": nbytes / (m * 1e-3) / 1e9, "pct_of_hbm_peak": 100.0 * nbytes / (m * 1e-3) / 1e9 / HBM_GBS,
                     "parity_rel_frobenius_sampled": ops.rel_frobenius(got, ops.avgpool2d_at(I, "f16", co, f, stride))})
        del dI, O, I
        torch.cuda.empty_cache()
    return rows


def ablation(gs, inputs):
    """Variants of the walk on this hardware (the design of the paper's ablation, Table VI): each
    constructs a schedule for three shapes; the schedule is then timed."""
    import torch
    variants = [("full", None),
                ("no_vthread", gs.ConstructOpts(0, 0, 0, 0, 0, 1)),
                ("printed_keep_probability", gs.ConstructOpts(0, 0, 0, 1, 0, 0)),
                ("footprint_ratio_inverted", gs.ConstructOpts(0, 0, 0, 0, 1, 0)),
                ("one_walk", gs.ConstructOpts(0, 0, 1, 0, 0, 0)),
                ("greedy_single_path", gs.ConstructOpts(0, 0, 1, 0, 0, 0, 0, 1)),
                ("T0_1_as_literal", gs.ConstructOpts(1.0, 2.0 ** -100, 0, 0, 0, 0))]
    out = []
    cfgs = inputs.all_configs()
    for name in ("cfg2", "cfg3_up", "cfg5_3x3"):
        wl = cfgs[name]
        row = {"workload": wl.name}
        for vname, opts in variants:
            try:
                c = Case(gs, inputs, wl, opts)
            except gs.GensorError as e:
                row[vname] = {"error": str(e)}
                continue
            m = c.time_median_ms(batches=3)
            row[vname] = {"kernel_id": c.sched.kernel_id, "vthread": [c.sched.vthread[0], c.sched.vthread[1]], "us": m * 1e3, "tflops": wl.flops / (m * 1e-3) / 1e12,
                          "predicted_us": c.sched.predicted_us, "states_scored": c.sched.states_scored,
                          "construct_s": c.construct_s}
            del c
            torch.cuda.empty_cache()
        out.append(row)
    return out


def cpu_baseline(w):
    """The oracle as it stands on a bounded slice (leading rows of A) of the headline GEMM."""
    from oracle import ops
    rows = 2 * ops.num_threads()
    t0 = time.perf_counter()
    ops.gemm(w.A[:rows], w.B, w.dtype, transA=w.transA, transB=w.transB)
    dt = time.perf_counter() - t0
    target = 12.0
    rows2 = int(min(w.M, max(rows, rows * target / max(dt, 1e-3))))
    rows2 = max(ops.num_threads(), rows2 - rows2 % ops.num_threads())
    t0 = time.perf_counter()
    ops.gemm(w.A[:rows2], w.B, w.dtype, transA=w.transA, transB=w.transB)
    dt = time.perf_counter() - t0
    flops = 2.0 * rows2 * w.N * w.K
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": ops.num_threads(), "kind": "oracle",
            "sample": f"first {rows2} of {w.M} rows of C (all {w.N} columns, full K={w.K}), {dt:.1f} s"}


def _row(c, wl, m, inputs, out_dtype="f32"):
    nbytes = _algorithmic_bytes(wl, inputs, out_dtype)
    tf = wl.flops / (m * 1e-3) / 1e12
    ceiling = min(PEAK_TFLOPS[wl.dtype], wl.flops / nbytes * HBM_GBS / 1e3)
    return {"workload": wl.name, "dtype": wl.dtype, "us": m * 1e3, "tflops": tf,
            "pct_of_mfma_peak": 100.0 * tf / PEAK_TFLOPS[wl.dtype], "algorithmic_GBs": nbytes / (m * 1e-3) / 1e9,
            "pct_of_hbm_peak": 100.0 * nbytes / (m * 1e-3) / 1e9 / HBM_GBS, "roofline_ceiling_tflops": ceiling,
            "pct_of_roofline_ceiling": 100.0 * tf / ceiling, "construct_s": c.construct_s, "kernel_id": c.sched.kernel_id,
            "schedule": "%dx%dx%d wave %dx%d V %d,%d stages %d direct %d split %d" % (
                c.sched.tile[0][0], c.sched.tile[1][0], c.sched.tile[2][0], c.sched.tile[0][1], c.sched.tile[1][1],
                c.sched.vthread[0], c.sched.vthread[1], c.sched.stages, c.sched.direct_lds, c.sched.split_k),
            "protocol": c.protocol}


def _compact(name, r):
    g = lambda x, n: None if x is None else float(("%." + str(n) + "g") % x)
    return {"w": name, "us": g(r["us"], 4), "tf": g(r["tflops"], 4), "pk": g(r["pct_of_mfma_peak"], 3),
            "ceil": g(r["pct_of_roofline_ceiling"], 3), "gbs": g(r["algorithmic_GBs"], 4), "id": r["kernel_id"],
            "cs": g(r["construct_s"], 2), "err": g(r.get("parity_rel_frobenius_sampled"), 2)}


def _progress(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=300,
                    help="untimed launches first; the shader clock needs tens of milliseconds of load to settle")
    ap.add_argument("--only-headline", action="store_true", help="skip the other operator shapes and the CPU legs")
    ap.add_argument("--no-settle", action="store_true",
                    help="skip the launches that settle the shader clock ahead of the warm-up (hardware-counter passes)")
    ap.add_argument("--launch-only", default="",
                    help="comma-separated workload names (cfg1..cfg5_1x1s2, u0..u4, d0..d3): construct, launch each "
                         "20 times and exit -- what a hardware-counter pass over one of the other shapes runs; "
                         "name:no_vthread constructs without setVThread")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain 256 MiB device copy, the known-size reference for HBM byte counters")
    ap.add_argument("--details", default=os.path.join(ROOT, "gpurun_out", "bench_details.json"),
                    help="file that receives the long sections (the stdout line stays short)")
    ap.add_argument("--sections", default="operators,unbalanced,deep_k,stream_k,variants,operator_table,ablation,cpu",
                    help="comma-separated sections to run besides the headline")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (single-GPU operators, "
              "no collectives)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    from paper_2502_11407_amd import binding as gs, inputs

    if args.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")     # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.launch_only:
        for item in args.launch_only.split(","):
            name, _, variant = item.partition(":")
            wl = (inputs.unbalanced_gemm(int(name[1:])) if name[0] == "u" else
                  inputs.deep_k_gemm(int(name[1:])) if name[0] == "d" else
                  inputs.paper_conv(int(name[1:]) - 1) if name[0] == "C" else inputs.all_configs()[name])
            c = Case(gs, inputs, wl, gs.ConstructOpts(0, 0, 0, 0, 0, 1) if variant == "no_vthread" else None)
            for _ in range(20):
                c.launch()
            torch.cuda.synchronize()
            print(item, "kernel", c.sched.kernel_id, "vthread", c.sched.vthread[0], c.sched.vthread[1], "split_k", c.sched.split_k)
            del c
            torch.cuda.empty_cache()
        return

    sections = set() if args.only_headline else set(x for x in args.sections.split(",") if x)
    w = inputs.config2_gemm_f16()
    head = Case(gs, inputs, w)
    # the shader clock needs tens of milliseconds of load to settle after an idle period (the first ~100 launches run
    # 15 % slow, and the launch time keeps falling by another 2 % over the next two thousand): whatever warm-up count
    # was asked for, 2000 launches (a quarter of a second) precede the timed ones, the extra ones reported
    settle = 0 if args.no_settle else max(0, 2000 - args.warmup)
    for _ in range(settle):
        head.launch()
    ms, wall_ms = head.time_ms(args.steps, args.warmup)
    tflops = w.flops / (ms * 1e-3) / 1e12
    peak = PEAK_TFLOPS[w.dtype]
    sd = head.sched.describe()
    traffic = MEASURED_TRAFFIC_BYTES.get(((sd["tile_m"][0], sd["tile_n"][0], sd["tile_k"][0]),
                                          (sd["tile_m"][1], sd["tile_n"][1]), sd["direct_lds"]))
    _progress("headline %.1f us over %d launches (kernel %d)" % (ms * 1e3, args.steps, head.sched.kernel_id))
    line = {
        "metric": "TFLOP/s and % of MFMA peak per operator on 1 MI355X; construction time (s)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "GEMM fp16 in / fp32 accumulate+out, M=N=K=4096, A row-major, B column-major, "
                               "uniform[-1,1) (configs[1])",
                   "kernel_id": head.sched.kernel_id,
                   "schedule": "%dx%dx%d wave %dx%d V %d,%d stages %d direct %d" % (
                       sd["tile_m"][0], sd["tile_n"][0], sd["tile_k"][0], sd["tile_m"][1], sd["tile_n"][1],
                       sd["vthread"][0], sd["vthread"][1], sd["stages"], sd["direct_lds"])},
        "pct_of_mfma_peak": 100.0 * tflops / peak,
        "construct_s": head.construct_s,
        "clock_settle_launches_before_warmup": settle,
        "roofline": {"bound": "mfma", "achieved": tflops, "peak": peak, "unit": "TFLOP/s",
                     "frac": tflops / peak, "traffic": traffic,
                     "traffic_source": TRAFFIC_SOURCE if traffic is not None else None},
    }
    details = {"headline_schedule": sd, "wall_ms_per_step": wall_ms}
    prop = torch.cuda.get_device_properties(0)
    ghz = prop.clock_rate / 1e6 if hasattr(prop, "clock_rate") else 2.4
    details["device"] = {
        "name": prop.name, "compute_units": prop.multi_processor_count, "clock_ghz": ghz,
        # one 32x32x16 16-bit MFMA (32768 flop) per SIMD every 32 cycles, one 32x32x2 fp32 MFMA (4096 flop) every 64
        "derived_peak_tflops": {"f16_bf16_mfma": prop.multi_processor_count * 4 * 1024 * ghz / 1e3,
                                "f32_mfma": prop.multi_processor_count * 4 * 64 * ghz / 1e3},
        "published_peaks_used": {"f16_bf16_mfma_tflops": PEAK_TFLOPS["f16"], "f32_mfma_tflops": PEAK_TFLOPS["f32"], "hbm_GBs": HBM_GBS},
        "flop_convention": "GEMM 2MNK, BMM 2BMNK, conv 2 N K P Q C R S (padded taps counted)"}
    if "operators" in sections:
        # the headline by the protocol of the other rows, and one launch at a time (graph replay: no overlap between the
        # tail of one launch and the head of the next)
        m = head.time_median_ms()
        hrow = _row(head, w, m, inputs)
        hrow["parity_rel_frobenius_sampled"] = head.parity()
        cold_ms, cold_sets = head.time_cold_ms()
        hrow["cold_us"] = cold_ms * 1e3
        hrow["us_in_graph"] = _graph_us(head.launch, launches=20, replays=25, warm_replays=15)
        ceil_tf = mfma_ceiling(gs, inputs, w.dtype)
        details["mfma_only_kernel_same_operand_distribution"] = {
            "tflops": ceil_tf, "headline_frac_of_it": hrow["tflops"] / ceil_tf,
            "note": "a kernel of nothing but fp16 MFMAs on uniform[-1,1) operands, timed in this run: what the chip's power "
                    "limit allows for such values (context; the roofline above is against the published peak)"}
        rows, compact = [], []
        for name, wl in inputs.all_configs().items():
            if name == "cfg2":
                r = hrow
            else:
                c = Case(gs, inputs, wl)
                m = c.time_median_ms()
                r = _row(c, wl, m, inputs)
                cold, _ = c.time_cold_ms()
                r["cold_us"] = cold * 1e3
                r["us_in_graph"] = _graph_us(c.launch)
                r["parity_rel_frobenius_sampled"] = c.parity(256)
                del c
                torch.cuda.empty_cache()
            rows.append(r)
            compact.append(_compact(name, r))
            _progress("%s %.1f us, %.1f %% of its ceiling, kernel %d" % (name, r["us"], r["pct_of_roofline_ceiling"], r["kernel_id"]))
        details["operators"] = rows
        line["operators"] = compact
        line["protocol"] = "rows: clock settle, then median of 5 batches of >=50 launches, repeated (2-4x) until two medians agree within 2 %; value: the --steps launches"
    if "unbalanced" in sections:
        # the paper's GEMM shapes with unbalanced dimensions (next in line after the five configurations)
        nxt = []
        for i in range(len(inputs.UNBALANCED_GEMMS)):
            wl = inputs.unbalanced_gemm(i)
            c = Case(gs, inputs, wl)
            m = c.time_median_ms(min_launches=50 if wl.flops < 2e11 else 10)
            r = _row(c, wl, m, inputs)
            r["parity_rel_frobenius_sampled"] = c.parity(128)
            nxt.append(r)
            _progress("%s %.1f us kernel %d" % (wl.name, r["us"], r["kernel_id"]))
            del c, wl
            torch.cuda.empty_cache()
        details["unbalanced_gemms"] = nxt
    if "deep_k" in sections:
        details["deep_k_gemms"] = deep_k_rows(gs, inputs)
        _progress("deep-k rows done")
    if "stream_k" in sections:
        details["stream_k_hybrid"] = stream_k_rows(gs, inputs)
        _progress("stream-k rows done")
    if "variants" in sections:
        details["variants"] = variant_rows(gs, inputs)
        _progress("output-type variants done")
    if "operator_table" in sections:
        details["operator_table"] = operator_table_rows(gs, inputs)
        _progress("operator table done")
    if "ablation" in sections:
        details["ablation"] = ablation(gs, inputs)
        line["ablation"] = [{"w": row["workload"], **{k: [v.get("kernel_id"), None if "us" not in v else float("%.4g" % v["us"])]
                                                     for k, v in row.items() if isinstance(v, dict)}} for row in details["ablation"]]
        _progress("ablation done")
    if "cpu" in sections:
        line["cpu_baseline"] = cpu_baseline(w)
    line["paper_context"] = "paper (RTX 4090, precision not stated): GEMM 45.2 TFLOP/s, Conv2d C1 34.54 TFLOP/s, construction 'a few seconds'"
    try:
        if not sections:
            raise OSError("no sections were run")
        os.makedirs(os.path.dirname(os.path.abspath(args.details)), exist_ok=True)
        with open(args.details, "w") as f:
            json.dump({"line": line, "details": details}, f, indent=1)
        line["details_file"] = os.path.relpath(args.details, ROOT)
    except OSError as e:
        line["details_file"] = None if not sections else "not written: %s" % e
    print(json.dumps(line))


if __name__ == "__main__":
    main()

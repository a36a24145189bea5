#!/usr/bin/env python3
"""Benchmark of the fused Chebyshev-KAN forward + backward pass on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input:
the stack's forward call, then its backward call (dx and dC of every layer),
enqueued through the C ABI on one stream.

Prints ONE JSON line.  The headline workload is the largest configuration
(c5, one 1024 -> 1024 layer of degree 8 on 16384 rows: the compute-bound case the
fp32-MFMA target is stated on); `value` is its rows per second, inputs resident
in HBM.  The tabular stack (c2: the memory-bound target) runs in the same process
and its full result is nested under `tabular_c2`; the speech- and audio-shaped stacks
follow under `speech_c3` and `audio_c4` (without the cold pass and the CPU baseline).

`roofline` describes the dominant kernel OF THE TIMED STEPS: the library brackets
every kernel it launches with two event records on the launch stream
(chebykan_trace_begin/end), so each kernel's duration comes from the timed region
itself; `kernels` lists all of them, keyed by kernel name and grid.  `traffic` is
read from profiles/<workload>_counters.md (rocprofv3 FETCH_SIZE / WRITE_SIZE of
the same step sequence, scaled by a plain copy of known size); null when that file
does not list the kernel at this grid.  `cpu_baseline` is the fp64 CPU oracle
timed on this machine's host cores on a bounded row sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F32_TFLOPS = 157.3     # MI355X dense fp32 matrix peak
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E peak
HEADLINE = "c5"
TABULAR = "c2"
OP_FORWARD, OP_DX, OP_DC, OP_SUM = 1, 2, 4, 8


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=HEADLINE, choices=["c1", "c2", "c3", "c4", "c5", "p1", "p2", "p3"])
    ap.add_argument("--no-tabular", action="store_true",
                    help="do not run the tabular stack (c2) and the two wide stacks (c3, c4) beside the headline workload")
    ap.add_argument("--tabular-steps", type=int, default=300, help="timed steps of the nested tabular run")
    ap.add_argument("--stack-steps", type=int, default=40, help="timed steps of the nested speech- and audio-shaped runs")
    ap.add_argument("--rotate", type=int, default=4,
                    help="number of distinct (x, dy) input sets cycled through, so inputs are not cache-resident")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--no-cold", action="store_true",
                    help="skip the cold pass (whole buffer sets rotated through at least 512 MB)")
    ap.add_argument("--trace-timed", default="auto", choices=["auto", "on", "off"],
                    help="per-kernel event records inside the timed steps: on, off (a second pass over the same "
                         "steps is traced instead), or auto = on when a step takes at least five milliseconds "
                         "(two records per kernel cost a few microseconds each: under 0.5 % of such a step)")
    ap.add_argument("--family", type=int, default=0, help="kernel family override (0 auto)")
    ap.add_argument("--basis", default="exact", choices=["exact", "lut", "lut2", "legendre", "hermite", "fourier"],
                    help="exact = Chebyshev recurrences (default); lut = the paper's table-interpolated variant "
                         "(Sec. 4.2); lut2 = the same with the auxiliary derivative table; legendre / hermite / "
                         "fourier = the other bases of Sec. 2.3 on the same kernels")
    ap.add_argument("--lut-size", type=int, default=1025, help="table samples for --basis lut")
    ap.add_argument("--graph", action="store_true",
                    help="capture the steps (one per rotated input set) in a HIP graph and time its replays; the "
                         "first replay is checked against the eager result")
    ap.add_argument("--probe", type=int, default=0,
                    help="counter-collection mode for rocprofv3 --pmc: one plain 256 MiB device copy (the "
                         "calibration kernel of known size), then this many steps exactly as the timed region "
                         "issues them, then exit")
    ap.add_argument("--probe-calls", action="store_true",
                    help="with --probe: issue every layer's forward, dx-only and dC-only call on its own (the calls of "
                         "the `calls` list) instead of the stack step, so the single-layer kernels show up too")
    return ap.parse_args()


class Stack:
    """Device buffers and the launch sequence of one workload."""

    def __init__(self, w, rotate, torch, binding, wl, lut=None, kind=0, dlut=None):
        self.w, self.torch, self.binding = w, torch, binding
        self.kind = kind        # 0 Chebyshev, 1 Legendre, 2 Hermite, 3 Fourier
        self.lut = lut          # device table [degree+1, samples] or None for the exact basis
        self.dlut = dlut        # device derivative table (same shape) or None
        B = w.batch
        self.B = B
        self.layers = w.layers
        self.d = w.degree
        x0, Cs, dy_last = wl.workload_inputs(w)
        self.x0_sets = [torch.from_numpy(x0).cuda()]
        self.dy_sets = [torch.from_numpy(dy_last).cuda()]
        for r in range(1, rotate):
            self.x0_sets.append(torch.from_numpy(
                wl.make_x(B, w.widths[0], wl.tensor_seed(w.index, 0, "x") + 100000 * r, w.x_mean, w.x_std)).cuda())
            self.dy_sets.append(torch.from_numpy(
                wl.make_dy(B, w.widths[-1], wl.tensor_seed(w.index, len(self.layers) - 1, "dy") + 100000 * r)).cuda())
        self.C = [torch.from_numpy(c).cuda() for c in Cs]
        self.y = [torch.empty((B, o), device="cuda") for (_, o) in self.layers]
        self.dx = [torch.empty((B, i), device="cuda") for (i, _) in self.layers]
        self.dC = [torch.empty_like(c) for c in self.C]
        self.ws = [binding.alloc_workspace(B, i, o, self.d) for (i, o) in self.layers]
        self.stream = torch.cuda.Stream()
        self.stack_ws = binding.alloc_stack_workspace(B, list(w.widths), self.d)

    def _fwd(self, xin, l, s):
        b = self.binding
        if self.kind:
            b.chebykan_forward_basis(self.kind, xin, self.C[l], self.y[l], self.ws[l], s)
        elif self.lut is None:
            b.chebykan_forward(xin, self.C[l], self.y[l], self.ws[l], s)
        else:
            b.chebykan_forward_lut(xin, self.C[l], self.lut, self.y[l], self.ws[l], s)

    def _bwd(self, xin, l, dy, dx, dC, s):
        b = self.binding
        if self.kind:
            b.chebykan_backward_basis(self.kind, xin, self.C[l], dy, dx, dC, self.ws[l], s)
        elif self.lut is None:
            b.chebykan_backward(xin, self.C[l], dy, dx, dC, self.ws[l], s)
        elif self.dlut is None:
            b.chebykan_backward_lut(xin, self.C[l], dy, self.lut, dx, dC, self.ws[l], s)
        else:
            b.chebykan_backward_lut2(xin, self.C[l], dy, self.lut, self.dlut, dx, dC, self.ws[l], s)

    def calls(self, step):
        """One step as single-layer ABI calls, in order: (tag, layer, thunk)."""
        n = len(self.layers)
        x0 = self.x0_sets[step % len(self.x0_sets)]
        dyl = self.dy_sets[step % len(self.dy_sets)]
        s = self.stream
        out = []
        for l in range(n):
            xin = x0 if l == 0 else self.y[l - 1]
            out.append(("fwd", l, lambda l=l, xin=xin: self._fwd(xin, l, s)))
        for l in reversed(range(n)):
            xin = x0 if l == 0 else self.y[l - 1]
            dy = dyl if l == n - 1 else self.dx[l + 1]
            out.append(("dx", l, lambda l=l, xin=xin, dy=dy: self._bwd(xin, l, dy, self.dx[l], None, s)))
            out.append(("dC", l, lambda l=l, xin=xin, dy=dy: self._bwd(xin, l, dy, None, self.dC[l], s)))
        return out

    def step(self, k):
        """One step as a user would issue it: the stack's forward call, then its backward call."""
        self.step_forward(k)
        self.step_backward(k)

    def step_forward(self, step):
        b, n, s = self.binding, len(self.layers), self.stream
        x0 = self.x0_sets[step % len(self.x0_sets)]
        if self.lut is None and not self.kind:
            b.chebykan_stack_forward(self.C, [x0] + self.y, self.stack_ws, s)
        else:
            for l in range(n):
                xin = x0 if l == 0 else self.y[l - 1]
                self._fwd(xin, l, s)

    def step_backward(self, step):
        n, s = len(self.layers), self.stream
        x0 = self.x0_sets[step % len(self.x0_sets)]
        dyl = self.dy_sets[step % len(self.dy_sets)]
        if self.lut is None and not self.kind:
            self.binding.chebykan_stack_backward(self.C, [x0] + self.y[:-1], self.dx + [dyl], self.dC, self.stack_ws, s)
            return
        for l in reversed(range(n)):
            xin = x0 if l == 0 else self.y[l - 1]
            dy = dyl if l == n - 1 else self.dx[l + 1]
            self._bwd(xin, l, dy, self.dx[l], self.dC[l], s)


def call_work(tag, B, I, O, d):
    """Algorithmic flops and HBM bytes of one call (fp32)."""
    K = d + 1
    if tag == "fwd":
        return 2 * B * I * O * K, 4 * (B * I + I * O * K + B * O)
    if tag == "dx":
        return 2 * B * I * O * d, 4 * (B * I + I * O * K + B * O + B * I)
    return 2 * B * I * O * K, 4 * (B * I + B * O + I * O * K)


def kernel_work(w, layer, ops):
    """Algorithmic flops and HBM bytes of the work a traced kernel stands for: the outputs in `ops` of
    `layer` (-1: of every layer).  A kernel that only adds partial results does no algorithmic work of
    its own.  A kernel that yields both gradients of a layer reads x, C and dy once."""
    if ops & OP_SUM:
        return 0, 0
    B, d = w.batch, w.degree
    K = d + 1
    fl = by = 0
    for l, (I, O) in enumerate(w.layers):
        if layer not in (-1, l):
            continue
        if ops & OP_FORWARD:
            f, b = call_work("fwd", B, I, O, d)
            fl, by = fl + f, by + b
        if (ops & OP_DX) and (ops & OP_DC):
            fl += 2 * B * I * O * (K + d)
            by += 4 * (B * I + I * O * K + B * O + B * I + I * O * K)
        elif ops & OP_DX:
            f, b = call_work("dx", B, I, O, d)
            fl, by = fl + f, by + b
        elif ops & OP_DC:
            f, b = call_work("dC", B, I, O, d)
            fl, by = fl + f, by + b
    return fl, by


def read_traffic(workload):
    """{(kernel name, grid 'XxY'): HBM bytes per launch} from profiles/<workload>_counters.md."""
    path = os.path.join(ROOT, "profiles", "%s_counters.md" % workload)
    out = {}
    if not os.path.exists(path):
        return out
    cols = None
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if line.startswith("| kernel"):
            cols = cells
        elif cols and line.startswith("| `") and len(cells) == len(cols):
            row = dict(zip(cols, cells))
            try:
                out[(row["kernel"].strip("`"), row["grid"].replace(" ", ""))] = \
                    (float(row["fetch MB"]) + float(row["write MB"])) * 1e6
            except (KeyError, ValueError):
                pass
    return out


def lookup_traffic(traffic, name, grid):
    """Counter bytes of a kernel at a grid.  The profiler spells out defaulted template arguments that the
    library's own kernel names leave off, so a row also matches when it is the only one of that kernel
    template at that grid."""
    if (name, grid) in traffic:
        return traffic[(name, grid)]
    base = name.split("<")[0]
    hits = [v for (n, g), v in traffic.items() if g == grid and n.split("<")[0] == base]
    return hits[0] if len(hits) == 1 else None


def summarise_kernels(recs, steps, w, traffic):
    """Per (kernel, grid): launches per step, average duration over the traced steps, algorithmic work, rates."""
    agg = {}
    order = []
    shares = {}
    for name, grid, block, layer, ops, share, layer2, ops2, us in recs:
        key = (name, "%dx%d" % (grid[0], grid[1]), layer, ops)
        shares[key] = (share, layer2, ops2)
        if key not in agg:
            agg[key] = []
            order.append(key)
        agg[key].append(us)
    total_us = sum(sum(v) for v in agg.values())
    out = []
    for key in order:
        name, grid, layer, ops = key
        v = np.array(agg[key])
        share, layer2, ops2 = shares[key]
        fl, by = kernel_work(w, layer, ops)
        fl, by = int(fl * share), int(by * share)                  # two launches tiling one output range
        if ops2:                                                   # a launch that holds two operations
            fl2, by2 = kernel_work(w, layer2, ops2)
            fl, by = fl + fl2, by + by2
        avg = float(v.mean())
        row = {"kernel": name, "grid": grid, "layer": layer, "ops": ops, "launches_per_step": len(v) / steps,
               "avg_us": round(avg, 2), "min_us": round(float(v.min()), 2), "share": round(float(v.sum()) / total_us, 4),
               "flops_per_launch": fl, "algorithmic_bytes_per_launch": by,
               "tflops": round(fl / (avg * 1e-6) / 1e12, 2), "gbs": round(by / (avg * 1e-6) / 1e9, 1),
               "mfma_frac": round(fl / (avg * 1e-6) / 1e12 / PEAK_MFMA_F32_TFLOPS, 4),
               "hbm_frac": round(by / (avg * 1e-6) / 1e9 / PEAK_HBM_GBS, 4),
               "traffic_bytes_per_launch": lookup_traffic(traffic, name, grid)}
        out.append(row)
    return out, total_us / steps


def roofline_of(dom):
    """The roofline block for one summarised kernel."""
    fl, by = dom["flops_per_launch"], dom["algorithmic_bytes_per_launch"]
    t_mfma, t_hbm = fl / (PEAK_MFMA_F32_TFLOPS * 1e12), by / (PEAK_HBM_GBS * 1e9)
    if t_mfma >= t_hbm:
        roof = {"bound": "mfma", "achieved": dom["tflops"], "peak": PEAK_MFMA_F32_TFLOPS, "unit": "TFLOP/s",
                "frac": dom["mfma_frac"]}
    else:
        roof = {"bound": "hbm", "achieved": dom["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": dom["hbm_frac"]}
    roof["traffic"] = dom["traffic_bytes_per_launch"]
    roof.update({"kernel": dom["kernel"], "grid": dom["grid"], "avg_us": dom["avg_us"],
                 "launches_per_step": dom["launches_per_step"], "flops_per_launch": fl,
                 "algorithmic_bytes_per_launch": by,
                 "source": "HIP event pairs around every launch of this kernel in the timed steps"})
    return roof


def measured_peaks(torch, binding, stream):
    """What this GPU sustains on a register-only fp32 MFMA loop and on a plain 256 MiB copy."""
    sink = torch.empty(512 * 256, dtype=torch.float32, device="cuda")
    src = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(reps):
            out = fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps, out

    # 512 workgroups = one resident round of 2 per CU; 2000 trips of 32 MFMAs per wave (about 2 ms)
    t_mfma, flops = timed(lambda: binding.chebykan_calibrate_mfma(sink, 512, 2000, stream), 5)
    t_copy, nbytes = timed(lambda: binding.chebykan_calibrate_copy(dst, src, stream), 10)
    return {"mfma_f32_tflops": round(flops / t_mfma / 1e12, 1), "copy_gbs_read_plus_write": round(2 * nbytes / t_copy / 1e9, 1),
            "note": "register-only v_mfma_f32_32x32x2_f32 loop on 512 workgroups; 256 MiB device copy"}


def cold_pass(st, make_stack, torch, rounds=3):
    """Steps over whole buffer sets (inputs, activations, gradients, workspaces) rotated through at least
    512 MB, so that no step finds its tensors in the caches from the one before; event-timed on the launch
    stream.  The default timing rotates only the inputs: activations are produced and consumed inside the
    step, as in training, and may stay cache-resident between steps."""
    def tensors(s):
        out = [s.x0_sets[0], s.dy_sets[0], s.stack_ws] + s.C + s.y + s.dx + s.dC + s.ws
        return [t for t in out if t is not None]
    per_set = sum(t.numel() * t.element_size() for t in tensors(st))
    n_sets = int(min(16, max(2, -(-(512 << 20) // per_set))))
    sets = [st]
    for _ in range(n_sets - 1):
        s = make_stack()
        s.stream = st.stream
        sets.append(s)
    for s in sets:
        s.step(0)
    torch.cuda.synchronize()
    n = rounds * n_sets
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    ev[0].record(st.stream)
    for k in range(n):
        sets[k % n_sets].step(0)
        ev[k + 1].record(st.stream)
    torch.cuda.synchronize()
    ms = np.array([ev[k].elapsed_time(ev[k + 1]) for k in range(n)])
    del sets
    return {"buffer_sets": n_sets, "bytes_rotated": int(per_set * n_sets), "steps": n,
            "step_ms_median": float(np.median(ms)), "step_ms_min": float(np.min(ms))}


def cpu_baseline(w, wl, target_seconds, lut_size=0, kind=0):
    """Time the fp64 oracle on the host cores over a bounded row sample of the workload."""
    import oracle
    threads = oracle.num_threads()
    lut = oracle.lut_build(w.degree, lut_size).astype(np.float32) if lut_size else None

    def one_pass(rows):
        x0, Cs, dy_last = wl.workload_inputs(w, batch=rows)
        t0 = time.perf_counter()
        xs = [x0.astype(np.float64)]
        for C in Cs:
            if kind:
                xs.append(oracle.forward_basis(kind, xs[-1], C))
            else:
                xs.append(oracle.forward(xs[-1], C) if lut is None else oracle.forward_lut(xs[-1], C, lut))
        dy = dy_last.astype(np.float64)
        for l in reversed(range(len(Cs))):
            if kind:
                dx, _ = oracle.backward_basis(kind, xs[l], Cs[l], dy)
            elif lut is None:
                dx, _ = oracle.backward(xs[l], Cs[l], dy)
            else:
                dx, _ = oracle.backward_lut(xs[l], Cs[l], dy, lut)
            dy = dx
        return time.perf_counter() - t0

    # size the sample from a small probe: target_seconds of CPU work spread over the threads the oracle uses
    wall_budget = max(1.0, 1.5 * target_seconds / max(threads, 1))
    probe_rows = int(min(w.batch, 256))
    one_pass(probe_rows)                      # first call also loads the library
    per_row = one_pass(probe_rows) / probe_rows
    rows = int(min(w.batch, max(probe_rows, wall_budget / max(per_row, 1e-9))))
    times = [one_pass(rows)]
    # a workload the oracle finishes quickly is timed over several passes (median), up to the same budget
    while rows == w.batch and len(times) < 15 and sum(times) + times[0] < wall_budget:
        times.append(one_pass(rows))
    dt = sorted(times)[len(times) // 2]
    return {"value": rows / dt, "unit": "samples/s", "cores": threads, "kind": "oracle",
            "sample": "%d of %d rows of workload %s, full stack fwd+bwd in fp64, %.2f s wall per pass on %d threads "
                      "(median of %d passes)" % (rows, w.batch, w.name, dt, threads, len(times))}


def run_workload(name, steps, warmup, args, torch, binding, wl, brief=False):
    """Everything bench.py measures on one workload, as a dict (brief: no cold pass, no CPU baseline)."""
    w = wl.WORKLOADS[name]
    lut = dlut = None
    if args.basis in ("lut", "lut2"):
        lut = binding.chebykan_lut_build(w.degree, args.lut_size).cuda()
        if args.basis == "lut2":
            dlut = binding.chebykan_lut_build_derivative(w.degree, args.lut_size).cuda()
    kind = {"legendre": 1, "hermite": 2, "fourier": 3}.get(args.basis, 0)
    if kind == 3 and w.degree % 2:
        raise SystemExit("the Fourier basis needs an even degree; workload %s has degree %d" % (w.name, w.degree))
    st = Stack(w, max(1, args.rotate), torch, binding, wl, lut, kind, dlut)
    B = w.batch
    traffic = read_traffic(w.name) if lut is None and not kind else {}

    # ---- throughput: W warm-up steps, then exactly K timed steps
    for k in range(warmup):
        st.step(k)
    torch.cuda.synchronize()
    kernels_per_step_cap = 64
    trace_timed = False
    if args.graph:
        # one graph holds one step per rotated input set; K steps = K / sets replays (K is rounded up to that)
        sets = len(st.x0_sets)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=st.stream):
            for k in range(sets):
                st.step(k)
        graph.replay()
        torch.cuda.synchronize()
        st.step(sets - 1)          # eager result of the set the graph ended on
        torch.cuda.synchronize()
        last = [t.clone() for t in (st.y[-1], st.dx[0], st.dC[0])]
        replays = (steps + sets - 1) // sets
        steps = replays * sets
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        for a, b_ in zip(last, (st.y[-1], st.dx[0], st.dC[0])):
            if not torch.equal(a, b_):
                raise RuntimeError("graph replay differs from the eager step")
    else:
        # is a step long enough that two event records per kernel do not show?
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st.stream)
        for k in range(3):
            st.step(k)
        e1.record(st.stream)
        torch.cuda.synchronize()
        trace_timed = args.trace_timed == "on" or (args.trace_timed == "auto" and e0.elapsed_time(e1) / 3 >= 5.0)
        if trace_timed:
            binding.chebykan_trace_begin(steps * kernels_per_step_cap)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            st.step(k)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / steps

    # ---- per-kernel durations: from the timed steps when they were traced, else from the same steps again
    if trace_timed:
        traced_steps, traced_ms = steps, ms_per_step
    else:
        traced_steps = min(steps, 200)
        binding.chebykan_trace_begin(traced_steps * kernels_per_step_cap)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(traced_steps):
            st.step(k)
        torch.cuda.synchronize()
        traced_ms = (time.perf_counter() - t0) * 1e3 / traced_steps
    n_rec, dropped = binding.chebykan_trace_end()
    recs = binding.chebykan_trace_records(n_rec)
    binding.chebykan_trace_free()
    if dropped:
        raise RuntimeError("kernel timing ran out of records (%d dropped)" % dropped)
    kernels, kernel_us_per_step = summarise_kernels(recs, traced_steps, w, traffic)
    work = [r for r in kernels if not (r["ops"] & OP_SUM)] or kernels
    dom = max(work, key=lambda r: r["avg_us"] * r["launches_per_step"])
    roof = roofline_of(dom)
    roof["source"] += "" if trace_timed else " of a second, traced pass over the same steps (records inside the " \
                                              "timed steps would cost a measurable share of a step this short)"

    # ---- whole steps with events: median / min per step, forward and backward apart
    nst = min(steps, 50)
    sev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(nst)]
    for k in range(nst):
        sev[k][0].record(st.stream)
        st.step_forward(k)
        sev[k][1].record(st.stream)
        st.step_backward(k)
        sev[k][2].record(st.stream)
    torch.cuda.synchronize()
    fwd_ms = np.array([sev[k][0].elapsed_time(sev[k][1]) for k in range(nst)])
    bwd_ms = np.array([sev[k][1].elapsed_time(sev[k][2]) for k in range(nst)])
    step_stats = {"steps": nst, "step_ms_median": float(np.median(fwd_ms + bwd_ms)), "step_ms_min": float(np.min(fwd_ms + bwd_ms)),
                  "forward_ms_median": float(np.median(fwd_ms)), "backward_ms_median": float(np.median(bwd_ms))}

    # ---- single-layer ABI calls one by one (each with its own slice-sum launch): per-layer rates
    n_calls = len(st.calls(0))
    ksteps = min(steps, 50)
    evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_calls)]
           for _ in range(ksteps)]
    for k in range(ksteps):
        for c, (tag, l, thunk) in enumerate(st.calls(k)):
            evs[k][c][0].record(st.stream)
            thunk()
            evs[k][c][1].record(st.stream)
    torch.cuda.synchronize()
    per_call = []
    for c, (tag, l, _) in enumerate(st.calls(0)):
        ms = float(np.median([evs[k][c][0].elapsed_time(evs[k][c][1]) for k in range(ksteps)]))   # robust to a stray slow launch
        I, O = w.layers[l]
        fl, by = call_work(tag, B, I, O, w.degree)
        per_call.append({"call": tag, "layer": l, "in": I, "out": O, "us": round(ms * 1e3, 2),
                         "tflops": round(fl / (ms * 1e-3) / 1e12, 3), "gbs": round(by / (ms * 1e-3) / 1e9, 1),
                         "mfma_frac": round(fl / (ms * 1e-3) / 1e12 / PEAK_MFMA_F32_TFLOPS, 4),
                         "hbm_frac": round(by / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)})

    total_flops = sum(wl.layer_flops(B, i, o, w.degree) for (i, o) in w.layers)
    total_bytes = sum(wl.layer_bytes(B, i, o, w.degree) for (i, o) in w.layers)
    # composite roofline of the step: per layer the larger of its MFMA time and its HBM time at the published peaks
    composite_us = sum(max(wl.layer_flops(B, i, o, w.degree) / (PEAK_MFMA_F32_TFLOPS * 1e12),
                           wl.layer_bytes(B, i, o, w.degree) / (PEAK_HBM_GBS * 1e9)) for (i, o) in w.layers) * 1e6
    basis_note = {"exact": "", "lut": ", table-interpolated basis with %d samples" % args.lut_size,
                  "lut2": ", table-interpolated basis and derivative table with %d samples" % args.lut_size}.get(
                      args.basis, ", %s basis" % args.basis)
    res = {
        "metric": "Cheby-KAN fwd+bwd samples/s", "value": B / (ms_per_step * 1e-3), "unit": "samples/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %s, batch %d, widths %s, degree %d%s" % (
            w.name, w.note, B, "->".join(map(str, w.widths)), w.degree, basis_note),
            "input_sets_rotated": len(st.x0_sets), "basis": args.basis,
            "launch": "hip graph replay" if args.graph else "eager",
            "kernel_timing_inside_timed_steps": trace_timed},
        "tflops": total_flops / (ms_per_step * 1e-3) / 1e12,
        "algorithmic_gbs": total_bytes / (ms_per_step * 1e-3) / 1e9,
        "mfma_frac": total_flops / (ms_per_step * 1e-3) / 1e12 / PEAK_MFMA_F32_TFLOPS,
        "hbm_frac": total_bytes / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "roofline": roof,
        "composite_roofline": {"us": round(composite_us, 2), "frac": round(composite_us / (ms_per_step * 1e3), 4),
                               "note": "sum over layers of max(MFMA time, HBM time) at the published peaks / measured step"},
        "kernels": kernels,
        "kernel_timing": {"steps": traced_steps, "ms_per_step_while_timed": traced_ms,
                          "kernel_us_per_step": round(kernel_us_per_step, 2)},
        "event_timed": step_stats,
        "calls": per_call,
    }
    if not args.no_cold and not brief:
        res["cold"] = cold_pass(st, lambda: Stack(w, 1, torch, binding, wl, lut, kind, dlut), torch)
    if not args.no_cpu_baseline and not brief:
        res["cpu_baseline"] = cpu_baseline(w, wl, args.cpu_seconds, args.lut_size if lut is not None else 0, kind)
    stream = st.stream
    del st
    torch.cuda.empty_cache()
    return res, stream


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (--gpus %d refused)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2511_14852_amd import binding, workloads as wl

    if not torch.cuda.is_available():
        raise RuntimeError("bench.py needs a GPU; there is no CPU fallback")
    binding.load()
    binding.chebykan_init()
    binding.chebykan_set_kernel_family(args.family)

    if args.probe > 0:
        w = wl.WORKLOADS[args.workload]
        st = Stack(w, max(1, args.rotate), torch, binding, wl)
        src = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        with torch.cuda.stream(st.stream):
            dst.copy_(src)                      # reads 256 MiB, writes 256 MiB
        for k in range(args.probe):
            if args.probe_calls:
                for (_tag, _l, thunk) in st.calls(k):
                    thunk()
            else:
                st.step(k)
        torch.cuda.synchronize()
        print(json.dumps({"probe_steps": args.probe, "copy_bytes_each_way": src.numel() * 4}), flush=True)
        return

    line, stream = run_workload(args.workload, args.steps, args.warmup, args, torch, binding, wl)
    line["measured_peaks"] = measured_peaks(torch, binding, stream)
    if args.workload == HEADLINE and not args.no_tabular and args.basis == "exact" and not args.graph:
        sub, _ = run_workload(TABULAR, args.tabular_steps, max(args.warmup, 20), args, torch, binding, wl)
        line["tabular_%s" % TABULAR] = sub
        for key, name in (("speech_c3", "c3"), ("audio_c4", "c4")):
            sub, _ = run_workload(name, args.stack_steps, args.warmup, args, torch, binding, wl, brief=True)
            line[key] = sub
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()

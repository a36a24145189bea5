#!/usr/bin/env python3
"""Benchmark of the fused Chebyshev-KAN forward + backward pass on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input:
forward through every layer of the workload's stack, then backward (dx and dC)
through every layer in reverse, all enqueued through the C ABI on one stream.

Prints ONE JSON line.  `value` is rows per second of the whole job, inputs
resident in HBM.  `roofline` describes the dominant kernel call, timed with
events on the launch stream in a second pass over the same steps (so the event
records do not perturb `value`).  `cpu_baseline` is the fp64 CPU oracle timed on
this machine's host cores on a bounded row sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F32_TFLOPS = 157.3     # MI355X dense fp32 matrix peak
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E peak

# HBM bytes per launch of a call (all kernels of the call), from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs scaled by the same counters on a 256 MiB copy (profiles/<workload>_counters.md).
# Keyed by (workload, call, layer); a call that is not listed reports traffic = null.
MEASURED_TRAFFIC_BYTES = {
    ("c2", "dC", 1): 48.4e6 + 14.8e6,      # slice kernel + combine
    ("c2", "dx", 1): 80.6e6,
    ("c2", "fwd", 1): 26.8e6,
    ("c5", "dC", 0): 959.4e6 + 264.3e6,
    ("c5", "fwd", 0): 754.7e6,
    ("c5", "dx", 0): 1760.5e6,
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5", "p1", "p2", "p3"])
    ap.add_argument("--rotate", type=int, default=4,
                    help="number of distinct (x, dy) input sets cycled through, so inputs are not cache-resident")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--no-cold", action="store_true",
                    help="skip the cold pass (whole buffer sets rotated through at least 512 MB)")
    ap.add_argument("--family", type=int, default=0, help="kernel family override (0 auto)")
    ap.add_argument("--basis", default="exact", choices=["exact", "lut", "legendre", "hermite", "fourier"],
                    help="exact = Chebyshev recurrences (default); lut = the paper's table-interpolated variant "
                         "(Sec. 4.2); legendre / hermite / fourier = the other bases of Sec. 2.3 on the same kernels")
    ap.add_argument("--lut-size", type=int, default=1025, help="table samples for --basis lut")
    ap.add_argument("--graph", action="store_true",
                    help="capture the steps (one per rotated input set) in a HIP graph and time its replays; the "
                         "first replay is checked against the eager result")
    ap.add_argument("--probe", type=int, default=0,
                    help="counter-collection mode for rocprofv3 --pmc: run this many steps of the split calls plus "
                         "one plain 256 MiB device copy (the calibration kernel of known size), then exit")
    return ap.parse_args()


class Stack:
    """Device buffers and the launch sequence of one workload."""

    def __init__(self, w, rotate, torch, binding, wl, lut=None, kind=0):
        self.w, self.torch, self.binding = w, torch, binding
        self.kind = kind        # 0 Chebyshev, 1 Legendre, 2 Hermite, 3 Fourier
        self.lut = lut          # device table [degree+1, samples] or None for the exact basis
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
        else:
            b.chebykan_backward_lut(xin, self.C[l], dy, self.lut, dx, dC, self.ws[l], s)

    def calls(self, step):
        """The ABI calls of one step, in order: (tag, layer, thunk)."""
        b, n = self.binding, len(self.layers)
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

    def step_fused_calls(self, step):
        """One step as a user would issue it: the stack's forward call (the library runs a narrow stack in
        one kernel, any other stack layer by layer), then one backward call per layer."""
        self.step_forward(step)
        self.step_backward(step)

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
            # the stack call: per-layer gradient kernels, then every slice sum in one launch
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
        s.step_fused_calls(0)
    torch.cuda.synchronize()
    n = rounds * n_sets
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    ev[0].record(st.stream)
    for k in range(n):
        sets[k % n_sets].step_fused_calls(0)
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
    binding.chebykan_set_kernel_family(args.family)
    w = wl.WORKLOADS[args.workload]
    lut = None
    if args.basis == "lut":
        lut = binding.chebykan_lut_build(w.degree, args.lut_size).cuda()
    kind = {"legendre": 1, "hermite": 2, "fourier": 3}.get(args.basis, 0)
    if kind == 3 and w.degree % 2:
        raise SystemExit("the Fourier basis needs an even degree; workload %s has degree %d" % (w.name, w.degree))
    st = Stack(w, max(1, args.rotate), torch, binding, wl, lut, kind)
    B = w.batch

    if args.probe > 0:
        src = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        with torch.cuda.stream(st.stream):
            dst.copy_(src)                      # reads 256 MiB, writes 256 MiB
        for k in range(args.probe):
            for (_tag, _l, thunk) in st.calls(k):
                thunk()
        torch.cuda.synchronize()
        print(json.dumps({"probe_steps": args.probe, "copy_bytes_each_way": src.numel() * 4}), flush=True)
        return

    # ---- throughput: W warm-up steps, then exactly K timed steps
    for k in range(args.warmup):
        st.step_fused_calls(k)
    torch.cuda.synchronize()
    if args.graph:
        # one graph holds one step per rotated input set; K steps = K / sets replays (K is rounded up to that)
        sets = len(st.x0_sets)
        st.step_fused_calls(0)
        torch.cuda.synchronize()
        eager = [t.clone() for t in (st.y[-1], st.dx[0], st.dC[0])]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=st.stream):
            for k in range(sets):
                st.step_fused_calls(k)
        graph.replay()
        torch.cuda.synchronize()
        st.step_fused_calls(sets - 1)          # eager result of the set the graph ended on
        torch.cuda.synchronize()
        last = [t.clone() for t in (st.y[-1], st.dx[0], st.dC[0])]
        replays = (args.steps + sets - 1) // sets
        args.steps = replays * sets
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        for a, b_ in zip(last, (st.y[-1], st.dx[0], st.dC[0])):
            if not torch.equal(a, b_):
                raise RuntimeError("graph replay differs from the eager step")
        del eager
    else:
        t0 = time.perf_counter()
        for k in range(args.steps):
            st.step_fused_calls(k)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    # ---- whole steps with events: median / min per step, forward and backward apart
    nst = min(args.steps, 50)
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

    # ---- per-call durations: the same steps again with events on the launch stream
    n_calls = len(st.calls(0))
    ksteps = min(args.steps, 50)
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
    dom = max(per_call, key=lambda r: r["us"])
    I, O = dom["in"], dom["out"]
    fl, by = call_work(dom["call"], B, I, O, w.degree)
    t_mfma, t_hbm = fl / (PEAK_MFMA_F32_TFLOPS * 1e12), by / (PEAK_HBM_GBS * 1e9)
    if t_mfma >= t_hbm:
        roof = {"bound": "mfma", "achieved": dom["tflops"], "peak": PEAK_MFMA_F32_TFLOPS, "unit": "TFLOP/s",
                "frac": round(dom["tflops"] / PEAK_MFMA_F32_TFLOPS, 4)}
    else:
        roof = {"bound": "hbm", "achieved": dom["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(dom["gbs"] / PEAK_HBM_GBS, 4)}
    roof["traffic"] = MEASURED_TRAFFIC_BYTES.get((w.name, dom["call"], dom["layer"])) if lut is None and not kind else None
    roof["algorithmic_bytes"] = by
    roof["kernel"] = "%s layer %d (%d->%d)" % (dom["call"], dom["layer"], I, O)
    roof["us"] = dom["us"]

    total_flops = sum(wl.layer_flops(B, i, o, w.degree) for (i, o) in w.layers)
    total_bytes = sum(wl.layer_bytes(B, i, o, w.degree) for (i, o) in w.layers)
    # composite roofline of the step: per layer the larger of its MFMA time and its HBM time at the published peaks
    composite_us = sum(max(wl.layer_flops(B, i, o, w.degree) / (PEAK_MFMA_F32_TFLOPS * 1e12),
                           wl.layer_bytes(B, i, o, w.degree) / (PEAK_HBM_GBS * 1e9)) for (i, o) in w.layers) * 1e6
    line = {
        "metric": "Cheby-KAN fwd+bwd samples/s", "value": B / (ms_per_step * 1e-3), "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %s, batch %d, widths %s, degree %d%s" % (
            w.name, w.note, B, "->".join(map(str, w.widths)), w.degree,
            (", %s basis" % args.basis if kind else "") if lut is None
            else ", table-interpolated basis with %d samples" % args.lut_size),
            "input_sets_rotated": len(st.x0_sets), "basis": args.basis,
            "launch": "hip graph replay" if args.graph else "eager"},
        "tflops": total_flops / (ms_per_step * 1e-3) / 1e12,
        "algorithmic_gbs": total_bytes / (ms_per_step * 1e-3) / 1e9,
        "mfma_frac": total_flops / (ms_per_step * 1e-3) / 1e12 / PEAK_MFMA_F32_TFLOPS,
        "hbm_frac": total_bytes / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "roofline": roof,
        "composite_roofline": {"us": round(composite_us, 2), "frac": round(composite_us / (ms_per_step * 1e3), 4),
                               "note": "sum over layers of max(MFMA time, HBM time) at the published peaks / measured step"},
        "event_timed": step_stats,
        "calls": per_call,
    }
    line["measured_peaks"] = measured_peaks(torch, binding, st.stream)
    if not args.no_cold:
        line["cold"] = cold_pass(st, lambda: Stack(w, 1, torch, binding, wl, lut, kind), torch)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, wl, args.cpu_seconds, args.lut_size if lut is not None else 0, kind)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()

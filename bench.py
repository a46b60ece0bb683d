#!/usr/bin/env python3
"""Benchmark of the hot path: fused dual-number forward + adjoint x partial backward.

One "step" = one forward call + one backward call over one batch of synthetic input
already resident in HBM.  Prints ONE JSON line.  The headline workload is the large HM-LSTM
cell update (hidden 4096, batch 1024, per-element z ~ Bernoulli(0.5)); the same line carries
a "configs" object with every benchmark configuration timed the same way in the same run.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

Workloads: cfg0 cfg1 cfg2 cfg3 (p via --p-index 0|1|2) cfg4 cfg4_f64, paper_n512 /
paper_n1024 / paper_n2048 (the paper's own experiment shape, Sec. 3.4), hmlstm_<H>x<B>,
linear12_<H>x<B>, branchy5_3d_<O>x<R>x<C>, branchy5_3dm_<O>x<R>x<C>.
"""
from __future__ import annotations

import argparse
import ctypes
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth

# HBM bytes per launch from rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE scaled by a copy kernel of
# known size): written by `python -m paper_1810_08297_amd.pmc_traffic`, which also records the
# kernel names and a hash of the kernel sources the figures were measured on.
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "hbm_traffic_pmc.json")

# the configurations of the "configs" object: (key, workload, p_index)
ALL_CONFIGS = [("cfg0", "cfg0", 1), ("cfg1", "cfg1", 1), ("cfg2", "cfg2", 1), ("cfg3_p0.05", "cfg3", 0),
               ("cfg3_p0.5", "cfg3", 1), ("cfg3_p0.95", "cfg3", 2), ("cfg4", "cfg4", 1), ("cfg4_f64", "cfg4_f64", 1)]


def source_hash():
    """sha256 over the library's sources (the same function as in pmc_traffic: a stored traffic
    figure counts as current only for the sources it was measured on)."""
    from paper_1810_08297_amd.pmc_traffic import source_hash as h
    return h()


def measured_traffic(workload, role):
    """(bytes per launch or None, matches the sources built here) for the forward / backward kernel."""
    try:
        with open(TRAFFIC_JSON) as f:
            table = json.load(f)
    except (OSError, ValueError):
        return None, None
    rec = table.get("workloads", {}).get(workload, {}).get(role)
    if rec is None:
        return None, None
    return rec["traffic_bytes"], table.get("source_hash") == source_hash()


def build_workload(name, p_index, uniform_run=0):
    import numpy as np
    from paper_1810_08297_amd import inputs
    dtype = np.float64 if name.endswith("_f64") else np.float32
    base = name.replace("_f64", "")
    if base.startswith("cfg"):
        idx = int(base[3:])
        op, args, adj = inputs.config_inputs(idx, dtype=dtype, p_index=p_index)
        desc = {0: "HM-LSTM update hidden=64 batch=16", 1: "tanh(x*y+b) 4096x4096",
                2: "HM-LSTM update hidden=1024 batch=256",
                3: f"HM-LSTM update hidden=4096 batch=1024, per-element z ~ Bernoulli({inputs.P_SWEEP[p_index]})",
                4: "branchy5 8192x8192"}[idx]
    elif base.startswith("hmlstm_"):  # hmlstm_<hidden>x<batch>: the HM-LSTM update at another size (beyond the five configs)
        H, Bt = (int(x) for x in base[len("hmlstm_"):].split("x"))
        args, adj = inputs.hmlstm_inputs(H, Bt, seed=inputs.BASE_SEED + 300 + H + Bt, dtype=dtype, z_per_element=True,
                                         p=inputs.P_SWEEP[p_index])
        op, desc = "hmlstm_update", f"HM-LSTM update hidden={H} batch={Bt}, per-element z ~ Bernoulli({inputs.P_SWEEP[p_index]})"
    elif base.startswith("linear12_"):  # the HM-LSTM update's argument list and traffic with trivial arithmetic
        H, Bt = (int(x) for x in base[len("linear12_"):].split("x"))
        args, adj = inputs.hmlstm_inputs(H, Bt, seed=inputs.BASE_SEED + 300 + H + Bt, dtype=dtype, z_per_element=True,
                                         p=inputs.P_SWEEP[p_index])
        op, desc = "linear12", f"linear12 (HM-LSTM traffic, no transcendental) hidden={H} batch={Bt}"
    elif base.startswith("branchy5_3d"):  # branchy5_3d_<O>x<R>x<C>: r broadcast along the middle dim only; branchy5_3dm_...: shapes that merge to two dims
        merging = base.startswith("branchy5_3dm_")
        O, R, C = (int(x) for x in base.split("_")[-1].split("x"))
        args, adj = inputs.branchy5_3d_inputs(O, R, C, seed=inputs.BASE_SEED + 500 + O + R + C, dtype=dtype, merging=merging)
        op = "branchy5"
        desc = (f"branchy5 over [{O} x {R} x {C}], " + (f"r [1 x 1 x {C}], s [{O} x {R} x 1] (merges to two dims)" if merging else
                                                     f"r [{O} x 1 x {C}], s [1 x {R} x 1] (stays three dims)"))
    elif base.startswith("paper_n"):
        n = int(base[len("paper_n"):])
        args, adj = inputs.update_c_inputs(n, seed=inputs.BASE_SEED + 100 + n, dtype=dtype, uniform_run=uniform_run)
        op, desc = "update_c", (f"paper's cell update c,f,i,g {n}x{n}, z vectors of {n}, " +
                                (f"control inputs constant over runs of {uniform_run}" if uniform_run else
                                 "random control inputs"))
    else:
        raise SystemExit(f"unknown workload {name}")
    return op, args, adj, desc, dtype


class Workload:
    """One workload resident in HBM (every full-shape buffer in the library's staggered slab layout)."""

    def __init__(self, name, p_index, a):
        import numpy as np
        import torch
        import paper_1810_08297_amd as P
        self.name = name
        self.op, self.args, self.adj, self.desc, self.dtype = build_workload(name, p_index, a.uniform_run)
        if a.transposed:
            self.args = [np.ascontiguousarray(x.T) for x in self.args]
            self.adj = [np.ascontiguousarray(x.T) for x in self.adj]
            self.desc += ", transposed"
        self.es = np.dtype(self.dtype).itemsize
        self.layout = getattr(a, "layout", "staggered")
        self.dev, self._slab_a = P.to_slab([torch.from_numpy(x).cuda() for x in self.args], layout=self.layout)
        self.adj_dev, self._slab_b = P.to_slab([torch.from_numpy(x).cuda() for x in self.adj], layout=self.layout)
        if a.sliced_gates and self.op in ("hmlstm_update", "linear12"):
            Bt = self.args[0].shape[1]
            wide = torch.empty(self.args[0].shape[0], 4 * Bt, dtype=self.dev[0].dtype, device="cuda")
            for k in range(4):
                wide[:, k * Bt:(k + 1) * Bt].copy_(self.dev[k])
                self.dev[k] = wide[:, k * Bt:(k + 1) * Bt]
            self.desc += ", gates as column slices of one buffer"


def measure(w, a, options, sptr, steps, warmup, lean=False, event_every=0):
    """Warm-up + `steps` timed steps of one workload for one partial-storage layout.  The whole
    step is timed on the host clock between two device synchronisations; on every `event_every`-th
    step each of the two launches also stamps a pair of HIP events with the kernel's own begin and
    end (the library hands them to hipExtLaunchKernelGGL; stream markers around the launches would
    also hold their own cost and the gap to the next launch, and slow the step they sit in)."""
    import numpy as np
    import torch
    import paper_1810_08297_amd as P
    fb = P.alloc_forward(w.op, w.dev, want_branch=False, lean=lean, options=options, layout=w.layout)
    didx = P.diff_arg_indices(fb.op_id)
    shapes = [w.args[j].shape for j in didx]
    bb = P.alloc_backward(w.adj_dev, fb.partials, shapes, options=options, layout=w.layout)
    E = int(np.prod(fb.outs[0].shape))
    M, Nd = len(fb.outs), len(didx)
    n_full_args = sum(1 for x in w.args if x.size == E)
    n_full_grads = sum(1 for s_ in shapes if int(np.prod(s_)) == E)
    n_stored = len({t.data_ptr() for t in fb.partials if t is not None})  # planes that cross the HBM interface
    fwd_words = n_full_args + M + n_stored
    bwd_words = M + n_stored + n_full_grads
    fwd_bytes, bwd_bytes = fwd_words * w.es * E, bwd_words * w.es * E
    fwd_call = fb.prepare(w.dev)                    # argument blocks marshalled once;
    bwd_call = bb.prepare(w.adj_dev, fb.partials)   # each launch() is one C-ABI call
    bplan = P.bcast_dual_backward_plan(w.adj_dev, fb.partials, bb.grads, options=options)
    for _ in range(warmup):
        fwd_call.launch(sptr)
        bwd_call.launch(sptr)
    torch.cuda.synchronize()
    if event_every <= 0:  # a few more untimed steps tell a long step from a short one
        w0 = time.perf_counter()
        for _ in range(8):
            fwd_call.launch(sptr)
            bwd_call.launch(sptr)
        torch.cuda.synchronize()
        event_every = 4 if (time.perf_counter() - w0) / 8 >= 100e-6 else 16
    timers = {k: (P.LaunchTimer(), P.LaunchTimer()) for k in range(0, steps, event_every)}
    timed = {k: (t[0].options(options), t[1].options(options)) for k, t in timers.items()}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        t = timed.get(k)
        if t is None:
            fwd_call.launch(sptr)
            bwd_call.launch(sptr)
        else:
            fwd_call.launch(sptr, t[0])
            bwd_call.launch(sptr, t[1])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev = list(timers.values())
    fwd_ms = np.array([t[0].ms() for t in ev])
    bwd_ms = np.array([t[1].ms() for t in ev])  # the main backward kernel (a second reduction pass is not in it)
    fwd_avg, bwd_avg = float(fwd_ms.mean()), float(bwd_ms.mean())
    both = (fwd_bytes + bwd_bytes) / ((fwd_avg + bwd_avg) * 1e-3) / 1e9
    return {
        "E": E, "M": M, "Nd": Nd, "n_stored": n_stored, "shapes": shapes, "wall": wall, "event_every": event_every,
        "value": E * steps / wall, "ms_per_step": wall * 1e3 / steps,
        "fwd_avg": fwd_avg, "bwd_avg": bwd_avg, "fwd_bytes": fwd_bytes, "bwd_bytes": bwd_bytes,
        "bwd_launches": bplan["n_launches"],
        "detail": {
            "elements": E,
            "forward": {"avg_ms": round(fwd_avg, 5), "median_ms": round(float(np.median(fwd_ms)), 5),
                        "bytes": fwd_bytes, "GBps": round(fwd_bytes / (fwd_avg * 1e-3) / 1e9, 1)},
            "backward": {"avg_ms": round(bwd_avg, 5), "median_ms": round(float(np.median(bwd_ms)), 5),
                         "bytes": bwd_bytes, "GBps": round(bwd_bytes / (bwd_avg * 1e-3) / 1e9, 1)},
            "event_samples": len(ev),
            "fwd_bwd_GBps_event_time": round(both, 1),
            "fwd_bwd_frac_of_hbm_peak": round(both / HBM_PEAK_GBS, 4),
            "elements_per_s_event_time": round(E / ((fwd_avg + bwd_avg) * 1e-3), 1),
            "bytes_per_element": (fwd_words + bwd_words) * w.es,
        },
    }


def config_record(run, workload):
    """One entry of the "configs" object: the whole step on the host clock and the two main kernels on
    their own event pairs, each against the algorithmic bytes it moves."""
    step_us = run["ms_per_step"] * 1e3
    total = run["fwd_bytes"] + run["bwd_bytes"]
    rec = {
        "elements": run["E"], "step_us": round(step_us, 2), "elements_per_s": round(run["value"], 1),
        "algorithmic_bytes": total, "step_GBps": round(total / (step_us * 1e-6) / 1e9, 1),
        "step_frac": round(total / (step_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
        "forward_kernel_us": round(run["fwd_avg"] * 1e3, 2), "forward_bytes": run["fwd_bytes"],
        "forward_frac": round(run["fwd_bytes"] / (run["fwd_avg"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "backward_kernel_us": round(run["bwd_avg"] * 1e3, 2), "backward_bytes": run["bwd_bytes"],
        "backward_frac": round(run["bwd_bytes"] / (run["bwd_avg"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "backward_launches": run["bwd_launches"], "event_samples": run["detail"]["event_samples"],
    }
    for role in ("forward", "backward"):
        traffic, current = measured_traffic(workload, role)
        if traffic is not None:
            rec[f"{role}_traffic"] = traffic
            rec["traffic_matches_build"] = current
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg3",
                    help="cfg0..cfg4, cfg4_f64, paper_n<N>, hmlstm_<hidden>x<batch>, linear12_<hidden>x<batch>, "
                         "branchy5_3d_<O>x<R>x<C>, branchy5_3dm_<O>x<R>x<C>")
    ap.add_argument("--p-index", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-threads", type=int, default=16)
    ap.add_argument("--uniform-run", type=int, default=0,
                    help="paper_n* workloads: make z1, z2 constant over aligned runs of this many elements")
    ap.add_argument("--no-lean-extra", action="store_true", help="skip the additional lean-layout and recompute measurements")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the \"configs\" object (every benchmark configuration timed in this run)")
    ap.add_argument("--configs-steps", type=int, default=60, help="timed steps per entry of the \"configs\" object")
    ap.add_argument("--unfused-baseline", action="store_true",
                    help="also time the same function as per-primitive library kernels with reverse-mode autograd")
    ap.add_argument("--transposed", action="store_true",
                    help="every array transposed (stored row-major again): the HM-LSTM update as [batch x hidden] with "
                         "[1 x hidden] biases, whose gradients are then sums over rows")
    ap.add_argument("--sliced-gates", action="store_true",
                    help="HM-LSTM workloads: f, i, o, g are column slices of one buffer four times as wide (row "
                         "stride 4 x batch), so that the views no longer share one row stride")
    ap.add_argument("--event-every", type=int, default=0,
                    help="per-kernel HIP event pairs on every n-th timed step (1 = every step; 0 = every 4th, "
                         "every 16th when a step takes under 100 us: a timed launch costs the host some 50 us)")
    ap.add_argument("--graph", action="store_true",
                    help="also replay the step from a captured HIP graph and report its rate")
    ap.add_argument("--lean", action="store_true",
                    help="store planes the op table declares identical once and leave always-zero planes out")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run the library's 1-in 1-out stream probe on a buffer of this many MiB "
                         "(a copy of known size, for scaling profiler byte counters)")
    ap.add_argument("--layout", choices=["staggered", "interleaved", "plain"], default="staggered",
                    help="how the full-shape buffers of a group (arguments; outputs + planes; adjoints; gradients) share "
                         "a slab: separate planes staggered by one page each (default), interleaved by row, or plain")
    ap.add_argument("--opt", type=lambda t: (t.split("=")[0], int(t.split("=")[1])), action="append", default=[],
                    help="FIELD=VALUE of bcast_dual_options for every call of the run (launch-shape sweeps), repeatable")
    a = ap.parse_args()
    if a.gpus != 1:
        raise SystemExit("bench.py: this build runs on exactly one GPU (--gpus 1); "
                         "no multi-GPU path exists and none is measured")

    import numpy as np
    import torch
    import paper_1810_08297_amd as P

    torch.cuda.set_device(0)
    options = P.Options(**dict(a.opt)) if a.opt else None
    stream = torch.cuda.current_stream()
    sptr = ctypes.c_void_p(stream.cuda_stream)

    w = Workload(a.workload, a.p_index, a)
    op, args, adj, desc, dtype, es, dev, adj_dev = w.op, w.args, w.adj, w.desc, w.dtype, w.es, w.dev, w.adj_dev

    run = measure(w, a, options, sptr, a.steps, a.warmup, lean=a.lean, event_every=a.event_every)
    event_every = run["event_every"]
    if a.copy_probe_mib > 0:
        n = a.copy_probe_mib * (1 << 20) // 4
        src = torch.empty(n, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            P.bcast_dual_stream_probe([src.data_ptr()], [1024], [dst.data_ptr()], [1024], n // 1024, sptr, options)
        torch.cuda.synchronize()
        del src, dst
    E, M, Nd, n_stored, shapes = run["E"], run["M"], run["Nd"], run["n_stored"], run["shapes"]
    value, ms_per_step, extra = run["value"], run["ms_per_step"], run["detail"]
    fwd_avg, bwd_avg = run["fwd_avg"], run["bwd_avg"]
    dom = "forward" if fwd_avg >= bwd_avg else "backward"
    dom_bytes = run["fwd_bytes"] if dom == "forward" else run["bwd_bytes"]
    dom_ms = max(fwd_avg, bwd_avg)
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    traffic, traffic_current = (None, None) if a.lean else measured_traffic(a.workload, dom)
    roofline = {
        "bound": "hbm", "kernel": f"{dom} ({'fwd_tiled_kernel' if dom == 'forward' else 'bwd_sig_kernel'})",
        "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4),
        "traffic": traffic, "traffic_matches_build": traffic_current,
        "algorithmic_bytes_per_launch": dom_bytes,
        "avg_launch_ms": round(dom_ms, 5),
    }
    # the same step with the leaner partial store (same outputs and gradients, fewer bytes), for reference
    lean_extra = None
    if not a.lean and not a.no_lean_extra:
        lr = measure(w, a, options, sptr, a.steps, a.warmup, lean=True, event_every=event_every)
        if lr["n_stored"] < n_stored:
            lean_extra = {"value": round(lr["value"], 1), "unit": "elements/s", "ms_per_step": round(lr["ms_per_step"], 5),
                          "planes_stored": lr["n_stored"], **lr["detail"]}

    # the other side of the paper's trade-off (end of Sec. 2.2.3): no planes at all, the dual
    # numbers are evaluated again in the reverse pass -- values-only forward + recompute backward
    recompute_extra = None
    if not a.lean and not a.no_lean_extra:
        try:
            fbv = P.alloc_forward(op, dev, want_branch=False, want_partials=False, options=options)
            rb = P.alloc_recompute(fbv.op_id, dev, adj_dev, shapes, options=options)
            fcall = fbv.prepare(dev)
            rcall = P.PreparedRecompute(fbv.op_id, dev, adj_dev, rb.grads, rb.workspace, options)
            fcall.launch(sptr)
            rcall.launch(sptr)  # a layout the recompute entry point refuses shows here
        except P.BcastError:
            fcall = None
        if fcall is not None:
            for _ in range(a.warmup):
                fcall.launch(sptr)
                rcall.launch(sptr)
            torch.cuda.synchronize()
            timers = {k: (P.LaunchTimer(), P.LaunchTimer()) for k in range(0, a.steps, event_every)}
            timed = {k: (t[0].options(options), t[1].options(options)) for k, t in timers.items()}
            t0 = time.perf_counter()
            for k in range(a.steps):
                t = timed.get(k)
                if t is None:
                    fcall.launch(sptr)
                    rcall.launch(sptr)
                else:
                    fcall.launch(sptr, t[0])
                    rcall.launch(sptr, t[1])
            torch.cuda.synchronize()
            wall = time.perf_counter() - t0
            ev = list(timers.values())
            f_ms = float(np.mean([t[0].ms() for t in ev]))
            r_ms = float(np.mean([t[1].ms() for t in ev]))
            n_full_args = sum(1 for x in args if x.size == E)
            n_full_grads = sum(1 for s_ in shapes if int(np.prod(s_)) == E)
            f_bytes, r_bytes = (n_full_args + M) * es * E, (n_full_args + M + n_full_grads) * es * E
            recompute_extra = {
                "value": round(E * a.steps / wall, 1), "unit": "elements/s", "ms_per_step": round(wall * 1e3 / a.steps, 5),
                "forward_values_only": {"avg_ms": round(f_ms, 5), "bytes": f_bytes,
                                        "GBps": round(f_bytes / (f_ms * 1e-3) / 1e9, 1)},
                "backward_recompute": {"avg_ms": round(r_ms, 5), "bytes": r_bytes,
                                       "GBps": round(r_bytes / (r_ms * 1e-3) / 1e9, 1)},
                "bytes_per_element": (f_bytes + r_bytes) // E,
            }
            del fbv, rb, fcall, rcall

    # the same step replayed from a HIP graph (one launch of the graph = forward + backward):
    # separates the host's per-call cost from the kernels' for the small, launch-bound configs
    graph_extra = None
    if a.graph:
        fb = P.alloc_forward(op, dev, want_branch=False, lean=a.lean, options=options)
        bb = P.alloc_backward(adj_dev, fb.partials, shapes, options=options)
        fcall, bcall = fb.prepare(dev), bb.prepare(adj_dev, fb.partials)
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            for _ in range(3):
                fcall.launch()
                bcall.launch()
        stream.wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fcall.launch()
            bcall.launch()
        for _ in range(a.warmup):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            g.replay()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        graph_extra = {"value": round(E * a.steps / wall, 1), "unit": "elements/s",
                       "ms_per_step": round(wall * 1e3 / a.steps, 5)}

    # unfused comparison: one library kernel per primitive, both branches + select, reverse mode
    unfused_extra = None
    if a.unfused_baseline:
        from paper_1810_08297_amd.unfused_baseline import UnfusedPrimitives, UnfusedStep
        # the library's own per-primitive kernels (written from the math), then the same chain on torch's
        prim = None
        try:
            up = UnfusedPrimitives(op, dev, adj_dev)
        except (KeyError, ValueError):
            up = None
        if up is not None:
            for _ in range(3):
                n_k = up.run(sptr)[2]
            torch.cuda.synchronize()
            n_un = max(5, a.steps // 4)
            t0 = time.perf_counter()
            for _ in range(n_un):
                up.run(sptr)
            torch.cuda.synchronize()
            wall = time.perf_counter() - t0
            prim = {"value": round(E * n_un / wall, 1), "unit": "elements/s", "steps": n_un, "ms_per_step": round(wall * 1e3 / n_un, 5),
                    "kernels_per_step": n_k, "kind": "the library's per-primitive kernels, reverse mode rule by rule"}
            g = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(stream)
            with torch.cuda.stream(side):
                up.run()
            stream.wait_stream(side)
            torch.cuda.synchronize()
            with torch.cuda.graph(g):
                up.run()
            for _ in range(3):
                g.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n_un):
                g.replay()
            torch.cuda.synchronize()
            wall = time.perf_counter() - t0
            prim["graph_replay"] = {"value": round(E * n_un / wall, 1), "ms_per_step": round(wall * 1e3 / n_un, 5)}
            del up, g
            torch.cuda.empty_cache()
        ust = UnfusedStep(op, dev, adj_dev)
        for _ in range(max(3, a.warmup // 4)):
            ust.run()
        torch.cuda.synchronize()
        n_un = max(5, a.steps // 4)
        t0 = time.perf_counter()
        for _ in range(n_un):
            ust.run()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        unfused_extra = {"value": round(E * n_un / wall, 1), "unit": "elements/s", "steps": n_un,
                         "ms_per_step": round(wall * 1e3 / n_un, 5), "kind": "torch elementwise kernels + autograd"}
        # the same kernels replayed from a HIP graph: takes the framework's host time out of the comparison
        try:
            side = torch.cuda.Stream()
            side.wait_stream(stream)
            with torch.cuda.stream(side):
                for _ in range(3):
                    ust.run()
            stream.wait_stream(side)
            torch.cuda.synchronize()
            ug = torch.cuda.CUDAGraph()
            with torch.cuda.graph(ug):
                ust.run()
            for _ in range(3):
                ug.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n_un):
                ug.replay()
            torch.cuda.synchronize()
            wall = time.perf_counter() - t0
            unfused_extra["graph_replay"] = {"value": round(E * n_un / wall, 1), "ms_per_step": round(wall * 1e3 / n_un, 5)}
        except Exception as e:  # capture of library kernels is best effort; the eager number stands
            unfused_extra["graph_replay"] = {"error": str(e)[:200]}
        unfused_extra = {"per_primitive_hip_kernels": prim, "torch_elementwise_autograd": unfused_extra}

    cpu = None
    if not a.no_cpu_baseline:
        import oracle
        threads = max(1, min(a.cpu_threads, os.cpu_count() or 1))
        # bounded sample: whole rows of the same workload (at most 4M elements), repeated
        # until about 1.5 s of wall time have passed
        rows = args[0].shape[0]
        cols = E // rows
        take = max(1, min(rows, (1 << 22) // max(1, cols)))
        sub = [x[:take] if x.shape[0] == rows else x for x in args]
        sub_adj = [x[:take] for x in adj]
        sub_shapes = [s if s[0] != rows else (take,) + tuple(s[1:]) for s in shapes]
        reps, c0 = 0, time.perf_counter()
        while True:
            o_out, o_parts, _ = oracle.forward(op, sub, threads=threads)
            oracle.backward(sub_adj, o_parts, sub_shapes, threads=threads)
            reps += 1
            c1 = time.perf_counter()
            if c1 - c0 >= 1.5 or reps >= 200:
                break
        cpu = {"value": round(reps * take * cols / (c1 - c0), 1), "unit": "elements/s", "cores": threads,
               "kind": "oracle", "sample": f"first {take} of {rows} rows ({take * cols} elements), forward + "
               f"backward {reps} times in {c1 - c0:.2f} s ({threads * (c1 - c0):.0f} core-seconds)"}
        # the same oracle on one core, on a smaller sample (at most 2^19 elements, once)
        take1 = max(1, min(take, (1 << 19) // max(1, cols)))
        sub1 = [x[:take1] if x.shape[0] == rows else x for x in args]
        shapes1 = [s if s[0] != rows else (take1,) + tuple(s[1:]) for s in shapes]
        s0 = time.perf_counter()
        o_out, o_parts, _ = oracle.forward(op, sub1, threads=1)
        oracle.backward([x[:take1] for x in adj], o_parts, shapes1, threads=1)
        s1 = time.perf_counter()
        cpu["single_thread"] = {"value": round(take1 * cols / (s1 - s0), 1), "unit": "elements/s",
                                "sample": f"first {take1} rows ({take1 * cols} elements), once, {s1 - s0:.2f} s"}

    # every benchmark configuration, timed the same way in this same run (all planes stored, default options
    # unless --opt); the entry of the headline workload is the headline run itself
    configs = None
    if not a.no_configs and not (a.lean or a.transposed or a.sliced_gates or a.uniform_run or a.layout != "staggered"):
        configs = {}
        headline_key = next((k for k, wl, pi in ALL_CONFIGS if wl == a.workload and pi == a.p_index), None)
        if headline_key:
            configs[headline_key] = config_record(run, a.workload)
        del w, dev, adj_dev, run
        torch.cuda.empty_cache()
        for key, wl, pi in ALL_CONFIGS:
            if key == headline_key:
                continue
            cw = Workload(wl, pi, a)
            small = cw.args[0].size <= (1 << 20)
            cr = measure(cw, a, options, sptr, a.configs_steps * (4 if small else 1), 10, event_every=a.event_every)
            configs[key] = config_record(cr, wl)
            del cw, cr
            torch.cuda.empty_cache()
        configs = {k: configs[k] for k, _, _ in ALL_CONFIGS if k in configs}

    line = {
        "metric": "fused fwd+bwd elements/s, HM-LSTM update" if op == "hmlstm_update"
                  else f"fused fwd+bwd elements/s, {op}",
        "value": round(value, 1), "unit": "elements/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64" if dtype == np.float64 else "f32", "data": "synthetic",
        "config": {"workload": f"{a.workload}: {desc}", "op": op, "elements": E,
                   "partial_planes": M * Nd, "planes_stored": n_stored,
                   "layout": f"row-major, {a.layout} slab, " + ("identical planes stored once, zero planes left out"
                                                                 if a.lean else "all planes stored"),
                   "options": dict(a.opt) if a.opt else "defaults"},
        "roofline": roofline, "cpu_baseline": cpu, "detail": extra, "lean_layout": lean_extra,
        "recompute_in_reverse": recompute_extra, "graph_replay": graph_extra,
        "unfused_baseline": unfused_extra, "configs": configs,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()

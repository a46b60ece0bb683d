"""Arity study (Sec. 3.4.1 of arXiv 1810.08297) on one MI355X.

  python -m paper_1810_08297_amd.arity_study [--n 1024] [--max-arity 18]

D(f).(x_1 .. x_N) with f = prod_i tanh(g(x_i)), g(x) = x if x > 1/2 else -x, every x_j an
n x n fp32 matrix: the dual-number forward kernel reads N planes and writes 1 + N, and its
register use grows with N.  Prints per arity the forward and backward times (HIP events on
the launch stream, median of 50) and the achieved fraction of the HBM peak, and beside them
the other side of the trade-off at the end of Sec. 2.2.3: no planes kept, a values-only
forward (reads N, writes 1) and a backward that evaluates the dual numbers again (reads
N + 1, writes N) -- N^2 arithmetic against 2 N planes of traffic.
"""
from __future__ import annotations

import argparse

import numpy as np


def main():
    import torch
    import paper_1810_08297_amd as P
    from paper_1810_08297_amd import inputs

    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=1024)
    ap.add_argument("--max-arity", type=int, default=18)
    a = ap.parse_args()
    E = a.n * a.n
    stream = torch.cuda.current_stream()

    def median_us(call, reps=50):
        ev = []
        for _ in range(reps + 5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            call()
            e1.record(stream)
            ev.append((e0, e1))
        torch.cuda.synchronize()
        return float(np.median([x.elapsed_time(y) for x, y in ev[5:]])) * 1e3

    print(f"{'N':>3s} {'fwd us':>9s} {'fwd GB/s':>9s} {'% peak':>7s} {'bwd us':>9s} {'bwd GB/s':>9s} {'% peak':>7s} |"
          f" {'values us':>9s} {'recomp us':>9s} {'GB/s':>8s} {'no planes / planes':>18s}")
    for k in range(1, a.max_arity + 1):
        xs, adj = inputs.prod_tanh_inputs(k, a.n, a.n, seed=inputs.BASE_SEED + 200 + k)
        dev, _s1 = P.to_slab([torch.from_numpy(x).cuda() for x in xs])
        adj_dev = [torch.from_numpy(adj[0]).cuda()]
        fb = P.alloc_forward(f"prod_tanh_{k}", dev)
        bb = P.alloc_backward(adj_dev, fb.partials, [x.shape for x in xs])
        f, b = fb.prepare(dev), bb.prepare(adj_dev, fb.partials)
        tf = median_us(lambda: f.launch())
        tb = median_us(lambda: b.launch())
        fbytes, bbytes = (2 * k + 1) * E * 4, (2 * k + 1) * E * 4
        fv = P.alloc_forward(f"prod_tanh_{k}", dev, want_partials=False)
        rb = P.alloc_recompute(fb.op_id, dev, adj_dev, [x.shape for x in xs])
        v, r = fv.prepare(dev), P.PreparedRecompute(fb.op_id, dev, adj_dev, rb.grads, rb.workspace)
        tv = median_us(lambda: v.launch())
        tr = median_us(lambda: r.launch())
        rbytes = (2 * k + 1) * E * 4
        print(f"{k:3d} {tf:9.2f} {fbytes / tf / 1e3:9.1f} {fbytes / tf / 1e3 / 80:7.1f} {tb:9.2f} "
              f"{bbytes / tb / 1e3:9.1f} {bbytes / tb / 1e3 / 80:7.1f} | {tv:9.2f} {tr:9.2f} {rbytes / tr / 1e3:8.1f} "
              f"{(tv + tr) / (tf + tb):18.2f}", flush=True)
        del dev, _s1, fb, bb, f, b, fv, rb, v, r
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()

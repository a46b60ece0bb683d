"""Roofline calibration with the library's stream probe.

  python -m paper_1810_08297_amd.probe [--rows 4096 --cols 1024]

Prints the rate at which one MI355X moves N read planes + M written planes of fp32
with the tiled kernels' access pattern and no arithmetic: the ceiling any kernel with
that plane mix can hope for.  Three situations per mix: the probe launched back to
back on its own, after a 1 GiB copy that flushes the caches, and (for the HM-LSTM
mix) alternating forward-like and backward-like launches on the same planes, which is
what a training step does.
"""
from __future__ import annotations

import argparse

import numpy as np


def main():
    import torch
    import paper_1810_08297_amd as P

    ap = argparse.ArgumentParser()
    ap.add_argument("--rows", type=int, default=4096)
    ap.add_argument("--cols", type=int, default=1024)
    ap.add_argument("--staggered", type=int, default=1)
    ap.add_argument("--stagger-bytes", type=int, default=-1,
                    help="place plane k at k * (plane bytes + this) in one buffer instead of using the library's slab layout")
    ap.add_argument("--mix", action="append", default=[], help="R,W: a mix of R read and W written planes (repeatable)")
    ap.add_argument("--lds-kib", type=int, default=0,
                    help="KiB of unused dynamic LDS per block: limits the blocks per CU (48 = three); 0 = no limit")
    ap.add_argument("--nt-loads", type=int, default=1, help="1 = nontemporal loads (what the kernels use), 0 = plain")
    a = ap.parse_args()
    opt_fwd = P.Options(probe_nt_loads=a.nt_loads, probe_lds_kib=a.lds_kib, reverse_tiles=0)  # chunks first to last
    E = a.rows * a.cols
    assert E % 1024 == 0
    chunks = E // 1024

    def planes(n):
        if a.stagger_bytes >= 0 and n > 0:
            stride = E * 4 + a.stagger_bytes
            slab = torch.empty((n * stride + 4096) // 4, dtype=torch.float32, device="cuda").normal_()
            base = (slab.data_ptr() + 4095) // 4096 * 4096
            return [base + k * stride for k in range(n)], slab
        t, slab = P.alloc_planes([(a.rows, a.cols)] * n, torch.float32, "cuda", bool(a.staggered))
        for x in t:
            x.normal_()
        return [x.data_ptr() for x in t], (t, slab)

    def ev():
        return torch.cuda.Event(enable_timing=True)

    big_a = torch.empty(256 << 20, dtype=torch.float32, device="cuda").normal_()
    big_b = torch.empty_like(big_a)

    def timed(fn, before=None, n=20):
        ts = []
        for _ in range(n + 3):
            if before is not None:
                before()
            e0, e1 = ev(), ev()
            e0.record()
            fn()
            e1.record()
            ts.append((e0, e1))
        torch.cuda.synchronize()
        return float(np.median([x.elapsed_time(y) for x, y in ts[3:]])) * 1e3

    print(f"planes of {a.rows} x {a.cols} fp32 ({E * 4 / 2**20:.0f} MiB), staggered layout: {bool(a.staggered)}, "
          f"nontemporal loads: {bool(a.nt_loads)}, dynamic LDS per block: {a.lds_kib} KiB")
    print(f"{'mix':>12s} {'back to back':>24s} {'after a 1 GiB copy':>24s}")
    mixes = [tuple(int(x) for x in m.split(",")) for m in a.mix]
    for nin, nout in mixes or ((1, 1), (2, 4), (4, 2), (7, 22), (22, 6), (8, 8), (16, 16), (29, 0), (0, 29)):
        ip, k1 = planes(nin)
        op, k2 = planes(nout)
        fn = lambda: P.bcast_dual_stream_probe(ip, [1024] * nin, op, [1024] * nout, chunks, options=opt_fwd)
        byt = (nin + nout) * E * 4
        t1 = timed(fn)
        t2 = timed(fn, before=lambda: big_b.copy_(big_a))
        print(f"{nin:4d}r + {nout:2d}w {t1:10.1f} us {byt / t1 / 1e3:8.1f} GB/s {t2:10.1f} us {byt / t2 / 1e3:8.1f} GB/s",
              flush=True)
        del k1, k2
    if mixes:
        return
    # a training step: 7 arguments -> 2 outputs + 20 planes, then 2 adjoints + 20 planes -> 6 gradients
    args, k1 = planes(7)
    outs, k2 = planes(22)
    adj, k3 = planes(2)
    grads, k4 = planes(6)
    for reverse in (0, 1):  # the backward-like launch walks its chunks first to last / last to first
        tf, tb = [], []
        for it in range(40):
            e0, e1, e2 = ev(), ev(), ev()
            e0.record()
            P.bcast_dual_stream_probe(args, [1024] * 7, outs, [1024] * 22, chunks, options=opt_fwd)
            e1.record()
            P.bcast_dual_stream_probe(adj + outs[2:], [1024] * 22, grads, [1024] * 6, chunks,
                                      options=opt_fwd.replace(reverse_tiles=reverse))
            e2.record()
            tf.append((e0, e1))
            tb.append((e1, e2))
        torch.cuda.synchronize()
        f = float(np.median([x.elapsed_time(y) for x, y in tf[5:]])) * 1e3
        b = float(np.median([x.elapsed_time(y) for x, y in tb[5:]])) * 1e3
        print(f"alternating, backward-like {'last to first' if reverse else 'first to last'}: forward-like 7r+22w {f:.1f} us "
              f"{29 * E * 4 / f / 1e3:.1f} GB/s | backward-like 22r+6w {b:.1f} us {28 * E * 4 / b / 1e3:.1f} GB/s | "
              f"step {f + b:.1f} us {57 * E * 4 / (f + b) / 1e3:.1f} GB/s")


if __name__ == "__main__":
    main()

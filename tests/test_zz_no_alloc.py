"""The backward entry point that allocates nothing (bcast_dual_backward_noalloc): same results, bit for
bit, as bcast_dual_backward with a caller's workspace; on two calls in a row that share the library's
static scratch array, the second on a smaller input."""
import numpy as np
import pytest
import torch

import oracle
import paper_1810_08297_amd as P
from gpu_util import check_close, to_dev
from paper_1810_08297_amd import inputs

pytestmark = pytest.mark.gpu


def _problem(op, args, adj):
    dev, adj_dev = [to_dev(a) for a in args], [to_dev(a) for a in adj]
    fb = P.alloc_forward(op, dev).run(dev)
    shapes = [args[j].shape for j in oracle.diff_arg_indices(op, len(args))]
    ref = P.alloc_backward(adj_dev, fb.partials, shapes)
    ref.run(adj_dev, fb.partials)
    torch.cuda.synchronize()
    return dev, adj_dev, fb, shapes, ref


def test_noalloc_backward_matches_backward_on_two_calls_in_a_row():
    # first call: config 4 at a quarter of its extents (column sums, row sums and a full sum through the
    # second pass: 2048 x 2048, workspace in use); second call: a smaller, ragged problem of the same op
    op, args, adj = inputs.config_inputs(4, scale=1 / 4)
    big = _problem(op, args, adj)
    rng = np.random.default_rng(17)
    R, C = 300, 1100
    small_args = [rng.standard_normal((R, C)).astype(np.float32), rng.uniform(0.1, 2, (R, C)).astype(np.float32),
                  rng.standard_normal((1, C)).astype(np.float32), rng.standard_normal((R, 1)).astype(np.float32),
                  rng.standard_normal((1, 1)).astype(np.float32)]
    small_adj = [rng.standard_normal((R, C)).astype(np.float32)]
    small = _problem(op, small_args, small_adj)
    for what, (dev, adj_dev, fb, shapes, ref), host_adj in (("first call", big, adj), ("second, smaller call", small, small_adj)):
        assert P.bcast_dual_backward_workspace(adj_dev, fb.partials, ref.grads) > 0, "the case must use the scratch memory"
        grads, _ = P.alloc_planes(shapes, adj_dev[0].dtype, "cuda")
        for g in grads:
            g.fill_(float("nan"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        P.bcast_dual_backward_noalloc(adj_dev, fb.partials, grads)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        for k, (g, w) in enumerate(zip(grads, ref.grads)):
            assert torch.equal(g, w), f"{what}: gradient {k} differs from bcast_dual_backward's"
        want = oracle.backward(host_adj, [p.cpu().numpy() for p in fb.partials], shapes, threads=8)
        for k, (g, w) in enumerate(zip(grads, want)):
            check_close(g.cpu().numpy(), w, f"{what}: gradient {k}")

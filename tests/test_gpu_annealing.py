"""Gossip's consensus floor moves with the step size (Section 4.3: after the
step size is annealed, gossiping SGD's replicas agree less well relative to
it than all-reduce's, which stay identical).  On the quadratic, with the
experiments' local step (Nesterov 0.9, weight decay 1e-4, Section 4.2) and the
step size annealed by 0.1 twice: the consensus distance settles on a plateau
per stage; the GPU's plateaus equal the oracle's to 1e-4, follow the
second-moment prediction of paper_1611_04581_amd.theory within 20 %, and drop
by about the square of the anneal factor; under all-reduce the consensus
distance is exactly zero throughout."""
import numpy as np
import pytest

from paper_1611_04581_amd import theory, workloads as W
from parity_util import assert_rows_close

pytestmark = pytest.mark.gpu
SEED = W.DEFAULT_SEED


def test_consensus_floor_through_annealing(oracle):
    import torch
    from paper_1611_04581_amd import gsgd as G
    k, d = 16, 60 * 1024 + 9
    ld = W.round_up(d, 1024)
    mu, sigma, wd = 0.9, 0.1, 1e-4
    stages, steps, tail = (0.1, 0.01, 0.001), 160, 30
    inp = W.make_inputs(k, d, ld, seed=61)
    xo = np.tile(inp.x0, (k, 1)).copy()                   # every node starts at the same point
    vo, go = np.zeros_like(xo), np.zeros_like(xo)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    with G.Context(k, d, ld, lr=stages[0], momentum=mu, sigma=sigma, seed=SEED) as ctx, \
         G.Context(k, d, ld, lr=stages[0], momentum=mu, sigma=sigma, seed=SEED) as ctx_ar:
        for c in (ctx, ctx_ar):
            c.set_local_step(wd, True)
        x, v, g = dev(xo), dev(vo), dev(go)
        xa, va = dev(xo), dev(vo)
        h, xs = dev(inp.h), dev(inp.xstar)
        t, gpu_floor, cpu_floor, pred = 0, [], [], []
        for lr in stages:
            ctx.set_lr(lr)
            ctx_ar.set_lr(lr)
            cg, co = [], []
            for s in range(steps):
                perm = G.make_perm(SEED, t, k)
                ctx.gen_grad(x, h, xs, g, t)
                ctx.step_gossip(x, v, g, perm, 0.5)
                oracle.gen_grad(xo, inp.h, inp.xstar, go, sigma, SEED, t, 0, n=d)
                oracle.step_gossip_ext(xo, vo, go, lr, mu, 0.5, perm, wd=wd, nesterov=True, n=d)
                ctx_ar.gen_grad(xa, h, xs, g, t)
                ctx_ar.step_allreduce(xa, va, g)
                t += 1
                if s >= steps - tail:
                    cg.append(ctx.stats(x, xs)[0])
                    co.append(oracle.stats(xo, inp.xstar, n=d)[0])
            assert ctx_ar.stats(xa, xs)[0] == 0.0           # all-reduce: the replicas never part
            gpu_floor.append(np.mean(cg))
            cpu_floor.append(np.mean(co))
            pred.append(k * theory.gossip_consensus_floor(inp.h[:d], lr, mu, sigma, k, 0.5, wd, True).sum())
        assert_rows_close(x.cpu().numpy()[:, :d], xo[:, :d], "x after the schedule")
    for a, b, p in zip(gpu_floor, cpu_floor, pred):
        assert abs(a / b - 1.0) <= 1e-4, (gpu_floor, cpu_floor)
        assert abs(a / p - 1.0) <= 0.2, (gpu_floor, pred)
    for s in (0, 1):
        ratio = gpu_floor[s] / gpu_floor[s + 1]
        assert 50 < ratio < 150                             # the floor scales with the square of the step size
        assert abs(ratio / (pred[s] / pred[s + 1]) - 1.0) <= 0.2

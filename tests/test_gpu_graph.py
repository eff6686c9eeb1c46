"""The step calls only enqueue kernels on the caller's stream (no allocation,
no memset, no synchronisation; the tile tickets reset themselves), so a caller
can record a run of them into a HIP graph.  Every replay must reproduce the
eager result and the oracle's, with ordinary eager work between replays."""
import numpy as np
import pytest

from paper_1611_04581_amd import workloads as W
from parity_util import assert_bitwise

pytestmark = pytest.mark.gpu

SEED = 0x161104581


@pytest.mark.parametrize("b", [0, 2048])
def test_captured_steps_replay_like_eager_runs(oracle, b):
    """b = 0: row-major matrices (the gossip steps run as walks along the peer map); b = 2048: blocked matrices (two
    ascending sweeps, the generator and the local step as row walks)."""
    import torch
    from paper_1611_04581_amd import gsgd as G
    k, d, steps = 8, 9 * 1024 + 5, 6
    ld = W.round_up(d, b or 1024)
    inp = W.make_inputs(k, d, ld, seed=81)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    mat = (lambda a: dev(W.to_blocked(a, b))) if b else dev                     # a matrix in the context's layout
    rows = (lambda t: W.from_blocked(t.cpu().numpy(), b)) if b else (lambda t: t.cpu().numpy())
    # what the run must produce, from the oracle
    xo, vo, go, co = inp.x.copy(), inp.v.copy(), inp.g.copy(), inp.center.copy()
    for t in range(steps):
        oracle.gen_grad(xo, inp.h, inp.xstar, go, 0.1, SEED, t, 1, n=d)
        if t % 3 == 0:
            oracle.step_gossip(xo, vo, go, 0.05, 0.9, 0.5, oracle.make_perm(SEED, t, k), n=d)
        elif t % 3 == 1:
            oracle.step_gossip(xo, vo, go, 0.05, 0.9, 0.5, oracle.make_targets(SEED, t, k), n=d)
        else:
            oracle.step_easgd(xo, vo, go, co, 0.05, 0.9, 0.1, n=d)

    with G.Context(k, d, ld, lr=0.05, momentum=0.9, sigma=0.1, seed=SEED, noise_kind=G.NOISE_UNIFORM,
                   block_columns=b) as ctx:
        x, v, g, c = mat(inp.x), mat(inp.v), mat(inp.g), dev(inp.center)
        h, xs = dev(inp.h), dev(inp.xstar)
        x_init, v_init, c_init = x.clone(), v.clone(), c.clone()
        stats_out = torch.zeros(4, dtype=torch.float64, device="cuda")

        def run():
            for t in range(steps):
                ctx.gen_grad(x, h, xs, g, t)
                if t % 3 == 0:
                    ctx.step_gossip(x, v, g, G.make_perm(SEED, t, k), 0.5)
                elif t % 3 == 1:
                    ctx.step_gossip_pull(x, v, g, G.make_targets(SEED, t, k), 0.5)
                else:
                    ctx.step_easgd(x, v, g, c, 0.1)
            # the statistics call that neither allocates nor waits can be recorded with the steps
            G.stats_static(k, d, ld, x, xs, stats_out, block_columns=b)

        run()                                            # eager
        torch.cuda.synchronize()
        assert_bitwise(rows(x), xo, "eager x")
        assert_bitwise(c.cpu().numpy(), co, "eager center")

        x.copy_(x_init); v.copy_(v_init); c.copy_(c_init)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run()                                        # recorded, not executed
        for replay in range(3):
            x.copy_(x_init); v.copy_(v_init); c.copy_(c_init)
            graph.replay()
            torch.cuda.synchronize()
            assert_bitwise(rows(x), xo, "replay %d x" % replay)
            assert_bitwise(rows(v), vo, "replay %d v" % replay)
            assert_bitwise(c.cpu().numpy(), co, "replay %d center" % replay)
            recorded = stats_out.cpu().numpy().copy()
            assert np.array_equal(recorded, ctx.stats(x, xs)), "replay %d statistics" % replay
            assert np.allclose(recorded, oracle.stats(xo, inp.xstar, n=d), rtol=1e-11, atol=0)
            stats_out.fill_(-1.0)
            # unrelated eager work through the same context between replays
            scratch_x, scratch_v = x.clone(), v.clone()
            ctx.step_allreduce(scratch_x, scratch_v, g)
            ctx.stats(scratch_x, xs)

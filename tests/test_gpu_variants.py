"""GPU parity for the variants beyond the algorithm boxes: the local step with
weight decay and Nesterov momentum (the paper's training setup, Section 4.2),
gossip with stale parameters (Section 6.2.1), and the local-only step used
between exchanges when the communication period is larger than 1.

All of these are fixed-order fp32 / fp64 arithmetic, so the bar is bit
equality with the CPU oracle on the same seeded inputs.
"""
import numpy as np
import pytest

from paper_1611_04581_amd import workloads as W
from parity_util import assert_bitwise, assert_rows_close

pytestmark = pytest.mark.gpu

SEED = 0x161104581
SHAPES = [(4, 5 * 1024 + 7, None), (3, 1, 4), (7, 1023, 1024), (32, 2 * 1024 + 2, 4096)]
LOCAL_STEPS = [(1e-4, False), (0.0, True), (1e-4, True), (0.03, True)]


@pytest.fixture(scope="module")
def G():
    import torch
    from paper_1611_04581_amd import gsgd
    assert torch.cuda.is_available()
    gsgd.lib()
    return gsgd


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.cpu().numpy()


def some_perms(k, oracle):
    out = [[(i + 1) % k for i in range(k)], [int(t) for t in oracle.make_perm(SEED, 5, k)]]
    if k >= 6:
        out.append([1, 2, 0, 3] + list(range(5, k)) + [4])
    return out


@pytest.mark.parametrize("k,d,ld", SHAPES)
@pytest.mark.parametrize("wd,nesterov", LOCAL_STEPS)
def test_gossip_with_weight_decay_and_nesterov(G, oracle, k, d, ld, wd, nesterov):
    ld = ld or W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=21)
    with G.Context(k, d, ld, lr=0.05, momentum=0.9) as ctx:
        ctx.set_local_step(wd, nesterov)
        for perm in some_perms(k, oracle):
            for stale in (False, True):
                x, v = dev(inp.x), dev(inp.v)
                (ctx.step_gossip_stale if stale else ctx.step_gossip)(x, v, dev(inp.g), perm, 0.5)
                xo, vo = inp.x.copy(), inp.v.copy()
                oracle.step_gossip_ext(xo, vo, inp.g, 0.05, 0.9, 0.5, perm, wd=wd, nesterov=nesterov, stale=stale,
                                       n=d)
                assert_bitwise(host(x), xo, "x perm=%s stale=%s" % (perm, stale))
                assert_bitwise(host(v), vo, "v")


@pytest.mark.parametrize("k,d,ld", SHAPES)
def test_stale_gossip_plain_local_step(G, oracle, k, d, ld):
    ld = ld or W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=22)
    with G.Context(k, d, ld, lr=0.05, momentum=0.9) as ctx:
        for beta in (0.5, 0.25):
            for perm in some_perms(k, oracle) + [list(range(k))]:
                x, v = dev(inp.x), dev(inp.v)
                ctx.step_gossip_stale(x, v, dev(inp.g), perm, beta)
                xo, vo = inp.x.copy(), inp.v.copy()
                oracle.step_gossip_ext(xo, vo, inp.g, 0.05, 0.9, beta, perm, stale=True, n=d)
                assert_bitwise(host(x), xo, "x perm=%s" % perm)
                assert_bitwise(host(v), vo, "v")


@pytest.mark.parametrize("k,d,ld", SHAPES)
@pytest.mark.parametrize("wd,nesterov", LOCAL_STEPS)
def test_allreduce_and_easgd_with_weight_decay_and_nesterov(G, oracle, k, d, ld, wd, nesterov):
    ld = ld or W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=23)
    with G.Context(k, d, ld, lr=0.05, momentum=0.9) as ctx:
        ctx.set_local_step(wd, nesterov)
        x, v = dev(inp.x), dev(inp.v)
        ctx.step_allreduce(x, v, dev(inp.g))
        xo, vo = inp.x.copy(), inp.v.copy()
        oracle.step_allreduce_ext(xo, vo, inp.g, 0.05, 0.9, wd=wd, nesterov=nesterov, n=d)
        assert_bitwise(host(x), xo, "allreduce x")
        assert_bitwise(host(v), vo, "allreduce v")

        x, v, c = dev(inp.x), dev(inp.v), dev(inp.center)
        ctx.step_easgd(x, v, dev(inp.g), c, 0.9 / k)
        xo, vo, co = inp.x.copy(), inp.v.copy(), inp.center.copy()
        oracle.step_easgd_ext(xo, vo, inp.g, co, 0.05, 0.9, 0.9 / k, wd=wd, nesterov=nesterov, n=d)
        assert_bitwise(host(x), xo, "easgd x")
        assert_bitwise(host(v), vo, "easgd v")
        assert_bitwise(host(c), co, "easgd center")


@pytest.mark.parametrize("k,d,ld", SHAPES)
@pytest.mark.parametrize("wd,nesterov", [(0.0, False)] + LOCAL_STEPS)
def test_local_step_alone(G, oracle, k, d, ld, wd, nesterov):
    """The local step is the gossip step against oneself (the mix term is zero)."""
    ld = ld or W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=24)
    with G.Context(k, d, ld, lr=0.05, momentum=0.9) as ctx:
        ctx.set_local_step(wd, nesterov)
        x, v = dev(inp.x), dev(inp.v)
        ctx.step_local(x, v, dev(inp.g))
        xo, vo = inp.x.copy(), inp.v.copy()
        oracle.step_gossip_ext(xo, vo, inp.g, 0.05, 0.9, 0.5, list(range(k)), wd=wd, nesterov=nesterov, n=d)
        assert_bitwise(host(x), xo, "x")
        assert_bitwise(host(v), vo, "v")


def test_segmented_layout_with_the_extended_local_step(G, oracle):
    k, d = 6, 7 * 1024 + 3
    ld = W.round_up(d, 4)
    off, sc = W.random_segments(d, 37, seed=3, align=1)
    lrc = oracle.expand_lr(0.05, d, off, sc)
    inp = W.make_inputs(k, d, ld, seed=25)
    perm = [int(t) for t in oracle.make_perm(SEED, 1, k)]
    with G.Context(k, d, ld, lr=0.05, momentum=0.9, seg_offsets=off, seg_lr_scale=sc) as ctx:
        ctx.set_local_step(1e-4, True)
        x, v = dev(inp.x), dev(inp.v)
        ctx.step_gossip_stale(x, v, dev(inp.g), perm, 0.5)
        xo, vo = inp.x.copy(), inp.v.copy()
        oracle.step_gossip_ext(xo, vo, inp.g, lrc, 0.9, 0.5, perm, wd=1e-4, nesterov=True, stale=True, n=d)
        assert_bitwise(host(x), xo, "stale gossip x")
        x, v = dev(inp.x), dev(inp.v)
        ctx.step_allreduce(x, v, dev(inp.g))
        xo, vo = inp.x.copy(), inp.v.copy()
        oracle.step_allreduce_ext(xo, vo, inp.g, lrc, 0.9, wd=1e-4, nesterov=True, n=d)
        assert_bitwise(host(x), xo, "allreduce x")
        assert_bitwise(host(v), vo, "allreduce v")
        x, v = dev(inp.x), dev(inp.v)
        ctx.step_local(x, v, dev(inp.g))
        xo, vo = inp.x.copy(), inp.v.copy()
        oracle.step_gossip_ext(xo, vo, inp.g, lrc, 0.9, 0.0, list(range(k)), wd=1e-4, nesterov=True, n=d)
        assert_bitwise(host(x), xo, "local x")


@pytest.mark.parametrize("kind", [1, 0])
def test_fused_generator_with_the_extended_local_step(G, oracle, kind):
    k, d = 8, 3 * 1024 + 6
    ld = W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=26)
    perm = [int(t) for t in oracle.make_perm(SEED, 2, k)]
    with G.Context(k, d, ld, sigma=0.2, seed=SEED, noise_kind=kind) as ctx:
        ctx.set_local_step(1e-4, True)
        xb, vb = dev(inp.x), dev(inp.v)
        ctx.step_gossip_fused(xb, vb, dev(inp.h), dev(inp.xstar), perm, 17, 0.5)
        xo, vo, go = inp.x.copy(), inp.v.copy(), inp.g.copy()
        oracle.gen_grad(xo, inp.h, inp.xstar, go, 0.2, SEED, 17, kind, n=d)
        oracle.step_gossip_ext(xo, vo, go, 0.05, 0.9, 0.5, perm, wd=1e-4, nesterov=True, n=d)
        if kind == 1:
            assert_bitwise(host(xb), xo, "x")
            assert_bitwise(host(vb), vo, "v")
        else:
            assert_rows_close(host(xb)[:, :d], xo[:, :d], "x")


def test_training_setup_trajectory_with_period_and_annealing(G, oracle):
    """The paper's schedule in miniature: Nesterov 0.9, weight decay 1e-4,
    exchange every tau = 10 iterations, step size annealed by 0.1 twice."""
    k, d, steps, tau = 8, 5 * 1024 + 3, 60, 10
    ld = W.round_up(d, 1024)
    inp = W.make_inputs(k, d, ld, seed=27)
    lr = 0.1
    xo, vo, go = inp.x.copy(), inp.v.copy(), inp.g.copy()
    oracle.init_replicas(xo, vo, None, inp.x0, SEED, 0, n=d)
    exchanges = 0
    with G.Context(k, d, ld, lr=lr, momentum=0.9, sigma=0.05, seed=SEED, noise_kind=G.NOISE_UNIFORM) as ctx:
        ctx.set_local_step(1e-4, True)
        x, v, g = dev(inp.x), dev(inp.v), dev(inp.g)
        h, xs = dev(inp.h), dev(inp.xstar)
        ctx.init_replicas(x, v, None, dev(inp.x0), G.INIT_BROADCAST)
        for t in range(steps):
            if t in (20, 40):
                lr *= 0.1
                ctx.set_lr(lr)
            ctx.gen_grad(x, h, xs, g, t)
            oracle.gen_grad(xo, inp.h, inp.xstar, go, 0.05, SEED, t, 1, n=d)
            if G.comm_due(t, tau):
                exchanges += 1
                perm = G.make_perm(SEED, t, k)
                ctx.step_gossip(x, v, g, perm, 0.5)
            else:
                perm = list(range(k))
                ctx.step_local(x, v, g)
            oracle.step_gossip_ext(xo, vo, go, np.float32(lr), 0.9, 0.5, perm, wd=1e-4, nesterov=True, n=d)
        assert exchanges == steps // tau
        assert_bitwise(host(x), xo, "x")
        assert_bitwise(host(v), vo, "v")


# ----------------------------------------------------------------------------
# pull-gossip on arbitrary maps (iid targets: several replicas may pull from one)

def some_maps(k, oracle):
    rng = np.random.default_rng(100 + k)
    maps = [[0] * k, [max(i - 1, 0) for i in range(k)], [i // 2 for i in range(k)],
            [(i - 1) // 3 if i else 0 for i in range(k)], [(i + 1) % k for i in range(k)]]
    maps += [[int(t) for t in oracle.make_targets(SEED, s, k)] for s in range(4)]
    maps += [[int(t) for t in rng.integers(0, k, size=k)] for _ in range(3)]
    return maps


@pytest.mark.parametrize("k,d,ld", SHAPES + [(128, 1024 + 12, None)])
def test_pull_gossip_on_arbitrary_maps(G, oracle, k, d, ld):
    ld = ld or W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=31)
    with G.Context(k, d, ld, lr=0.05, momentum=0.9) as ctx:
        for peer in some_maps(k, oracle):
            assert np.array_equal(G.make_targets(SEED, 3, k), oracle.make_targets(SEED, 3, k))
            for stale in (False, True):
                x, v = dev(inp.x), dev(inp.v)
                ctx.step_gossip_pull(x, v, dev(inp.g), peer, 0.5, stale)
                xo, vo = inp.x.copy(), inp.v.copy()
                if stale:
                    oracle.step_gossip_ext(xo, vo, inp.g, 0.05, 0.9, 0.5, peer, stale=True, n=d)
                else:
                    oracle.step_gossip(xo, vo, inp.g, 0.05, 0.9, 0.5, peer, n=d)
                assert_bitwise(host(x), xo, "x peer=%s stale=%s" % (peer, stale))
                assert_bitwise(host(v), vo, "v")
        ctx.set_local_step(1e-4, True)
        for peer in some_maps(k, oracle)[5:8]:
            x, v = dev(inp.x), dev(inp.v)
            ctx.step_gossip_pull(x, v, dev(inp.g), peer, 0.3)
            xo, vo = inp.x.copy(), inp.v.copy()
            oracle.step_gossip_ext(xo, vo, inp.g, 0.05, 0.9, 0.3, peer, wd=1e-4, nesterov=True, n=d)
            assert_bitwise(host(x), xo, "x peer=%s nesterov" % peer)
        with pytest.raises(G.GsgdError) as e:
            ctx.step_gossip_pull(x, v, dev(inp.g), [k] * k, 0.5)
        assert e.value.code == G.ERR_BAD_PERM


def test_pull_gossip_max_replicas_deep_and_bushy_maps(G, oracle):
    k, d = G.MAX_K, 1024 + 4
    inp = W.make_inputs(k, d, seed=32)
    maps = [[max(i - 1, 0) for i in range(k)],                  # one chain of 512
            [(i - 1) // 2 if i else 0 for i in range(k)],       # complete binary tree: the most stack slots
            [int(t) for t in oracle.make_targets(SEED, 11, k)]]
    with G.Context(k, d) as ctx:
        for peer in maps:
            x, v = dev(inp.x), dev(inp.v)
            ctx.step_gossip_pull(x, v, dev(inp.g), peer, 0.5)
            xo, vo = inp.x.copy(), inp.v.copy()
            oracle.step_gossip(xo, vo, inp.g, 0.05, 0.9, 0.5, peer)
            assert_bitwise(host(x), xo, "x")
            assert_bitwise(host(v), vo, "v")


def test_iid_pull_gossip_trajectory_and_theorem_bound(G, oracle):
    """Synchronous pull-gossip with iid targets and no momentum, the setting of
    the paper's first theorem: the trajectory is bit-exact against the oracle
    and the summed squared distance to the optimum stays under the theorem's
    bound (m = min h, L = max h) at every checked step."""
    k, d, steps = 16, 6 * 1024 + 2, 60
    ld = W.round_up(d, 1024)
    lr, sigma = 0.5, 0.05
    inp = W.make_inputs(k, d, ld, seed=33)
    xo, vo, go = inp.x.copy(), inp.v.copy(), inp.g.copy()
    oracle.init_replicas(xo, vo, None, inp.x0, SEED, 0, n=d)
    m, L = float(inp.h[:d].min()), float(inp.h[:d].max())
    assert lr <= 2.0 / (m + L)
    rate = 1.0 - 2.0 * lr * m * L / (m + L)
    floor = k * lr * sigma**2 * (m + L) / (2 * m * L) * d
    with G.Context(k, d, ld, lr=lr, momentum=0.0, sigma=sigma, seed=SEED, noise_kind=G.NOISE_UNIFORM) as ctx:
        x, v, g = dev(inp.x), dev(inp.v), dev(inp.g)
        h, xs = dev(inp.h), dev(inp.xstar)
        ctx.init_replicas(x, v, None, dev(inp.x0), G.INIT_BROADCAST)
        d0 = ctx.stats(x, xs)[1]
        for t in range(steps):
            peer = G.make_targets(SEED, t, k)
            ctx.gen_grad(x, h, xs, g, t)
            ctx.step_gossip_pull(x, v, g, peer, 0.5)
            oracle.gen_grad(xo, inp.h, inp.xstar, go, sigma, SEED, t, 1, n=d)
            oracle.step_gossip(xo, vo, go, lr, 0.0, 0.5, peer, n=d)
            if t % 10 == 9:
                assert ctx.stats(x, xs)[1] <= rate ** (t + 1) * d0 + floor
        assert_bitwise(host(x), xo, "x")


# ----------------------------------------------------------------------------
# push-gossip (Algorithm 4): average of a variable number of received messages

def assert_push_close(got, want, what):
    """The kernel adds the received values in visiting order, the oracle in
    ascending sender index, both in fp64: the rounded averages agree except
    where an fp64 sum was itself inexact, so nearly every element is bit-equal
    and the rest are within the parameter tolerance."""
    assert_rows_close(got, want, what)
    same = (np.ascontiguousarray(got).view(np.uint32) == np.ascontiguousarray(want).view(np.uint32)).mean()
    assert same >= 0.9999, "%s: only %.6f of the elements are bit-equal" % (what, same)


@pytest.mark.parametrize("k,d,ld", SHAPES + [(128, 1024 + 12, None)])
def test_push_gossip_on_arbitrary_maps(G, oracle, k, d, ld):
    ld = ld or W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=41)
    with G.Context(k, d, ld, lr=0.05, momentum=0.9) as ctx:
        maps = some_maps(k, oracle) + [list(range(k))]
        if k >= 2:
            maps += [[int(t) for t in oracle.make_targets(SEED, s, k, True)] for s in range(3)]
            assert np.array_equal(G.make_targets(SEED, 3, k, True), oracle.make_targets(SEED, 3, k, True))
        for target in maps:
            x, v = dev(inp.x), dev(inp.v)
            ctx.step_gossip_push(x, v, dev(inp.g), target)
            xo, vo = inp.x.copy(), inp.v.copy()
            oracle.step_gossip_push(xo, vo, inp.g, 0.05, 0.9, target, n=d)
            assert_push_close(host(x)[:, :d], xo[:, :d], "x target=%s" % target)
            assert_bitwise(host(x)[:, d:], xo[:, d:], "x padding")
            assert_bitwise(host(v), vo, "v")
        ctx.set_local_step(1e-4, True)
        for target in maps[5:8]:
            x, v = dev(inp.x), dev(inp.v)
            ctx.step_gossip_push(x, v, dev(inp.g), target)
            xo, vo = inp.x.copy(), inp.v.copy()
            oracle.step_gossip_push(xo, vo, inp.g, 0.05, 0.9, target, wd=1e-4, nesterov=True, n=d)
            assert_push_close(host(x)[:, :d], xo[:, :d], "x nesterov target=%s" % target)
            assert_bitwise(host(v), vo, "v")
        with pytest.raises(G.GsgdError) as e:
            ctx.step_gossip_push(x, v, dev(inp.g), [-1] * k)
        assert e.value.code == G.ERR_BAD_PERM


def test_push_gossip_max_replicas_and_segments(G, oracle):
    k, d = G.MAX_K, 1024 + 4
    inp = W.make_inputs(k, d, seed=42)
    off, sc = W.random_segments(d, 9, seed=2, align=1)
    lrc = oracle.expand_lr(0.05, d, off, sc)
    maps = [[max(i - 1, 0) for i in range(k)], [(i - 1) // 2 if i else 0 for i in range(k)], [0] * k,
            [int(t) for t in oracle.make_targets(SEED, 11, k, True)]]
    with G.Context(k, d, seg_offsets=off, seg_lr_scale=sc) as ctx:
        for target in maps:
            x, v = dev(inp.x), dev(inp.v)
            ctx.step_gossip_push(x, v, dev(inp.g), target)
            xo, vo = inp.x.copy(), inp.v.copy()
            oracle.step_gossip_push(xo, vo, inp.g, lrc, 0.9, target)
            assert_push_close(host(x), xo, "x")
            assert_bitwise(host(v), vo, "v")


def test_push_gossip_trajectory(G, oracle):
    """Push-gossip with fresh uniform targets among the other nodes, Gaussian
    gradient noise, 40 steps: parameters within tolerance of the oracle's and
    the replicas pulled together (consensus distance far below a run without
    any exchange)."""
    k, d, steps = 16, 6 * 1024 + 2, 40
    ld = W.round_up(d, 1024)
    inp = W.make_inputs(k, d, ld, seed=43)
    xo, vo, go = inp.x.copy(), inp.v.copy(), inp.g.copy()
    oracle.init_replicas(xo, vo, None, None, SEED, 1, n=d)
    with G.Context(k, d, ld, lr=0.05, momentum=0.9, sigma=0.1, seed=SEED) as ctx:
        x, v, g = dev(xo), dev(vo), dev(inp.g)
        xi, vi = x.clone(), v.clone()                      # the same run without exchanges
        h, xs = dev(inp.h), dev(inp.xstar)
        for t in range(steps):
            target = G.make_targets(SEED, t, k, True)
            ctx.gen_grad(x, h, xs, g, t)
            ctx.step_gossip_push(x, v, g, target)
            oracle.gen_grad(xo, inp.h, inp.xstar, go, 0.1, SEED, t, 0, n=d)
            oracle.step_gossip_push(xo, vo, go, 0.05, 0.9, target, n=d)
            ctx.gen_grad(xi, h, xs, g, t)
            ctx.step_local(xi, vi, g)
        assert_rows_close(host(x)[:, :d], xo[:, :d], "x")
        assert ctx.stats(x, xs)[0] < 0.05 * ctx.stats(xi, xs)[0]


# ----------------------------------------------------------------------------
# asynchronous pull-gossip, tick by tick (Section 6.1.2)

@pytest.mark.parametrize("k,d,ld", SHAPES)
def test_async_tick_with_given_gradient(G, oracle, k, d, ld):
    ld = ld or W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=51)
    pairs = [(0, k - 1), (k - 1, 0), (k // 2, k // 2)] + [G.make_tick(SEED, t, k) for t in range(4)]
    with G.Context(k, d, ld, lr=0.05, momentum=0.9) as ctx:
        for wd, nest in ((0.0, False), (1e-4, True)):
            ctx.set_local_step(wd, nest)
            x, v, g = dev(inp.x), dev(inp.v), dev(inp.g)
            xo, vo = inp.x.copy(), inp.v.copy()
            for (i, j) in pairs:
                ctx.step_async_tick(x, v, g, i, j, 0.5)
                oracle.async_tick(xo, vo, inp.g[i].copy(), 0.05, 0.9, 0.5, i, j, wd=wd, nesterov=nest, n=d)
            assert_bitwise(host(x), xo, "x")
            assert_bitwise(host(v), vo, "v")
        for bad in ((-1, 0), (0, k), (k, 0)):
            with pytest.raises(G.GsgdError) as e:
                ctx.step_async_tick(x, v, g, bad[0], bad[1], 0.5)
            assert e.value.code == G.ERR_INVALID_ARG


@pytest.mark.parametrize("kind", [1, 0])
def test_async_ticks_fused_generator_and_driver(G, oracle, kind):
    """n ticks through gsgd_run_async_ticks (tick draw, gradient generator and
    update all in the library) against the oracle taking the same ticks one by
    one; per-layer step sizes on."""
    k, d, ticks = 6, 5 * 1024 + 3, 40
    ld = W.round_up(d, 1024)
    off, sc = W.random_segments(d, 11, seed=4, align=1)
    lrc = oracle.expand_lr(0.05, d, off, sc)
    inp = W.make_inputs(k, d, ld, seed=52)
    xo, vo = inp.x.copy(), inp.v.copy()
    g_row = np.zeros(ld, np.float32)
    with G.Context(k, d, ld, lr=0.05, momentum=0.9, sigma=0.2, seed=SEED, noise_kind=kind, seg_offsets=off,
                   seg_lr_scale=sc) as ctx:
        x, v = dev(inp.x), dev(inp.v)
        h, xs = dev(inp.h), dev(inp.xstar)
        ctx.run_async_ticks(x, v, h, xs, 5, ticks, 0.5)
        for t in range(5, 5 + ticks):
            i, j = oracle.make_tick(SEED, t, k)
            assert (i, j) == G.make_tick(SEED, t, k)
            oracle.gen_grad_row(xo, inp.h, inp.xstar, g_row, i, 0.2, SEED, t, kind, n=d)
            oracle.async_tick(xo, vo, g_row, lrc, 0.9, 0.5, i, j, n=d)
        if kind == 1:
            assert_bitwise(host(x), xo, "x")
            assert_bitwise(host(v), vo, "v")
        else:
            assert_rows_close(host(x)[:, :d], xo[:, :d], "x")
            assert_bitwise(host(x)[:, d:], xo[:, d:], "x padding")
        # one explicit tick equals one driven tick
        x2, v2 = x.clone(), v.clone()
        i, j = G.make_tick(SEED, 99, k)
        ctx.step_async_tick_fused(x, v, h, xs, i, j, 99, 0.5)
        ctx.run_async_ticks(x2, v2, h, xs, 99, 1, 0.5)
        assert_bitwise(host(x2), host(x), "driver vs explicit")


def test_async_theorem_bounds_on_the_gpu(G, oracle):
    """Both bounds of the asynchronous theorem (distance to the optimum,
    distance to the replica mean) along 1600 ticks run by the library."""
    k, d, ticks = 8, 64 * 1024, 1600
    lr, sigma, beta = 0.5, 0.1, 0.5
    inp = W.make_inputs(k, d, seed=53)
    m_, L_ = float(inp.h.min()), float(inp.h.max())
    rate = 1.0 - 2.0 * lr / k * m_ * L_ / (m_ + L_)
    floor = k * lr * (sigma**2 * d) * (m_ + L_) / (2 * m_ * L_)
    lam = 1.0 - 2 * beta * (1 - beta) / k - 2 * beta**2 / k
    C2 = float(((inp.h * (np.abs(inp.x - inp.xstar)).max(0)) ** 2).sum())
    crate = lam * (1.0 - lr * m_ / k)
    cfloor = lam * lr**2 * (C2 + sigma**2 * d) / (1.0 - crate)
    with G.Context(k, d, lr=lr, momentum=0.0, sigma=sigma, seed=SEED) as ctx:
        x, v = dev(inp.x), dev(np.zeros_like(inp.v))
        h, xs = dev(inp.h), dev(inp.xstar)
        st0 = ctx.stats(x, xs)
        for t0 in range(0, ticks, 200):
            ctx.run_async_ticks(x, v, h, xs, t0, 200, beta)
            st = ctx.stats(x, xs)
            assert st[1] <= 1.05 * (rate ** (t0 + 200) * st0[1] + floor)
            assert st[0] <= 1.05 * (crate ** (t0 + 200) * st0[0] + cfloor)
        assert st[1] < 0.05 * st0[1] and st[0] < 0.05 * st0[0]


@pytest.mark.parametrize("k,d,ld", SHAPES)
def test_easgd_one_client_at_a_time(G, oracle, k, d, ld):
    """Algorithm 2 as a client/server exchange: clients take turns, the centre
    moves after every one of them."""
    ld = ld or W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=61)
    order = [int(i) for i in np.random.default_rng(k).integers(0, k, size=2 * k)]
    with G.Context(k, d, ld, lr=0.05, momentum=0.9) as ctx:
        for wd, nest in ((0.0, False), (1e-4, True)):
            ctx.set_local_step(wd, nest)
            x, v, g, c = dev(inp.x), dev(inp.v), dev(inp.g), dev(inp.center)
            xo, vo, co = inp.x.copy(), inp.v.copy(), inp.center.copy()
            for i in order:
                ctx.step_easgd_tick(x, v, g, c, i, 0.9 / k)
                oracle.easgd_tick(xo, vo, inp.g[i].copy(), co, 0.05, 0.9, 0.9 / k, i, wd=wd, nesterov=nest, n=d)
            assert_bitwise(host(x), xo, "x")
            assert_bitwise(host(v), vo, "v")
            assert_bitwise(host(c), co, "center")
        with pytest.raises(G.GsgdError):
            ctx.step_easgd_tick(x, v, g, c, k, 0.1)


# ----------------------------------------------------------------------------
# row norms and the diffusion potential (Section 3.1)

@pytest.mark.parametrize("k,d,ld", SHAPES + [(128, 300 * 1024 + 5, None)])
def test_row_sqnorms(G, oracle, k, d, ld):
    ld = ld or W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=71)
    with G.Context(k, d, ld) as ctx:
        got = ctx.row_sqnorms(dev(inp.x))
    want = (inp.x[:, :d].astype(np.float64) ** 2).sum(1)
    assert np.allclose(got, want, rtol=1e-12, atol=0)


@pytest.mark.parametrize("kind", ["pull", "push"])
def test_diffusion_potential_along_pure_gossip_rounds(G, oracle, kind):
    """Gossip rounds without gradient steps on the device; the potential from
    the library (row norms on the device, weights on the host) against the
    oracle's term-by-term definition on the starting vectors."""
    k, d = 8, 3 * 1024 + 2
    ld = W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=72)
    theta0 = inp.x[:, :d].astype(np.float64)
    V = np.eye(k)
    Vo = np.eye(k)
    with G.Context(k, d, ld, lr=0.0, momentum=0.0) as ctx:
        x, v, g = dev(inp.x), dev(np.zeros_like(inp.v)), dev(np.zeros_like(inp.g))
        n0 = ctx.row_sqnorms(x)
        phi0 = G.diffusion_potential(V, n0, n0)
        assert np.isclose(phi0, oracle.diffusion_potential(theta0, Vo), rtol=1e-10)
        last = phi0
        for r in range(10):
            if kind == "pull":
                peer = G.make_targets(SEED, r, k)
                ctx.step_gossip_pull(x, v, g, peer, 0.5)
                G.weights_pull(V, peer, 0.5)
                Vo = oracle.mixing_matrix_pull(peer, 0.5) @ Vo
            else:
                target = G.make_targets(SEED, r, k, True)
                ctx.step_gossip_push(x, v, g, target)
                G.weights_push(V, target)
                Vo = oracle.mixing_matrix_push(target) @ Vo
            phi = G.diffusion_potential(V, n0, ctx.row_sqnorms(x))
            assert np.isclose(phi, oracle.diffusion_potential(theta0, Vo), rtol=1e-5)
            last = phi
        assert last < 0.3 * phi0
        # the device rows are the weighted averages the weights say they are
        assert np.allclose(host(x)[:, :d], Vo @ theta0, rtol=0, atol=1e-5)


# ----------------------------------------------------------------------------
# generator-fused forms of pull- and push-gossip

@pytest.mark.parametrize("kind", [1, 0])
def test_fused_generator_pull_and_push(G, oracle, kind):
    """g never touches memory: the fused calls must equal gen_grad followed by
    the step call, and the oracle."""
    k, d = 12, 4 * 1024 + 6
    ld = W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=91)
    peer = [int(t) for t in oracle.make_targets(SEED, 4, k)]
    perm = [int(t) for t in oracle.make_perm(SEED, 4, k)]
    target = [int(t) for t in oracle.make_targets(SEED, 5, k, True)]
    with G.Context(k, d, ld, sigma=0.2, seed=SEED, noise_kind=kind) as ctx:
        h, xs = dev(inp.h), dev(inp.xstar)
        for wd, nest in ((0.0, False), (1e-4, True)):
            ctx.set_local_step(wd, nest)
            for name, the_map, stale in (("pull", peer, False), ("pull", peer, True), ("pull", perm, True),
                                         ("push", target, False)):
                xa, va, g = dev(inp.x), dev(inp.v), dev(inp.g)
                xb, vb = dev(inp.x), dev(inp.v)
                xo, vo, go = inp.x.copy(), inp.v.copy(), inp.g.copy()
                ctx.gen_grad(xa, h, xs, g, 23)
                oracle.gen_grad(xo, inp.h, inp.xstar, go, 0.2, SEED, 23, kind, n=d)
                if name == "pull":
                    ctx.step_gossip_pull(xa, va, g, the_map, 0.5, stale)
                    ctx.step_gossip_pull_fused(xb, vb, h, xs, the_map, 23, 0.5, stale)
                    oracle.step_gossip_ext(xo, vo, go, 0.05, 0.9, 0.5, the_map, wd=wd, nesterov=nest, stale=stale, n=d)
                else:
                    ctx.step_gossip_push(xa, va, g, the_map)
                    ctx.step_gossip_push_fused(xb, vb, h, xs, the_map, 23)
                    oracle.step_gossip_push(xo, vo, go, 0.05, 0.9, the_map, wd=wd, nesterov=nest, n=d)
                assert_bitwise(host(xb), host(xa), "%s stale=%s: fused vs two kernels, x" % (name, stale))
                assert_bitwise(host(vb), host(va), "fused vs two kernels, v")
                if kind == 1 and name == "pull":
                    assert_bitwise(host(xb), xo, "x against the oracle")
                else:
                    assert_rows_close(host(xb)[:, :d], xo[:, :d], "x against the oracle")
        with pytest.raises(G.GsgdError):
            ctx.step_gossip_pull_fused(xb, vb, h, xs, [k] * k, 0)
        with pytest.raises(G.GsgdError):
            ctx.step_gossip_push_fused(xb, vb, h, xs, target, 2**32)


@pytest.mark.parametrize("width", [1, 5, 100000])
def test_map_walks_with_segments_and_any_launch_width(G, oracle, width):
    """Tree walk (pull), senders-first walk (push) and the stale rule with
    per-layer step sizes, for launch widths below and above the tile count."""
    k, d = 9, 6 * 1024 + 3
    ld = W.round_up(d, 4)
    off, sc = W.random_segments(d, 29, seed=6, align=1)
    lrc = oracle.expand_lr(0.05, d, off, sc)
    inp = W.make_inputs(k, d, ld, seed=92)
    peer = [int(t) for t in oracle.make_targets(SEED, 8, k)]
    target = [int(t) for t in oracle.make_targets(SEED, 9, k, True)]
    with G.Context(k, d, ld, lr=0.05, momentum=0.9, seg_offsets=off, seg_lr_scale=sc) as ctx:
        for kern in (G.KERNEL_GOSSIP, G.KERNEL_GOSSIP_FUSED):
            ctx.set_launch_width(kern, width)
        x, v, g = dev(inp.x), dev(inp.v), dev(inp.g)
        xo, vo = inp.x.copy(), inp.v.copy()
        for rep in range(2):
            ctx.step_gossip_pull(x, v, g, peer, 0.5)
            ctx.step_gossip_pull(x, v, g, peer, 0.25, True)
            oracle.step_gossip(xo, vo, inp.g, lrc, 0.9, 0.5, peer, n=d)
            oracle.step_gossip_ext(xo, vo, inp.g, lrc, 0.9, 0.25, peer, stale=True, n=d)
        assert_bitwise(host(x), xo, "pull x")
        assert_bitwise(host(v), vo, "pull v")
        ctx.step_gossip_push(x, v, g, target)
        oracle.step_gossip_push(xo, vo, inp.g, lrc, 0.9, target, n=d)
        assert_rows_close(host(x)[:, :d], xo[:, :d], "push x")
        assert_bitwise(host(v), vo, "push v")

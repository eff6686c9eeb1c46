"""GPU parity at the full sizes of the benchmark configurations, in the launch
configuration bench.py times (same library calls, matrices in the blocked
layout each configuration is benchmarked in, flat or ResNet-segmented step
sizes); the metric shape also with row-major matrices.

Every rule is independent per column, and the random streams are indexed by
the global column, so the oracle recomputes sampled column slices of the
full problem exactly: the first tiles, an unaligned slice in the middle, a
slice across per-layer tensor boundaries, and the ragged end of the rows.
With uniform noise the sampled columns must match bit for bit after the whole
run; with Gaussian noise to the tolerance of parity_util.  Properties that hold
at any size (replica mean kept by the mix, consensus distance shrinking,
all-reduce rows staying identical) are checked on the whole arrays.
"""
import numpy as np
import pytest

from paper_1611_04581_amd import workloads as W
from parity_util import assert_bitwise, assert_rows_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import torch
    from paper_1611_04581_amd import gsgd
    assert torch.cuda.is_available()
    gsgd.lib()
    return gsgd


def _shared_vectors(d, ld, seed):
    rng = np.random.default_rng(seed)
    out = []
    for draw in (rng.standard_normal, lambda n: rng.uniform(0.1, 1.0, n), rng.standard_normal):
        a = np.zeros(ld, np.float32)
        a[:d] = draw(d).astype(np.float32)
        out.append(a)
    return out          # xstar, h, x0


def _slices(d, layout):
    s = [(0, 2048 + 3), (d // 2 + 1, 1500), (d - 1027, 1027)]
    if layout is not None:
        off = layout[0]
        b = int(off[len(off) // 2])               # a tensor boundary in the middle of the model
        s.append((b - 700, 1400))
        s.append((int(off[3]) - 5, 300))          # around the small BN tensors at the front
    return s


def _columns(t, c0, n, k, b):
    """Columns c0 .. c0+n-1 of every row of a device matrix (k x n, host), whatever layout it is kept in."""
    import torch
    if not b:
        return np.ascontiguousarray(t[:, c0:c0 + n].cpu().numpy())
    j = torch.arange(c0, c0 + n, device="cuda", dtype=torch.int64)
    flat = ((j // b) * (k * b) + j % b)[None, :] + torch.arange(k, device="cuda", dtype=torch.int64)[:, None] * b
    return np.ascontiguousarray(torch.take(t, flat).cpu().numpy())


def _run(G, oracle, cfg, steps, kind, mode=0, check_identical_rows=False, block_columns=None):
    import torch
    k, d = cfg.k, cfg.d
    b = cfg.block_columns if block_columns is None else block_columns
    ld = W.round_up(d, b or 1024)
    layout = None
    seg = {}
    if cfg.layout:
        off, sc, _ = W.resnet_layout(cfg.layout)
        layout = (off, sc)
        seg = dict(seg_offsets=off, seg_lr_scale=sc)
    xstar, h, x0 = _shared_vectors(d, ld, seed=77)
    slices = _slices(d, layout)
    wd, nest = cfg.weight_decay, cfg.nesterov
    with G.Context(k, d, ld, lr=cfg.lr, momentum=cfg.momentum, sigma=cfg.sigma, seed=cfg.seed, noise_kind=kind,
                   block_columns=b, **seg) as ctx:
        ctx.set_local_step(wd, nest)
        x = torch.empty((k, ld), dtype=torch.float32, device="cuda")
        v = torch.empty_like(x)
        g = torch.empty_like(x)
        dxs, dh, dx0 = (torch.from_numpy(a).cuda() for a in (xstar, h, x0))
        c = torch.empty(ld, dtype=torch.float32, device="cuda")
        ctx.init_replicas(x, v, c, dx0, mode)
        # oracle state for the sampled slices
        st = []
        for (c0, n) in slices:
            if mode == 0:
                xo = np.tile(x0[c0:c0 + n], (k, 1)).copy()
                co = x0[c0:c0 + n].copy()
            else:                       # per-replica Gaussian start: take the device's values as the common start
                xo = _columns(x, c0, n, k, b)
                co = np.ascontiguousarray(c[c0:c0 + n].cpu().numpy())
            lrc = oracle.expand_lr(cfg.lr, n, *(layout or (None, None)), col0=c0)
            st.append(dict(c0=c0, n=n, x=xo, v=np.zeros((k, n), np.float32), g=np.zeros((k, n), np.float32), c=co,
                           lr=lrc, xs=xstar[c0:c0 + n].copy(), h=h[c0:c0 + n].copy()))
        cons = [ctx.stats(x, dxs)[0]]
        identity = list(range(k))
        for t in range(steps):
            rule = cfg.rule if G.comm_due(t, cfg.tau) else "local"
            perm = None
            if rule in ("gossip", "gossip_stale"):
                perm = G.make_perm(cfg.seed, t, k)
            elif rule in ("gossip_pull", "gossip_push"):
                perm = G.make_targets(cfg.seed, t, k, rule == "gossip_push")
            ctx.gen_grad(x, dh, dxs, g, t)
            if rule == "gossip":
                ctx.step_gossip(x, v, g, perm, cfg.beta)
            elif rule == "gossip_stale":
                ctx.step_gossip_stale(x, v, g, perm, cfg.beta)
            elif rule == "gossip_pull":
                ctx.step_gossip_pull(x, v, g, perm, cfg.beta)
            elif rule == "gossip_push":
                ctx.step_gossip_push(x, v, g, perm)
            elif rule == "local":
                ctx.step_local(x, v, g)
            elif rule == "allreduce":
                ctx.step_allreduce(x, v, g)
            else:
                ctx.step_easgd(x, v, g, c, cfg.alpha_e)
            for s in st:
                oracle.gen_grad(s["x"], s["h"], s["xs"], s["g"], cfg.sigma, cfg.seed, t, kind, col0=s["c0"])
                if rule == "gossip" and not (wd or nest):
                    oracle.step_gossip(s["x"], s["v"], s["g"], s["lr"], cfg.momentum, cfg.beta, perm)
                elif rule in ("gossip", "gossip_stale", "gossip_pull", "local"):
                    oracle.step_gossip_ext(s["x"], s["v"], s["g"], s["lr"], cfg.momentum, cfg.beta,
                                           identity if rule == "local" else perm, wd=wd, nesterov=nest,
                                           stale=rule == "gossip_stale")
                elif rule == "gossip_push":
                    oracle.step_gossip_push(s["x"], s["v"], s["g"], s["lr"], cfg.momentum, perm, wd=wd, nesterov=nest)
                elif rule == "allreduce":
                    oracle.step_allreduce(s["x"], s["v"], s["g"], s["lr"], cfg.momentum)
                else:
                    oracle.step_easgd(s["x"], s["v"], s["g"], s["c"], s["lr"], cfg.momentum, cfg.alpha_e)
            if t in (0, steps // 2):
                cons.append(ctx.stats(x, dxs)[0])
        final = ctx.stats(x, dxs)
        cons.append(final[0])
        for s in st:
            c0, n = s["c0"], s["n"]
            gx = _columns(x, c0, n, k, b)
            gv = _columns(v, c0, n, k, b)
            if kind == G.NOISE_UNIFORM and cfg.rule != "gossip_push":
                assert_bitwise(gx, s["x"], "x cols %d..%d" % (c0, c0 + n))
                assert_bitwise(gv, s["v"], "v cols %d..%d" % (c0, c0 + n))
            else:         # Gaussian transform, or push-gossip's fp64 sums taken in a different order
                assert_rows_close(gx, s["x"], "x cols %d..%d" % (c0, c0 + n))
            if cfg.rule == "easgd":
                gc = np.ascontiguousarray(c[c0:c0 + n].cpu().numpy())
                if kind == G.NOISE_UNIFORM:
                    assert_bitwise(gc, s["c"], "center")
                else:
                    assert_rows_close(gc, s["c"], "center")
        if check_identical_rows:
            xr, vr = (W.from_blocked(t, b) if b else t for t in (x, v))
            assert bool((xr[1:, :d] == xr[0, :d]).all()) and bool((vr[1:, :d] == vr[0, :d]).all())
            del xr, vr
        # padding columns were never written by any step kernel (init leaves them as allocated)
        return cons, final, (x, v, g, dxs, ctx, d)


def test_allreduce_resnet18_200_steps(G, oracle):
    cfg = W.CONFIGS["allreduce_r18"]
    cons, final, _ = _run(G, oracle, cfg, cfg.steps, G.NOISE_UNIFORM, check_identical_rows=True)
    assert all(c == 0.0 for c in cons)                 # identical start: all-reduce keeps the replicas identical
    assert final[2] < 0.01 * 2 * cfg.d                 # the mean went from ~2d to near x*


def test_gossip_resnet18_200_steps_mean_and_consensus(G, oracle):
    import torch
    cfg = W.CONFIGS["gossip_r18"]
    cons, final, _ = _run(G, oracle, cfg, cfg.steps, G.NOISE_UNIFORM, mode=1)
    assert cons[-1] < 1e-2 * cons[0] and cons[1] < cons[0]          # consensus distance shrinks from a spread start
    # the mix leaves the replica mean where the local step put it (whole arrays, one step)
    k, d = cfg.k, cfg.d
    ld = W.round_up(d, 1024)
    with G.Context(k, d, ld, lr=cfg.lr, momentum=cfg.momentum, sigma=cfg.sigma, seed=cfg.seed) as ctx:
        x = torch.empty((k, ld), dtype=torch.float32, device="cuda")
        v = torch.empty_like(x)
        g = torch.randn((k, ld), dtype=torch.float32, device="cuda", generator=torch.Generator("cuda").manual_seed(1))
        ctx.init_replicas(x, v, None, None, G.INIT_PER_REPLICA)
        xl, vl = x.clone(), v.clone()
        perm = G.make_perm(cfg.seed, 0, k)
        ctx.step_gossip(xl, vl, g, perm, 0.0)
        ctx.step_gossip(x, v, g, perm, 0.5)
        ml = xl[:, :d].double().mean(0)
        mm = x[:, :d].double().mean(0)
        bound = 1e-5 * max(1.0, float(ml.abs().max()))
        assert float((mm - ml).abs().max()) <= bound
        assert bool((v == vl).all())


@pytest.mark.parametrize("kind,row_major", [(1, False), (0, False), (1, True)])
def test_gossip_resnet50_metric_shape(G, oracle, kind, row_major):
    cfg = W.CONFIGS["gossip_r50"]
    steps = cfg.steps if kind == 1 else 60
    cons, final, _ = _run(G, oracle, cfg, steps, kind, block_columns=0 if row_major else None)
    assert cons[0] == 0.0 and cons[-1] > 0.0             # identical start: consensus distance rises to its noise floor


def test_easgd_resnet50_200_steps(G, oracle):
    cfg = W.CONFIGS["easgd_r50"]
    _run(G, oracle, cfg, cfg.steps, G.NOISE_UNIFORM)


def test_segmented_gossip_k128_100_steps(G, oracle):
    cfg = W.CONFIGS["seg_gossip_r50_k128"]
    _run(G, oracle, cfg, cfg.steps, G.NOISE_UNIFORM)


@pytest.mark.parametrize("name", ["pull_gossip_r50", "stale_gossip_r50", "push_gossip_r50"])
def test_other_gossip_forms_at_the_metric_shape(G, oracle, name):
    """iid pull targets (Algorithm 3), stale parameters (Section 6.2.1) and
    push-gossip (Algorithm 4) at k = 32, ResNet-50 size, from a spread start."""
    cfg = W.CONFIGS[name]
    cons, final, _ = _run(G, oracle, cfg, 50, G.NOISE_UNIFORM, mode=1)
    assert cons[-1] < 1e-2 * cons[0]


def test_paper_training_recipe_resnet18(G, oracle):
    """Section 4.2's recipe on the quadratic: push-gossip, 16 nodes, Nesterov
    0.9, weight decay 1e-4, step size 0.1, exchange every 10th iteration."""
    cfg = W.CONFIGS["paper_setup_r18"]
    _run(G, oracle, cfg, cfg.steps, G.NOISE_UNIFORM)

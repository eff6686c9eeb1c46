"""GPU parity: every entry point of libgsgd, called through the C ABI, against
the CPU oracle on the same seeded inputs.

Bar: bit-exact for the Philox words, the permutation and everything whose
arithmetic is fixed-order fp32/fp64 (uniform-noise gradients, the three step
rules); the tolerance of parity_util for what involves the Gaussian transform
(device logf/sincospif against the oracle's fp64 Box-Muller).
"""
import numpy as np
import pytest

from paper_1611_04581_amd import workloads as W
from parity_util import assert_bitwise, assert_rows_close, mean_preserved

pytestmark = pytest.mark.gpu

SEED = 0x161104581
# several 1024-column workgroup tiles plus a ragged tail, and the degenerate sizes
SHAPES = [(4, 5 * 1024 + 7, None), (3, 1, 4), (1, 4, None), (7, 1023, 1024), (32, 2 * 1024 + 2, 4096), (5, 2, 8)]


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


def perms_for(k, oracle):
    out = [list(range(k)), [(i + 1) % k for i in range(k)], [int(t) for t in oracle.make_perm(SEED, 3, k)]]
    if k >= 2:
        inv = list(range(k))
        for a in range(0, k - 1, 2):
            inv[a], inv[a + 1] = a + 1, a
        out.append(inv)
    if k >= 6:
        # a 3-cycle, a fixed point and one long cycle over the rest
        out.append([1, 2, 0, 3] + list(range(5, k)) + [4])
    for p in out:
        assert sorted(p) == list(range(k))
    return out


# ----------------------------------------------------------------------------
def test_philox_words_bit_exact(G, oracle):
    import torch
    n = 3000
    with G.Context(4, 64, seed=SEED) as ctx:
        for (c1, c2, c3) in [(0, 0, 0), (3, 41, 0), (31, 199, 5), (0xFFFFFFFF, 0xFFFFFFFF, 0xFFFFFFFF)]:
            out = torch.zeros(4 * n, dtype=torch.int32, device="cuda")
            ctx.philox_raw(c1, c2, c3, n, out)
            got = host(out).view(np.uint32).reshape(n, 4)
            for q in list(range(0, 40)) + list(range(n - 40, n)) + list(range(1000, 1016)):
                want = oracle.philox4x32_10((q, c1, c2, c3), (SEED & 0xFFFFFFFF, SEED >> 32))
                assert tuple(int(w) for w in got[q]) == want, (q, c1, c2, c3)


def test_noise_alu_probe_is_the_generators_arithmetic(G, oracle):
    """The measurement hook folds the same Philox blocks and noise values the
    gradient generator draws: uniform kind bit for bit, Gaussian at tolerance."""
    import torch
    wgs, iters = 2, 5
    for kind in (G.NOISE_UNIFORM, G.NOISE_GAUSSIAN):
        with G.Context(4, 64, seed=SEED, noise_kind=kind) as ctx:
            out = torch.zeros(wgs * 256, dtype=torch.float32, device="cuda")
            ctx.noise_alu_probe(wgs, iters, out)
            got = host(out)
        key = (SEED & 0xFFFFFFFF, SEED >> 32)
        for t in (0, 1, 63, 64, 255, 256, 511):
            acc = np.zeros(4, np.float32)
            for it in range(iters):
                acc = (acc + oracle.noise4(oracle.philox4x32_10((t, it, 0, 0), key), kind)).astype(np.float32)
            want = np.float32(np.float32(acc[0] + acc[1]) + np.float32(acc[2] + acc[3]))
            if kind == G.NOISE_UNIFORM:
                assert got[t].view(np.uint32) == want.view(np.uint32), t
            else:
                assert abs(float(got[t]) - float(want)) <= 2e-6 * max(1.0, abs(float(want))), t


def test_gaussian_transform_accuracy_over_two_million_draws(G, oracle):
    """The device Box-Muller (hardware log2 and square root, series sine / cosine,
    all fp32) against the oracle's fp64 transform rounded once, on 2^21 draws
    that reach |xi| = 5: the bound is a few units in the last place of the
    largest values (one unit at 4..8 is 4.8e-7), far inside the 1e-6 bar once
    scaled by sigma * lr in a step."""
    import torch
    d = (1 << 21) + 3
    ld = W.round_up(d, 4)
    with G.Context(2, d, ld, seed=SEED) as ctx:
        t = torch.zeros(ld, device="cuda")
        ctx.fill(t, G.FILL_X0)
        got = host(t)[:d].astype(np.float64)
    want = oracle.fill(d, SEED, oracle.STREAM_X0).astype(np.float64)
    err = np.abs(got - want)
    assert np.abs(want).max() > 4.5
    assert err.max() <= 1.5e-6, err.max()
    assert np.sqrt((err ** 2).mean()) <= 1.2e-7
    assert (got == want).mean() > 0.4          # about half the draws round to the same float


def test_fill_and_init(G, oracle):
    import torch
    k, d, ld = 5, 3 * 1024 + 5, 3 * 1024 + 8
    with G.Context(k, d, ld, seed=SEED) as ctx:
        bufs = {}
        for which in (G.FILL_XSTAR, G.FILL_H, G.FILL_X0):
            t = torch.full((ld,), 777.0, device="cuda")
            ctx.fill(t, which)
            bufs[which] = host(t)
            assert (bufs[which][d:] == 777.0).all()
        assert_bitwise(bufs[G.FILL_H][:d], oracle.fill(d, SEED, oracle.STREAM_H), "h")
        assert_rows_close(bufs[G.FILL_XSTAR][:d], oracle.fill(d, SEED, oracle.STREAM_XSTAR), "xstar")
        assert_rows_close(bufs[G.FILL_X0][:d], oracle.fill(d, SEED, oracle.STREAM_X0), "x0")

        inp = W.make_inputs(k, d, ld, seed=1)
        x, v, c = dev(inp.x), dev(inp.v), dev(inp.center)
        ctx.init_replicas(x, v, c, dev(inp.x0), G.INIT_BROADCAST)
        xo, vo, co = inp.x.copy(), inp.v.copy(), inp.center.copy()
        oracle.init_replicas(xo, vo, co, inp.x0, SEED, 0, n=d)
        assert_bitwise(host(x), xo, "x")
        assert_bitwise(host(v), vo, "v")
        assert_bitwise(host(c), co, "center")

        ctx.init_replicas(x, v, c, None, G.INIT_PER_REPLICA)
        oracle.init_replicas(xo, vo, co, None, SEED, 1, n=d)
        assert_rows_close(host(x)[:, :d], xo[:, :d], "x")
        assert_bitwise(host(v), vo, "v")
        assert_rows_close(host(c)[:d], co[:d], "center")
        assert (host(x)[:, d:] == 777.0).all() and (host(c)[d:] == 777.0).all()
        ctx.init_replicas(x, v, None, None, G.INIT_PER_REPLICA)     # centre is optional


@pytest.mark.parametrize("k,d,ld", SHAPES)
def test_gen_grad(G, oracle, k, d, ld):
    ld = ld or W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=2)
    for kind, step in ((G.NOISE_UNIFORM, 0), (G.NOISE_UNIFORM, 123456), (G.NOISE_GAUSSIAN, 7)):
        with G.Context(k, d, ld, sigma=0.3, seed=SEED, noise_kind=kind) as ctx:
            g = dev(inp.g)
            ctx.gen_grad(dev(inp.x), dev(inp.h), dev(inp.xstar), g, step)
            go = inp.g.copy()
            oracle.gen_grad(inp.x, inp.h, inp.xstar, go, 0.3, SEED, step, kind, n=d)
            if kind == G.NOISE_UNIFORM:
                assert_bitwise(host(g), go, "g")
            else:
                assert_rows_close(host(g)[:, :d], go[:, :d], "g")
                assert_bitwise(host(g)[:, d:], go[:, d:], "g padding")


@pytest.mark.parametrize("k,d,ld", SHAPES)
def test_step_gossip_bit_exact(G, oracle, k, d, ld):
    ld = ld or W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=3)
    with G.Context(k, d, ld, lr=0.05, momentum=0.9) as ctx:
        for beta in (0.5, 0.3):
            for perm in perms_for(k, oracle):
                x, v = dev(inp.x), dev(inp.v)
                ctx.step_gossip(x, v, dev(inp.g), perm, beta)
                xo, vo = inp.x.copy(), inp.v.copy()
                oracle.step_gossip(xo, vo, inp.g, 0.05, 0.9, beta, perm, n=d)
                assert_bitwise(host(x), xo, "x perm=%s" % perm)
                assert_bitwise(host(v), vo, "v")
                # same call again from the same inputs: the in-place walk has no race
                x2, v2 = dev(inp.x), dev(inp.v)
                ctx.step_gossip(x2, v2, dev(inp.g), perm, beta)
                assert_bitwise(host(x2), host(x), "x repeat")


@pytest.mark.parametrize("k,d,ld", SHAPES)
def test_step_allreduce_bit_exact(G, oracle, k, d, ld):
    ld = ld or W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=4)
    with G.Context(k, d, ld, lr=0.05, momentum=0.9) as ctx:
        x, v = dev(inp.x), dev(inp.v)
        ctx.step_allreduce(x, v, dev(inp.g))
        xo, vo = inp.x.copy(), inp.v.copy()
        oracle.step_allreduce(xo, vo, inp.g, 0.05, 0.9, n=d)
        assert_bitwise(host(x), xo, "x")
        assert_bitwise(host(v), vo, "v")


@pytest.mark.parametrize("k,d,ld", SHAPES)
def test_step_easgd_bit_exact(G, oracle, k, d, ld):
    ld = ld or W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=5)
    alpha_e = 0.9 / k
    with G.Context(k, d, ld, lr=0.05, momentum=0.9) as ctx:
        x, v, c = dev(inp.x), dev(inp.v), dev(inp.center)
        ctx.step_easgd(x, v, dev(inp.g), c, alpha_e)
        xo, vo, co = inp.x.copy(), inp.v.copy(), inp.center.copy()
        oracle.step_easgd(xo, vo, inp.g, co, 0.05, 0.9, alpha_e, n=d)
        assert_bitwise(host(x), xo, "x")
        assert_bitwise(host(v), vo, "v")
        assert_bitwise(host(c), co, "center")


@pytest.mark.parametrize("n_seg,align", [(1, 1), (37, 1), (37, 4), (100, 64), (1500, 1)])
def test_segmented_steps_bit_exact(G, oracle, n_seg, align):
    """Per-layer step sizes: table staged in LDS (<= 1024 segments) or searched
    in global memory (1500), boundaries aligned to quads or not."""
    k, d = 6, 7 * 1024 + 3
    ld = W.round_up(d, 4)
    off, sc = W.random_segments(d, n_seg, seed=n_seg, align=align)
    inp = W.make_inputs(k, d, ld, seed=6)
    lrc = oracle.expand_lr(0.05, d, off, sc)
    perm = [int(t) for t in oracle.make_perm(SEED, 1, k)]
    with G.Context(k, d, ld, lr=0.05, momentum=0.9, seg_offsets=off, seg_lr_scale=sc) as ctx:
        x, v = dev(inp.x), dev(inp.v)
        ctx.step_gossip(x, v, dev(inp.g), perm, 0.5)
        xo, vo = inp.x.copy(), inp.v.copy()
        oracle.step_gossip(xo, vo, inp.g, lrc, 0.9, 0.5, perm, n=d)
        assert_bitwise(host(x), xo, "gossip x")
        assert_bitwise(host(v), vo, "gossip v")

        x, v = dev(inp.x), dev(inp.v)
        ctx.step_allreduce(x, v, dev(inp.g))
        xo, vo = inp.x.copy(), inp.v.copy()
        oracle.step_allreduce(xo, vo, inp.g, lrc, 0.9, n=d)
        assert_bitwise(host(x), xo, "allreduce x")
        assert_bitwise(host(v), vo, "allreduce v")

        x, v, c = dev(inp.x), dev(inp.v), dev(inp.center)
        ctx.step_easgd(x, v, dev(inp.g), c, 0.1)
        xo, vo, co = inp.x.copy(), inp.v.copy(), inp.center.copy()
        oracle.step_easgd(xo, vo, inp.g, co, lrc, 0.9, 0.1, n=d)
        assert_bitwise(host(x), xo, "easgd x")
        assert_bitwise(host(c), co, "easgd center")


def test_max_replicas(G, oracle):
    k, d = G.MAX_K, 1024 + 4
    inp = W.make_inputs(k, d, seed=7)
    perm = [int(t) for t in oracle.make_perm(SEED, 9, k)]
    with G.Context(k, d) as ctx:
        x, v = dev(inp.x), dev(inp.v)
        ctx.step_gossip(x, v, dev(inp.g), perm, 0.5)
        xo, vo = inp.x.copy(), inp.v.copy()
        oracle.step_gossip(xo, vo, inp.g, 0.05, 0.9, 0.5, perm)
        assert_bitwise(host(x), xo, "x")
        x, v = dev(inp.x), dev(inp.v)
        ctx.step_allreduce(x, v, dev(inp.g))
        xo, vo = inp.x.copy(), inp.v.copy()
        oracle.step_allreduce(xo, vo, inp.g, 0.05, 0.9)
        assert_bitwise(host(x), xo, "x")


@pytest.mark.parametrize("kind", [1, 0])
def test_fused_generator_gossip(G, oracle, kind):
    k, d = 8, 3 * 1024 + 6
    ld = W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=8)
    perm = [int(t) for t in oracle.make_perm(SEED, 2, k)]
    with G.Context(k, d, ld, sigma=0.2, seed=SEED, noise_kind=kind) as ctx:
        h, xs = dev(inp.h), dev(inp.xstar)
        xa, va, g = dev(inp.x), dev(inp.v), dev(inp.g)
        ctx.gen_grad(xa, h, xs, g, 17)
        ctx.step_gossip(xa, va, g, perm, 0.5)
        xb, vb = dev(inp.x), dev(inp.v)
        ctx.step_gossip_fused(xb, vb, h, xs, perm, 17, 0.5)
        assert_bitwise(host(xb), host(xa), "fused vs two-kernel x")
        assert_bitwise(host(vb), host(va), "fused vs two-kernel v")
        xo, vo, go = inp.x.copy(), inp.v.copy(), inp.g.copy()
        oracle.gen_grad(xo, inp.h, inp.xstar, go, 0.2, SEED, 17, kind, n=d)
        oracle.step_gossip(xo, vo, go, 0.05, 0.9, 0.5, perm, n=d)
        if kind == 1:
            assert_bitwise(host(xb), xo, "x")
        else:
            assert_rows_close(host(xb)[:, :d], xo[:, :d], "x")


def test_stats(G, oracle):
    k, d, ld = 9, 4 * 1024 + 3, 4 * 1024 + 8
    inp = W.make_inputs(k, d, ld, seed=9)
    with G.Context(k, d, ld) as ctx:
        got = ctx.stats(dev(inp.x), dev(inp.xstar))
    want = oracle.stats(inp.x, inp.xstar, n=d)
    assert np.allclose(got, want, rtol=1e-11, atol=0)
    # identical rows: consensus distance exactly zero
    inp2 = W.make_inputs(4, 1000, seed=10, identical_rows=True)
    with G.Context(4, 1000) as ctx:
        assert ctx.stats(dev(inp2.x), dev(inp2.xstar))[0] == 0.0


def _stats_cases():
    rng = np.random.default_rng(5)
    k, d = 13, 3 * 1024 + 2
    yield "clustered_far_from_zero", (3.0 + 1e-5 * rng.standard_normal((k, d))).astype(np.float32)
    a = (1e-3 * rng.standard_normal((k, d))).astype(np.float32)
    a[0] = 1e3
    yield "first_row_an_outlier", a
    b = (1e-3 * rng.standard_normal((k, d))).astype(np.float32)
    b[-1] = -1e3
    yield "last_row_an_outlier", b
    yield "one_replica", rng.standard_normal((1, d)).astype(np.float32)
    yield "most_replicas", rng.standard_normal((128, 1024 + 1)).astype(np.float32)
    yield "huge", (1e18 * rng.standard_normal((k, d))).astype(np.float32)
    yield "subnormal", (1e-41 * rng.standard_normal((k, d))).astype(np.float32)
    c = np.repeat(rng.standard_normal((1, d)).astype(np.float32), k, axis=0)
    c[5, 7] = np.nextafter(c[5, 7], np.float32(9))
    yield "one_value_one_ulp_off", c


@pytest.mark.parametrize("name,x", list(_stats_cases()), ids=[n for n, _ in _stats_cases()])
def test_stats_where_one_pass_could_cancel(G, oracle, name, x):
    """The kernel reads x once and takes deviations from the first row; the oracle is the two-pass definition
    (Section 6.1's quantities).  Inputs where a one-pass sum of squares would lose everything."""
    k, d = x.shape
    ld = W.round_up(d, 4)
    xp = np.zeros((k, ld), np.float32)
    xp[:, :d] = x
    xs = np.zeros(ld, np.float32)
    xs[:d] = np.random.default_rng(1).standard_normal(d).astype(np.float32)
    want = oracle.stats(xp, xs, n=d)
    with G.Context(k, d, ld) as ctx:
        got = ctx.stats(dev(xp), dev(xs))
    assert np.allclose(got, want, rtol=1e-11, atol=0), (name, got, want)
    if k == 1:
        assert got[0] == 0.0


@pytest.mark.parametrize("k,tiles,b", [(3, 2100, 0), (3, 2100, 4096), (20, 1100, 0), (20, 1100, 2048),
                                       (32, 700, 0), (32, 700, 16384), (45, 600, 1024), (128, 520, 0)])
def test_stats_when_workgroups_take_several_tiles(G, oracle, k, tiles, b):
    """Vectors longer than the statistics pass has workgroups (2048 up to 8 replicas, 1024 up to 16, 512 beyond), so
    that workgroups stride over several tiles, some over one more than others; replica counts that fill the
    batches of rows exactly, leave rows over, or fit no batch at all; both layouts."""
    d = tiles * 1024 + 13
    ld = W.round_up(d, b or 1024)
    rng = np.random.default_rng(77 + k)
    x = np.zeros((k, ld), np.float32)
    x[:, :d] = 2.0 + 0.1 * rng.standard_normal((k, d)).astype(np.float32)
    xs = np.zeros(ld, np.float32)
    xs[:d] = rng.standard_normal(d).astype(np.float32)
    want = oracle.stats(x, xs, n=d)
    with G.Context(k, d, ld, block_columns=b) as ctx:
        xd = dev(W.to_blocked(x, b) if b else x)
        got = ctx.stats(xd, dev(xs))
        again = ctx.stats(xd, dev(xs))
    assert np.allclose(got, want, rtol=1e-11, atol=0), (got, want)
    assert np.array_equal(got, again)


def test_bad_arguments_leave_state_untouched(G):
    import torch
    k, d = 4, 1024
    inp = W.make_inputs(k, d, seed=11)
    with G.Context(k, d) as ctx:
        x, v, g = dev(inp.x), dev(inp.v), dev(inp.g)
        for bad in ([0, 1, 2, 2], [0, 1, 2, 4], [-1, 0, 1, 2]):
            with pytest.raises(G.GsgdError) as e:
                ctx.step_gossip(x, v, g, bad, 0.5)
            assert e.value.code == G.ERR_BAD_PERM
        with pytest.raises(G.GsgdError) as e:
            ctx.step_gossip(x, v, x, [0, 1, 2, 3], 0.5)               # aliasing
        assert e.value.code == G.ERR_INVALID_ARG
        with pytest.raises(G.GsgdError) as e:
            big = torch.zeros(k * d + 8, dtype=torch.float32, device="cuda")
            ctx.step_allreduce(big[1:1 + k * d], v, g)                 # misaligned
        assert e.value.code == G.ERR_INVALID_ARG
        with pytest.raises(G.GsgdError):
            ctx.gen_grad(x, dev(inp.h), dev(inp.xstar), g, 2**32)
        torch.cuda.synchronize()
        assert_bitwise(host(x), inp.x, "x")
        assert_bitwise(host(v), inp.v, "v")


# ----------------------------------------------------------------------------
# whole trajectories

def _run_both(G, oracle, cfg, d, steps, kind, layout=None, mode=0, sigma=None):
    """cfg-shaped run on both sides, inputs from the seeded numpy generator."""
    k = cfg.k
    ld = W.round_up(d, 1024)
    sigma = cfg.sigma if sigma is None else sigma
    inp = W.make_inputs(k, d, ld, seed=12)
    seg = {}
    lrc = cfg.lr
    if layout is not None:
        off, sc = layout
        seg = dict(seg_offsets=off, seg_lr_scale=sc)
        lrc = oracle.expand_lr(cfg.lr, d, off, sc)
    xo, vo, go, co = inp.x.copy(), inp.v.copy(), inp.g.copy(), inp.center.copy()
    oracle.init_replicas(xo, vo, co, inp.x0, cfg.seed, mode, n=d)
    means = []
    with G.Context(k, d, ld, lr=cfg.lr, momentum=cfg.momentum, sigma=sigma, seed=cfg.seed, noise_kind=kind, **seg) as ctx:
        x, v, g, c = dev(inp.x), dev(inp.v), dev(inp.g), dev(inp.center)
        h, xs = dev(inp.h), dev(inp.xstar)
        ctx.init_replicas(x, v, c, dev(inp.x0), mode)
        if mode == 1:                     # Gaussian init differs in the last place: start both sides from the oracle's
            x.copy_(dev(xo)); c.copy_(dev(co))
        for t in range(steps):
            ctx.gen_grad(x, h, xs, g, t)
            oracle.gen_grad(xo, inp.h, inp.xstar, go, sigma, cfg.seed, t, kind, n=d)
            if cfg.rule == "gossip":
                perm = G.make_perm(cfg.seed, t, k)
                assert np.array_equal(perm, oracle.make_perm(cfg.seed, t, k))
                ctx.step_gossip(x, v, g, perm, cfg.beta)
                oracle.step_gossip(xo, vo, go, lrc, cfg.momentum, cfg.beta, perm, n=d)
            elif cfg.rule == "allreduce":
                ctx.step_allreduce(x, v, g)
                oracle.step_allreduce(xo, vo, go, lrc, cfg.momentum, n=d)
            else:
                ctx.step_easgd(x, v, g, c, cfg.alpha_e)
                oracle.step_easgd(xo, vo, go, co, lrc, cfg.momentum, cfg.alpha_e, n=d)
        st = ctx.stats(x, xs)
        return host(x), host(v), host(c), xo, vo, co, st, inp


def test_tiny_config_full_trajectory(G, oracle):
    """The 'tiny' benchmark configuration: k=4, d=65,536, sigma=0.01, 100 gossip steps."""
    cfg = W.CONFIGS["tiny"]
    x, v, c, xo, vo, co, st, inp = _run_both(G, oracle, cfg, cfg.d, cfg.steps, G.NOISE_UNIFORM)
    assert_bitwise(x, xo, "x (uniform noise: whole trajectory bit-exact)")
    assert_bitwise(v, vo, "v")
    x, v, c, xo, vo, co, st, inp = _run_both(G, oracle, cfg, cfg.d, cfg.steps, G.NOISE_GAUSSIAN)
    assert_rows_close(x[:, :cfg.d], xo[:, :cfg.d], "x")
    # v is a small difference quantity (|v| ~ lr * sigma ~ 1e-3 near x*) formed from O(1) parameters: the two sides'
    # x agree to ~1e-7 absolutely, so v agrees to lr * h * 1e-7 / (1 - mu) ~ 1e-8 absolutely, which is 1e-5 of |v|
    assert_rows_close(v[:, :cfg.d], vo[:, :cfg.d], "v", rtol=1e-5)
    # the statistics are sums of squares of differences ~3e-3 of parameters ~1 that agree to ~1e-7: 2 * 1e-7 / 3e-3
    # ~ 1e-4 relative in the worst case (the bit-exact uniform-noise runs compare them at 1e-10)
    assert np.allclose(st, oracle.stats(xo, inp.xstar, n=cfg.d), rtol=1e-4)
    # converged towards x*: distance shrank by orders of magnitude from the start
    d0 = ((inp.x0[:cfg.d].astype(np.float64) - inp.xstar[:cfg.d]) ** 2).sum() * cfg.k
    assert st[1] < 0.05 * d0


@pytest.mark.parametrize("rule", ["allreduce", "easgd", "gossip_seg", "gossip_spread"])
def test_small_trajectories_all_rules(G, oracle, rule):
    d, steps = 9 * 1024 + 5, 40
    if rule == "allreduce":
        cfg = W.Config("t", "allreduce", 8, d, steps)
        x, v, c, xo, vo, co, st, inp = _run_both(G, oracle, cfg, d, steps, G.NOISE_UNIFORM)
        assert_bitwise(x, xo, "x"); assert_bitwise(v, vo, "v")
        assert all(np.array_equal(x[0], x[i]) for i in range(1, cfg.k))      # identical start stays identical
    elif rule == "easgd":
        cfg = W.Config("t", "easgd", 16, d, steps, alpha_e=0.9 / 16)
        x, v, c, xo, vo, co, st, inp = _run_both(G, oracle, cfg, d, steps, G.NOISE_UNIFORM)
        assert_bitwise(x, xo, "x"); assert_bitwise(c, co, "center")
        x, v, c, xo, vo, co, st, inp = _run_both(G, oracle, cfg, d, steps, G.NOISE_GAUSSIAN)
        assert_rows_close(x[:, :d], xo[:, :d], "x"); assert_rows_close(c[:d], co[:d], "center")
    elif rule == "gossip_seg":
        cfg = W.Config("t", "gossip", 12, d, steps)
        layout = W.random_segments(d, 50, seed=1, align=4)
        x, v, c, xo, vo, co, st, inp = _run_both(G, oracle, cfg, d, steps, G.NOISE_UNIFORM, layout=layout)
        assert_bitwise(x, xo, "x"); assert_bitwise(v, vo, "v")
    else:
        cfg = W.Config("t", "gossip", 32, d, steps)
        x, v, c, xo, vo, co, st, inp = _run_both(G, oracle, cfg, d, steps, G.NOISE_GAUSSIAN, mode=1)
        assert_rows_close(x[:, :d], xo[:, :d], "x")
        so = oracle.stats(xo, inp.xstar, n=d)
        assert np.allclose(st, so, rtol=1e-4)


def test_gossip_preserves_replica_mean_and_shrinks_consensus(G, oracle):
    """One call = local step then mix; the mix must not move the replica mean.
    Compare against the same call with beta = 0 (local step only)."""
    k, d = 32, 16 * 1024
    inp = W.make_inputs(k, d, seed=13)
    with G.Context(k, d) as ctx:
        g = dev(inp.g)
        cons = []
        x, v = dev(inp.x), dev(inp.v)
        xs = dev(inp.xstar)
        cons.append(ctx.stats(x, xs)[0])
        for t in range(6):
            perm = G.make_perm(SEED, t, k)
            xl, vl = x.clone(), v.clone()
            ctx.step_gossip(xl, vl, g, perm, 0.0)          # local step only
            ctx.step_gossip(x, v, g, perm, 0.5)
            mean_preserved(host(xl), host(x))
            g.zero_()                                      # pure gossip rounds after the first
            v.zero_()
            cons.append(ctx.stats(x, xs)[0])
        # expected halving per round (E[M^T M] = (I + 11^T/k)/2): six rounds shrink it ~64x
        assert cons[-1] < cons[1] / 16
        assert all(b < a for a, b in zip(cons[1:], cons[2:]))


@pytest.mark.parametrize("width", [1, 3, 255, 100000])
def test_results_do_not_depend_on_launch_width(G, oracle, width):
    """The streaming kernels run as `width` persistent workgroups pulling tiles
    from a ticket counter; any width (fewer or more workgroups than tiles) must
    give the oracle's bits, call after call (the counter resets itself)."""
    k, d = 6, 9 * 1024 + 5
    ld = W.round_up(d, 4)
    off, sc = W.random_segments(d, 23, seed=5, align=1)
    lrc = oracle.expand_lr(0.05, d, off, sc)
    inp = W.make_inputs(k, d, ld, seed=14)
    perm = [int(t) for t in oracle.make_perm(SEED, 4, k)]
    with G.Context(k, d, ld, sigma=0.2, seed=SEED, noise_kind=G.NOISE_UNIFORM, seg_offsets=off, seg_lr_scale=sc) as ctx:
        for kern in (G.KERNEL_GOSSIP, G.KERNEL_ALLREDUCE, G.KERNEL_EASGD, G.KERNEL_GEN_GRAD, G.KERNEL_GOSSIP_FUSED):
            ctx.set_launch_width(kern, width)
        h, xs = dev(inp.h), dev(inp.xstar)
        x, v, g, c = dev(inp.x), dev(inp.v), dev(inp.g), dev(inp.center)
        xo, vo, go, co = inp.x.copy(), inp.v.copy(), inp.g.copy(), inp.center.copy()
        for t in range(3):
            ctx.gen_grad(x, h, xs, g, t)
            ctx.step_gossip(x, v, g, perm, 0.5)
            ctx.step_allreduce(x, v, g)
            ctx.step_easgd(x, v, g, c, 0.1)
            ctx.step_gossip_fused(x, v, h, xs, perm, 100 + t, 0.5)
            oracle.gen_grad(xo, inp.h, inp.xstar, go, 0.2, SEED, t, 1, n=d)
            oracle.step_gossip(xo, vo, go, lrc, 0.9, 0.5, perm, n=d)
            oracle.step_allreduce(xo, vo, go, lrc, 0.9, n=d)
            oracle.step_easgd(xo, vo, go, co, lrc, 0.9, 0.1, n=d)
            oracle.gen_grad(xo, inp.h, inp.xstar, go, 0.2, SEED, 100 + t, 1, n=d)
            oracle.step_gossip(xo, vo, go, lrc, 0.9, 0.5, perm, n=d)
        assert_bitwise(host(x), xo, "x")
        assert_bitwise(host(v), vo, "v")
        assert_bitwise(host(c), co, "center")
        with pytest.raises(G.GsgdError):
            ctx.set_launch_width(9, 1)
        ctx.set_launch_width(G.KERNEL_GOSSIP, 0)          # back to the default

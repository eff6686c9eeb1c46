"""The blocked matrix layout (gsgd_config.block_columns): the same entry points
on matrices whose columns are stored in blocks, each block holding its k row
pieces back to back.  The oracle only knows row-major matrices, so every case
converts its inputs to the blocked order on the host, runs the library, converts
the results back and compares them with the oracle's, to the same bar as the
row-major tests (bit-exact; tolerance for push-gossip's fp64 sums and for
Gaussian noise).  Padding columns carry a sentinel that must survive."""
import numpy as np
import pytest

from paper_1611_04581_amd import workloads as W
from parity_util import assert_bitwise, assert_rows_close, assert_ulp_close

pytestmark = pytest.mark.gpu

SEED = 0x161104581


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _blocked(a, b):
    return _dev(W.to_blocked(a, b))


def _rowmajor(t, b):
    return W.from_blocked(t.cpu().numpy(), b)


@pytest.mark.parametrize("case", range(24))
def test_random_case_blocked(oracle, case):
    """The chain of every step rule of the row-major random cases, on blocked matrices: several blocks, a last
    block that ends inside a tile or inside a quad, vectors shorter than one block, a trailing unused block."""
    from paper_1611_04581_amd import gsgd as G
    rng = np.random.default_rng(5000 + case)
    k = int(rng.choice([1, 2, 3, 5, 7, 13, 17, 33, 64, 65]))
    b = int(rng.choice([1024, 2048, 8192]))
    d = int(rng.choice([1, 3, 1021, 1024, 1025, 2047, 2048, 4099, 8192, 8195, 9001, 17000, 20481]))
    ld = W.round_up(d, b) + b * int(rng.integers(0, 2))
    lr = float(rng.choice([0.01, 0.05, 0.3]))
    mu = float(rng.choice([0.0, 0.5, 0.9]))
    wd = float(rng.choice([0.0, 0.0, 1e-4, 0.01]))
    nest = bool(rng.integers(0, 2)) and mu > 0
    beta = float(rng.choice([0.5, 0.25, 0.7]))
    seg = {}
    lrc = lr
    if rng.integers(0, 2) and d >= 8:
        n_seg = int(rng.integers(1, min(d // 2, 40) + 1))
        off, sc = W.random_segments(d, n_seg, seed=case, align=int(rng.choice([1, 4])))
        seg = dict(seg_offsets=off, seg_lr_scale=sc)
        lrc = oracle.expand_lr(lr, d, off, sc)
    inp = W.make_inputs(k, d, ld, seed=6000 + case)
    perm = [int(t) for t in rng.permutation(k)]
    peer = [int(t) for t in rng.integers(0, k, size=k)]
    target = [int(t) for t in rng.integers(0, k, size=k)]
    i, j = int(rng.integers(0, k)), int(rng.integers(0, k))
    alpha_e = 0.9 / k
    split = int(rng.choice([G.ROW_SPLIT_AUTO, G.ROW_SPLIT_OFF, G.ROW_SPLIT_ON]))
    form = int(rng.choice([G.GOSSIP_AUTO, G.GOSSIP_WALK, G.GOSSIP_SWEEP, G.GOSSIP_SWEEP_SPLIT]))
    what = "k=%d d=%d ld=%d block=%d gossip form %d" % (k, d, ld, b, form)
    with G.Context(k, d, ld, lr=lr, momentum=mu, block_columns=b, **seg) as ctx:
        ctx.set_local_step(wd, nest)
        ctx.set_row_split(split)
        ctx.set_gossip_form(form)
        x, v, g, c = _blocked(inp.x, b), _blocked(inp.v, b), _blocked(inp.g, b), _dev(inp.center)
        xo, vo, co = inp.x.copy(), inp.v.copy(), inp.center.copy()
        ctx.step_gossip(x, v, g, perm, beta)
        oracle.step_gossip_ext(xo, vo, inp.g, lrc, mu, beta, perm, wd=wd, nesterov=nest, n=d)
        ctx.step_gossip_pull(x, v, g, peer, beta)
        oracle.step_gossip_ext(xo, vo, inp.g, lrc, mu, beta, peer, wd=wd, nesterov=nest, n=d)
        ctx.step_gossip_pull(x, v, g, peer, beta, True)
        oracle.step_gossip_ext(xo, vo, inp.g, lrc, mu, beta, peer, wd=wd, nesterov=nest, stale=True, n=d)
        ctx.step_gossip_stale(x, v, g, perm, beta)
        oracle.step_gossip_ext(xo, vo, inp.g, lrc, mu, beta, perm, wd=wd, nesterov=nest, stale=True, n=d)
        ctx.step_local(x, v, g)
        oracle.step_gossip_ext(xo, vo, inp.g, lrc, mu, 0.0, list(range(k)), wd=wd, nesterov=nest, n=d)
        ctx.step_async_tick(x, v, g, i, j, beta)
        oracle.async_tick(xo, vo, inp.g[i].copy(), lrc, mu, beta, i, j, wd=wd, nesterov=nest, n=d)
        ctx.step_easgd_tick(x, v, g, c, j, alpha_e)
        oracle.easgd_tick(xo, vo, inp.g[j].copy(), co, lrc, mu, alpha_e, j, wd=wd, nesterov=nest, n=d)
        assert_bitwise(_rowmajor(x, b), xo, "x before the k-way sums (%s)" % what)
        def after_k_way_sum(xo, vo, co, rule):
            if split == G.ROW_SPLIT_OFF:
                assert_bitwise(_rowmajor(x, b), xo, "%s x (%s)" % (rule, what))
                assert_bitwise(_rowmajor(v, b), vo, "%s v" % rule)
                assert_bitwise(c.cpu().numpy(), co, "%s center" % rule)
                return xo, vo, co
            # the row-split kernels add the replicas' terms in another order: same bar as their own tests
            assert_ulp_close(_rowmajor(x, b)[:, :d], xo[:, :d], "%s x (%s)" % (rule, what))
            assert_ulp_close(_rowmajor(v, b)[:, :d], vo[:, :d], "%s v" % rule)
            assert_ulp_close(c.cpu().numpy()[:d], co[:d], "%s center" % rule)
            assert_bitwise(_rowmajor(x, b)[:, d:], xo[:, d:], "x padding")
            assert_bitwise(_rowmajor(v, b)[:, d:], vo[:, d:], "v padding")
            assert_bitwise(c.cpu().numpy()[d:], co[d:], "center padding")
            # carry on from the library's own state so that later comparisons stay exact
            return _rowmajor(x, b), _rowmajor(v, b), c.cpu().numpy().copy()

        ctx.step_easgd(x, v, g, c, alpha_e)
        oracle.step_easgd_ext(xo, vo, inp.g, co, lrc, mu, alpha_e, wd=wd, nesterov=nest, n=d)
        xo, vo, co = after_k_way_sum(xo, vo, co, "easgd")
        ctx.step_allreduce(x, v, g)
        oracle.step_allreduce_ext(xo, vo, inp.g, lrc, mu, wd=wd, nesterov=nest, n=d)
        xo, vo, co = after_k_way_sum(xo, vo, co, "allreduce")
        ctx.step_gossip_push(x, v, g, target)
        oracle.step_gossip_push(xo, vo, inp.g, lrc, mu, target, wd=wd, nesterov=nest, n=d)
        xh = _rowmajor(x, b)
        assert_rows_close(xh[:, :d], xo[:, :d], "push x")
        assert_bitwise(xh[:, d:], xo[:, d:], "padding")
        assert_bitwise(_rowmajor(v, b), vo, "push v")
        assert_bitwise(_rowmajor(g, b), inp.g, "g is read-only")
        assert np.allclose(ctx.stats(x, _dev(inp.xstar)), oracle.stats(xh, inp.xstar, n=d), rtol=1e-10, atol=1e-300)
        assert np.allclose(ctx.row_sqnorms(x), (xh[:, :d].astype(np.float64) ** 2).sum(1), rtol=1e-12, atol=0)


@pytest.mark.parametrize("k,d,b", [(5, 3 * 1024 + 7, 1024), (9, 9 * 1024 + 5, 4096), (3, 700, 2048), (33, 70000, 65536)])
@pytest.mark.parametrize("kind", [1, 0])
def test_generator_and_fused_steps_blocked(oracle, k, d, b, kind):
    """init, gen_grad and the generator-fused steps: the noise of element (i, j) is keyed by its column and replica,
    not by where the layout puts it."""
    from paper_1611_04581_amd import gsgd as G
    ld = W.round_up(d, b)
    inp = W.make_inputs(k, d, ld, seed=71)
    sigma = 0.2
    with G.Context(k, d, ld, lr=0.05, momentum=0.9, sigma=sigma, seed=SEED, noise_kind=kind, block_columns=b) as ctx:
        h, xs, x0 = _dev(inp.h), _dev(inp.xstar), _dev(inp.x0)
        # initialisation, both modes (Gaussian draws per replica: tolerance)
        for mode in (G.INIT_BROADCAST, G.INIT_PER_REPLICA):
            x, v, c = _blocked(inp.x, b), _blocked(inp.v, b), _dev(inp.center)
            xo, vo, co = inp.x.copy(), inp.v.copy(), inp.center.copy()
            ctx.init_replicas(x, v, c, x0, mode)
            oracle.init_replicas(xo, vo, co, inp.x0, SEED, mode, n=d)
            assert_bitwise(_rowmajor(v, b), vo, "init v")
            if mode == G.INIT_BROADCAST:
                assert_bitwise(_rowmajor(x, b), xo, "init x")
                assert_bitwise(c.cpu().numpy(), co, "init center")
            else:
                assert_rows_close(_rowmajor(x, b)[:, :d], xo[:, :d], "init x")
                assert_bitwise(_rowmajor(x, b)[:, d:], xo[:, d:], "init x padding")
                assert_rows_close(c.cpu().numpy()[:d], co[:d], "init center")
        x, v, g = _blocked(inp.x, b), _blocked(inp.v, b), _blocked(inp.g, b)
        xo, vo, go = inp.x.copy(), inp.v.copy(), inp.g.copy()
        ctx.gen_grad(x, h, xs, g, 3)
        oracle.gen_grad(xo, inp.h, inp.xstar, go, sigma, SEED, 3, kind, n=d)
        gh = _rowmajor(g, b)
        if kind == 1:
            assert_bitwise(gh, go, "g")
        else:
            assert_rows_close(gh[:, :d], go[:, :d], "g")
            assert_bitwise(gh[:, d:], go[:, d:], "g padding")
        perm = G.make_perm(SEED, 4, k)
        peer = G.make_targets(SEED, 5, k)
        target = G.make_targets(SEED, 6, k, True) if k > 1 else [0]
        ctx.step_gossip_fused(x, v, h, xs, perm, 4, 0.5)
        oracle.gen_grad(xo, inp.h, inp.xstar, go, sigma, SEED, 4, kind, n=d)
        oracle.step_gossip(xo, vo, go, 0.05, 0.9, 0.5, perm, n=d)
        ctx.step_gossip_pull_fused(x, v, h, xs, peer, 5, 0.5)
        oracle.gen_grad(xo, inp.h, inp.xstar, go, sigma, SEED, 5, kind, n=d)
        oracle.step_gossip(xo, vo, go, 0.05, 0.9, 0.5, peer, n=d)
        if kind == 1:
            assert_bitwise(_rowmajor(x, b), xo, "fused x")
            assert_bitwise(_rowmajor(v, b), vo, "fused v")
        else:
            assert_rows_close(_rowmajor(x, b)[:, :d], xo[:, :d], "fused x")
            xo, vo = _rowmajor(x, b), _rowmajor(v, b)
        ctx.step_gossip_push_fused(x, v, h, xs, target, 6)
        oracle.gen_grad(xo, inp.h, inp.xstar, go, sigma, SEED, 6, kind, n=d)
        oracle.step_gossip_push(xo, vo, go, 0.05, 0.9, target, n=d)
        assert_rows_close(_rowmajor(x, b)[:, :d], xo[:, :d], "push fused x")
        assert_bitwise(_rowmajor(x, b)[:, d:], xo[:, d:], "padding")
        if kind == 1:
            # asynchronous ticks driven by the library (tick draw, generator, update)
            xo, vo = _rowmajor(x, b), _rowmajor(v, b)
            g_row = np.zeros(ld, np.float32)
            ctx.run_async_ticks(x, v, h, xs, 7, 12, 0.5)
            for t in range(7, 19):
                i, j = oracle.make_tick(SEED, t, k)
                oracle.gen_grad_row(xo, inp.h, inp.xstar, g_row, i, sigma, SEED, t, kind, n=d)
                oracle.async_tick(xo, vo, g_row, 0.05, 0.9, 0.5, i, j, n=d)
            assert_bitwise(_rowmajor(x, b), xo, "ticks x")
            assert_bitwise(_rowmajor(v, b), vo, "ticks v")


@pytest.mark.parametrize("k,b", [(8, 4096), (16, 16384), (17, 4096), (24, 16384), (36, 4096), (40, 16384), (48, 4096),
                                 (56, 16384), (64, 4096), (65, 16384), (100, 4096), (144, 16384)])
def test_the_form_the_library_picks_on_vectors_that_fill_the_chip(oracle, k, b):
    """More 1024-column tiles than compute units, so that the library's own choice of kernel is the one for long
    vectors (whole tiles with a thread per quad or under eight wavefronts, split tiles with one or two workgroups per
    compute unit and four, eight or twelve wavefronts), with a row length that ends inside a 256-column tile and inside
    a quad: every gossip rule, gradient given or drawn by the fused generator, bit-equal to the oracle."""
    from paper_1611_04581_amd import gsgd as G
    d = 263 * 1024 + 300 + 3
    ld = W.round_up(d, b)
    inp = W.make_inputs(k, d, ld, seed=700 + k)
    rng = np.random.default_rng(900 + k)
    sigma = 0.2
    with G.Context(k, d, ld, lr=0.05, momentum=0.9, sigma=sigma, seed=SEED, noise_kind=G.NOISE_UNIFORM,
                   block_columns=b) as ctx:
        h, xs = _dev(inp.h), _dev(inp.xstar)
        x, v, g = _blocked(inp.x, b), _blocked(inp.v, b), _blocked(inp.g, b)
        xo, vo, go = inp.x.copy(), inp.v.copy(), inp.g.copy()
        perm = [int(t) for t in rng.permutation(k)]
        peer = [int(t) for t in rng.integers(0, k, size=k)]
        target = [int(t) for t in rng.integers(0, k, size=k)]
        ctx.step_gossip(x, v, g, perm, 0.5)
        oracle.step_gossip(xo, vo, go, 0.05, 0.9, 0.5, perm, n=d)
        ctx.step_gossip_stale(x, v, g, perm, 0.3)
        oracle.step_gossip_ext(xo, vo, go, 0.05, 0.9, 0.3, perm, stale=True, n=d)
        ctx.step_gossip_pull(x, v, g, peer, 0.5)
        oracle.step_gossip(xo, vo, go, 0.05, 0.9, 0.5, peer, n=d)
        ctx.step_gossip_push(x, v, g, target)
        oracle.step_gossip_push(xo, vo, inp.g, 0.05, 0.9, target, n=d)
        ctx.step_gossip_fused(x, v, h, xs, perm, 21, 0.5)
        oracle.gen_grad(xo, inp.h, inp.xstar, go, sigma, SEED, 21, 1, n=d)
        oracle.step_gossip(xo, vo, go, 0.05, 0.9, 0.5, perm, n=d)
        ctx.step_gossip_pull_fused(x, v, h, xs, peer, 22, 0.5, True)
        oracle.gen_grad(xo, inp.h, inp.xstar, go, sigma, SEED, 22, 1, n=d)
        oracle.step_gossip_ext(xo, vo, go, 0.05, 0.9, 0.5, peer, stale=True, n=d)
        ctx.step_gossip_push_fused(x, v, h, xs, target, 23)
        oracle.gen_grad(xo, inp.h, inp.xstar, go, sigma, SEED, 23, 1, n=d)
        oracle.step_gossip_push(xo, vo, go, 0.05, 0.9, target, n=d)
        ctx.set_local_step(1e-3, True)
        ctx.step_gossip_push(x, v, g, target)
        oracle.step_gossip_push(xo, vo, inp.g, 0.05, 0.9, target, wd=1e-3, nesterov=True, n=d)
        assert_bitwise(_rowmajor(x, b), xo, "x (k=%d block=%d)" % (k, b))
        assert_bitwise(_rowmajor(v, b), vo, "v (k=%d block=%d)" % (k, b))
        assert_bitwise(_rowmajor(g, b), inp.g, "g is read-only")
        ctx.stats(x, xs)                # the tile counters of every launch above drained to zero


@pytest.mark.parametrize("b", [0, 1024, 4096])
@pytest.mark.parametrize("k", [1, 2, 16, 17, 19, 20, 36, 37, 48, 49, 64, 65, 72, 73, 144, 145, 200])
def test_gossip_forms_at_their_capacity_edges(oracle, k, b):
    """The walk and the two sweep forms of the pull-gossip step (fresh and stale parameters, gradient given or drawn
    by the fused generator), forced one after the other in one context, in both layouts: all bit-equal to the
    oracle.  The replica counts sit on either side of what each sweep form can park (36 / 144 rows); beyond it the call
    falls back to the next form.  16 / 17, 48 / 49 and 64 / 65 are the sizes the kernels are compiled
    for; 19, 20, 72 and 73 leave rows over after the full batches."""
    from paper_1611_04581_amd import gsgd as G
    d = 2 * 1024 + 256 + 7                      # two whole 1024-column tiles, one whole 256-column tile, a ragged rest
    ld = W.round_up(d, b or 4)
    inp = W.make_inputs(k, d, ld, seed=300 + k)
    rng = np.random.default_rng(k)
    sigma = 0.2
    lay = (lambda a: _blocked(a, b)) if b else _dev
    back = (lambda t: _rowmajor(t, b)) if b else (lambda t: t.cpu().numpy())
    with G.Context(k, d, ld, lr=0.05, momentum=0.9, sigma=sigma, seed=SEED, noise_kind=G.NOISE_UNIFORM,
                   block_columns=b) as ctx:
        h, xs = _dev(inp.h), _dev(inp.xstar)
        for form in (G.GOSSIP_WALK, G.GOSSIP_SWEEP, G.GOSSIP_SWEEP_SPLIT, G.GOSSIP_AUTO):
            ctx.set_gossip_form(form)
            x, v, g = lay(inp.x), lay(inp.v), lay(inp.g)
            xo, vo, go = inp.x.copy(), inp.v.copy(), inp.g.copy()
            perm = [int(t) for t in rng.permutation(k)]
            peer = [int(t) for t in rng.integers(0, k, size=k)]
            ctx.step_gossip(x, v, g, perm, 0.5)
            oracle.step_gossip(xo, vo, go, 0.05, 0.9, 0.5, perm, n=d)
            ctx.step_gossip_stale(x, v, g, perm, 0.3)
            oracle.step_gossip_ext(xo, vo, go, 0.05, 0.9, 0.3, perm, stale=True, n=d)
            ctx.step_gossip_pull(x, v, g, peer, 0.5)
            oracle.step_gossip(xo, vo, go, 0.05, 0.9, 0.5, peer, n=d)
            ctx.step_gossip_pull(x, v, g, peer, 0.7, True)
            oracle.step_gossip_ext(xo, vo, go, 0.05, 0.9, 0.7, peer, stale=True, n=d)
            ctx.step_gossip_fused(x, v, h, xs, perm, 11, 0.5)
            oracle.gen_grad(xo, inp.h, inp.xstar, go, sigma, SEED, 11, 1, n=d)
            oracle.step_gossip(xo, vo, go, 0.05, 0.9, 0.5, perm, n=d)
            ctx.step_gossip_pull_fused(x, v, h, xs, peer, 12, 0.5, True)
            oracle.gen_grad(xo, inp.h, inp.xstar, go, sigma, SEED, 12, 1, n=d)
            oracle.step_gossip_ext(xo, vo, go, 0.05, 0.9, 0.5, peer, stale=True, n=d)
            ctx.set_local_step(1e-3, True)          # the extended local step through the same forms
            ctx.step_gossip(x, v, g, perm, 0.5)
            oracle.step_gossip_ext(xo, vo, inp.g, 0.05, 0.9, 0.5, perm, wd=1e-3, nesterov=True, n=d)
            ctx.set_local_step(0.0, False)
            assert_bitwise(back(x), xo, "x (k=%d block=%d form=%d)" % (k, b, form))
            assert_bitwise(back(v), vo, "v (k=%d block=%d form=%d)" % (k, b, form))
            assert_bitwise(back(g), inp.g, "g is read-only")
            # push-gossip: the sweep forms add what a row received in the oracle's order (own value, then senders
            # ascending) and are bit-equal to it; the walk adds in visiting order (adjacent floats at worst)
            target = [int(t) for t in rng.integers(0, k, size=k)]
            ctx.step_gossip_push(x, v, g, target)
            oracle.step_gossip_push(xo, vo, inp.g, 0.05, 0.9, target, n=d)
            ctx.step_gossip_push_fused(x, v, h, xs, target, 13)
            oracle.gen_grad(xo, inp.h, inp.xstar, go, sigma, SEED, 13, 1, n=d)
            oracle.step_gossip_push(xo, vo, go, 0.05, 0.9, target, n=d)
            swept = form != G.GOSSIP_WALK and (form != G.GOSSIP_AUTO or b != 0) and k <= 144
            if swept:
                assert_bitwise(back(x), xo, "push x (k=%d block=%d form=%d)" % (k, b, form))
                assert_bitwise(back(v), vo, "push v")
            else:
                assert_rows_close(back(x)[:, :d], xo[:, :d], "push x (k=%d block=%d form=%d)" % (k, b, form))
                assert_bitwise(back(x)[:, d:], xo[:, d:], "push x padding")
        with pytest.raises(G.GsgdError) as e:
            ctx.set_gossip_form(4)
        assert e.value.code == G.ERR_INVALID_ARG


def test_blocked_and_row_major_contexts_agree_bitwise():
    """The layout moves elements, it does not change any of them: the same steps through a row-major and a blocked
    context give the same numbers (more than one tile per block, more blocks than workgroups need)."""
    import torch
    from paper_1611_04581_amd import gsgd as G
    k, b = 12, 4096
    d = 40 * 1024 + 13
    ld = W.round_up(d, b)
    inp = W.make_inputs(k, d, ld, seed=77)
    with G.Context(k, d, ld, sigma=0.3, seed=SEED) as row, G.Context(k, d, ld, sigma=0.3, seed=SEED, block_columns=b) as blk:
        h, xs, c1, c2 = _dev(inp.h), _dev(inp.xstar), _dev(inp.center), _dev(inp.center)
        x1, v1, g1 = _dev(inp.x), _dev(inp.v), _dev(inp.g)
        x2, v2, g2 = _blocked(inp.x, b), _blocked(inp.v, b), _blocked(inp.g, b)
        for t in range(6):
            for ctx, x, v, g, c in ((row, x1, v1, g1, c1), (blk, x2, v2, g2, c2)):
                ctx.gen_grad(x, h, xs, g, t)
                ctx.step_gossip(x, v, g, G.make_perm(SEED, t, k), 0.5)
                ctx.step_easgd(x, v, g, c, 0.05)
                ctx.step_allreduce(x, v, g)
                ctx.step_gossip_fused(x, v, h, xs, G.make_perm(SEED, 100 + t, k), 100 + t, 0.5)
        torch.cuda.synchronize()
        assert_bitwise(_rowmajor(x2, b), x1.cpu().numpy(), "x")
        assert_bitwise(_rowmajor(v2, b), v1.cpu().numpy(), "v")
        assert_bitwise(_rowmajor(g2, b), g1.cpu().numpy(), "g")
        assert_bitwise(c2.cpu().numpy(), c1.cpu().numpy(), "center")
        assert np.array_equal(row.stats(x1, xs), blk.stats(x2, xs))


@pytest.mark.parametrize("k", [5, 20])
def test_launch_widths_do_not_change_results_blocked(oracle, k):
    """On blocked matrices the local step and (from 12 replicas on) the generator run as persistent workgroups whose
    number gsgd_set_launch_width sets; below, the generator is a banded grid and the number is its band."""
    from paper_1611_04581_amd import gsgd as G
    b, d = 2048, 9 * 1024 + 5
    ld = W.round_up(d, b)
    inp = W.make_inputs(k, d, ld, seed=88)
    xo, vo, go = inp.x.copy(), inp.v.copy(), inp.g.copy()
    oracle.gen_grad(xo, inp.h, inp.xstar, go, 0.1, SEED, 4, 1, n=d)
    oracle.step_gossip_ext(xo, vo, go, 0.05, 0.9, 0.0, list(range(k)), n=d)
    with G.Context(k, d, ld, sigma=0.1, seed=SEED, noise_kind=G.NOISE_UNIFORM, block_columns=b) as ctx:
        h, xs = _dev(inp.h), _dev(inp.xstar)
        for width in (0, 1, 2, 3, 7, 64, 5000):
            for kern in (G.KERNEL_GEN_GRAD, G.KERNEL_LOCAL):
                ctx.set_launch_width(kern, width)
            x, v, g = _blocked(inp.x, b), _blocked(inp.v, b), _blocked(inp.g, b)
            ctx.gen_grad(x, h, xs, g, 4)
            ctx.step_local(x, v, g)
            assert_bitwise(_rowmajor(g, b), go, "g (width %d)" % width)
            assert_bitwise(_rowmajor(x, b), xo, "x (width %d)" % width)
            assert_bitwise(_rowmajor(v, b), vo, "v (width %d)" % width)
        ctx.stats(x, xs)          # the tile counters of every launch above drained to zero


@pytest.mark.parametrize("k,d", [(1, 5), (3, 1024), (7, 9 * 1024 + 6), (33, 70001)])
def test_relayout_moves_every_element_and_nothing_else(k, d):
    """gsgd_relayout against the host-side converters: row-major -> blocked -> another row stride -> another block
    width -> row-major; padding columns of every destination keep what they held."""
    import torch
    from paper_1611_04581_amd import gsgd as G
    rng = np.random.default_rng(k)
    src_ld = W.round_up(d, 4) + 8
    a = np.full((k, src_ld), -5.0, np.float32)
    a[:, :d] = rng.standard_normal((k, d)).astype(np.float32)
    cur, cur_ld, cur_b = _dev(a), src_ld, 0
    for (ld_unit, b) in ((2048, 2048), (4, 0), (65536, 65536), (1024, 1024), (4, 0)):
        ld = W.round_up(d, ld_unit) + (12 if b == 0 else 0)
        dst = torch.full((k, ld), 777.0, dtype=torch.float32, device="cuda")
        G.relayout(k, d, cur, cur_ld, cur_b, dst, ld, b)
        want = np.full((k, ld), 777.0, np.float32)
        want[:, :d] = a[:, :d]
        got = W.from_blocked(dst.cpu().numpy(), b) if b else dst.cpu().numpy()
        assert_bitwise(got, want, "k=%d d=%d into ld=%d block=%d" % (k, d, ld, b))
        cur, cur_ld, cur_b = dst, ld, b
    L = G.lib()
    p = cur.data_ptr()
    assert L.gsgd_relayout(k, d, cur_ld, 0, p, cur_ld, 0, p, None) == G.ERR_INVALID_ARG           # onto itself
    assert L.gsgd_relayout(k, d, cur_ld, 0, p, 3000, 3000, p + 4 * k * cur_ld, None) == G.ERR_INVALID_ARG
    assert L.gsgd_relayout(0, d, cur_ld, 0, p, cur_ld, 0, p, None) == G.ERR_INVALID_ARG


def test_block_columns_validation():
    from paper_1611_04581_amd import gsgd as G
    for bad in (-1024, 512, 1000, 3072):                  # negative, below a tile, not a power of two (twice)
        with pytest.raises(G.GsgdError) as e:
            G.Context(4, 4096, 4096 if bad <= 0 else W.round_up(4096, abs(bad)), block_columns=bad)
        assert e.value.code == G.ERR_INVALID_ARG
    with pytest.raises(G.GsgdError) as e:
        G.Context(4, 4000, 4000, block_columns=1024)      # ld is not a whole number of blocks
    assert e.value.code == G.ERR_INVALID_ARG
    import torch
    with G.Context(4, 4000, 4096, block_columns=1024) as ctx:
        short = torch.zeros(3 * 4 * 1024 + 3 * 1024 + 900, device="cuda")          # short of the span
        ok = torch.zeros(3 * 4 * 1024 + 3 * 1024 + 928, device="cuda")
        with pytest.raises(ValueError):
            ctx.step_local(short, ok.clone(), ok.clone())
        ctx.step_local(ok, ok.clone(), ok.clone())

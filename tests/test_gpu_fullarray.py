"""Tile-complete parity at the benchmark sizes, in the launch configuration
bench.py times (persistent workgroups pulling 1024-column tiles through the
ticket counter; matrices in the blocked layout each configuration is
benchmarked in, row length rounded up to whole blocks) and in the row-major
layout (row stride rounded up to 1024).

The small parity tests run at most a handful of tiles; here every one of the
11,416 (ResNet-18 size) or 24,959 (ResNet-50 size) tiles is compared with the
oracle, so a tile that the ticket loop dropped, handed out twice or gave to
the wrong columns cannot hide:

  * all-reduce (k = 8) and gossip (k = 32) at ResNet-18 size: FULL arrays of x
    and v, bit for bit, after 20 steps of generator + step (uniform noise);
  * gossip at the metric shape (k = 32, ResNet-50 size): FULL arrays after 5,
    12 and 20 steps;
  * elastic averaging (k = 16, ResNet-50 size): FULL arrays and the centre
    after 5 steps;
  * pull-gossip on iid targets (tree walk), stale-parameter gossip and
    push-gossip (k = 32, ResNet-18 size): FULL arrays after 6 steps;
  * segmented gossip at k = 128 (ResNet-50 layout, 39 GB of state): one whole
    quad of every tile, at a lane that changes from tile to tile, through 4
    steps (the oracle recomputes the gathered columns from the device's own g;
    the generator is compared on the same quads).

Each test stays well under a minute so that a run never looks hung.
"""
import numpy as np
import pytest

from paper_1611_04581_amd import workloads as W

pytestmark = pytest.mark.gpu
SIGMA = 0.1


@pytest.fixture(scope="module")
def G():
    import torch
    from paper_1611_04581_amd import gsgd
    assert torch.cuda.is_available()
    gsgd.lib()
    return gsgd


def _shared(d, ld, seed):
    rng = np.random.default_rng(seed)
    xstar = np.zeros(ld, np.float32)
    h = np.zeros(ld, np.float32)
    x0 = np.zeros(ld, np.float32)
    xstar[:d] = rng.standard_normal(d, dtype=np.float32)
    h[:d] = rng.uniform(0.1, 1.0, d).astype(np.float32)
    x0[:d] = rng.standard_normal(d, dtype=np.float32)
    return xstar, h, x0


LAYOUTS = ["blocked", "row_major"]


def _block_columns(cfg, layout):
    """The blocked layout the benchmark runs this configuration in, or 0 for row-major."""
    if layout == "row_major":
        return 0
    assert cfg.block_columns > 0
    return cfg.block_columns


def _assert_full_equal(dev_t, ref, d, what, block_columns=0):
    """Whole k x d array on the device against the oracle's, bit for bit; names the first differing tile."""
    if block_columns and dev_t.dim() == 2 and dev_t.shape[0] > 1:
        dev_t = W.from_blocked(dev_t, block_columns)
    got = dev_t.cpu().numpy()
    a = got[:, :d].view(np.uint32)
    b = ref[:, :d].view(np.uint32)
    if np.array_equal(a, b):
        return
    bad = np.argwhere(a != b)
    i, j = bad[0]
    raise AssertionError("%s: %d of %d elements differ; first at replica %d column %d (tile %d): %r vs %r"
                         % (what, len(bad), a.size, i, j, j // 1024, got[i, j], ref[i, j]))


class _Run:
    """One benchmark configuration advanced step by step on both sides, whole arrays."""

    def __init__(self, G, oracle, cfg, block_columns=0):
        import torch
        self.G, self.oracle, self.cfg, self.b = G, oracle, cfg, block_columns
        k, d = cfg.k, cfg.d
        self.k, self.d, self.ld = k, d, W.round_up(d, block_columns or 1024)
        ld = self.ld
        self.xstar, self.h, x0 = _shared(d, ld, seed=1234)
        self.ctx = G.Context(k, d, ld, lr=cfg.lr, momentum=cfg.momentum, sigma=SIGMA, seed=cfg.seed,
                             noise_kind=G.NOISE_UNIFORM, block_columns=block_columns)
        self.x = torch.empty((k, ld), dtype=torch.float32, device="cuda")
        self.v = torch.empty_like(self.x)
        self.g = torch.empty_like(self.x)
        self.c = torch.empty(ld, dtype=torch.float32, device="cuda")
        self.dh, self.dxs, dx0 = (torch.from_numpy(a).cuda() for a in (self.h, self.xstar, x0))
        self.ctx.init_replicas(self.x, self.v, self.c, dx0, G.INIT_BROADCAST)
        self.xo = np.empty((k, ld), np.float32)
        self.vo = np.empty((k, ld), np.float32)
        self.go = np.zeros((k, ld), np.float32)
        self.co = np.empty(ld, np.float32)
        oracle.init_replicas(self.xo, self.vo, self.co, x0, cfg.seed, 0, n=d)
        self.lrc = np.full(d, np.float32(cfg.lr), np.float32)
        self.t = 0

    def advance(self, until):
        G, o, cfg, d = self.G, self.oracle, self.cfg, self.d
        while self.t < until:
            t = self.t
            self.ctx.gen_grad(self.x, self.dh, self.dxs, self.g, t)
            o.gen_grad(self.xo, self.h, self.xstar, self.go, SIGMA, cfg.seed, t, 1, n=d)
            if cfg.rule == "gossip":
                perm = G.make_perm(cfg.seed, t, self.k)
                self.ctx.step_gossip(self.x, self.v, self.g, perm, cfg.beta)
                o.step_gossip(self.xo, self.vo, self.go, self.lrc, cfg.momentum, cfg.beta, perm, n=d)
            elif cfg.rule == "gossip_pull":                       # iid targets: the tree walk
                peer = G.make_targets(cfg.seed, t, self.k)
                self.ctx.step_gossip_pull(self.x, self.v, self.g, peer, cfg.beta)
                o.step_gossip(self.xo, self.vo, self.go, self.lrc, cfg.momentum, cfg.beta, peer, n=d)
            elif cfg.rule == "gossip_stale":
                perm = G.make_perm(cfg.seed, t, self.k)
                self.ctx.step_gossip_stale(self.x, self.v, self.g, perm, cfg.beta)
                o.step_gossip_ext(self.xo, self.vo, self.go, self.lrc, cfg.momentum, cfg.beta, perm, stale=True, n=d)
            elif cfg.rule == "gossip_push":                       # senders-first walk, fp64 sums in visiting order
                target = G.make_targets(cfg.seed, t, self.k, True)
                self.ctx.step_gossip_push(self.x, self.v, self.g, target)
                o.step_gossip_push(self.xo, self.vo, self.go, self.lrc, cfg.momentum, target, n=d)
            elif cfg.rule == "allreduce":
                self.ctx.step_allreduce(self.x, self.v, self.g)
                o.step_allreduce(self.xo, self.vo, self.go, self.lrc, cfg.momentum, n=d)
            else:
                self.ctx.step_easgd(self.x, self.v, self.g, self.c, cfg.alpha_e)
                o.step_easgd(self.xo, self.vo, self.go, self.co, self.lrc, cfg.momentum, cfg.alpha_e, n=d)
            self.t += 1

    def rows(self, t):
        """A device matrix as k row-major rows, whatever layout the context keeps it in."""
        return W.from_blocked(t, self.b) if self.b else t

    def check(self):
        what = "%s after %d steps (block_columns %d)" % (self.cfg.name, self.t, self.b)
        if self.cfg.rule == "gossip_push":
            # both sides round fp64 sums taken in different orders: adjacent floats at worst, and a last-place
            # difference then travels through the later steps, so the bar is the parameter tolerance on every element
            got = self.rows(self.x).cpu().numpy()[:, :self.d]
            ref = self.xo[:, :self.d]
            assert np.abs(got.astype(np.float64) - ref).max() <= 1e-6 * max(1.0, np.abs(ref).max()), what
            assert (got.view(np.uint32) == ref.view(np.uint32)).mean() >= 0.9999, what
            return
        _assert_full_equal(self.x, self.xo, self.d, what + ": x", self.b)
        _assert_full_equal(self.v, self.vo, self.d, what + ": v", self.b)
        if self.cfg.rule == "easgd":
            _assert_full_equal(self.c[None], self.co[None], self.d, what + ": center")
        st = self.ctx.stats(self.x, self.dxs)          # also checks that the stream's tile counters drained to zero
        assert np.isfinite(st).all()

    def close(self):
        self.ctx.close()


@pytest.mark.parametrize("layout", LAYOUTS)
def test_allreduce_resnet18_full_arrays_20_steps(G, oracle, layout):
    cfg = W.CONFIGS["allreduce_r18"]
    run = _Run(G, oracle, cfg, _block_columns(cfg, layout))
    try:
        run.advance(20)
        run.check()
        xr = run.rows(run.x)
        assert bool((xr[1:, :run.d] == xr[0, :run.d]).all())      # identical start: replicas stay identical
    finally:
        run.close()


@pytest.mark.parametrize("layout", LAYOUTS)
def test_gossip_resnet18_full_arrays_20_steps(G, oracle, layout):
    cfg = W.CONFIGS["gossip_r18"]
    run = _Run(G, oracle, cfg, _block_columns(cfg, layout))
    try:
        run.advance(20)
        run.check()
    finally:
        run.close()


@pytest.mark.parametrize("layout", LAYOUTS)
def test_easgd_resnet50_full_arrays_5_steps(G, oracle, layout):
    cfg = W.CONFIGS["easgd_r50"]
    run = _Run(G, oracle, cfg, _block_columns(cfg, layout))
    try:
        run.advance(5)
        run.check()
    finally:
        run.close()


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("rule", ["gossip_pull", "gossip_stale", "gossip_push"])
def test_other_gossip_forms_resnet18_full_arrays(G, oracle, rule, layout):
    """Tree walk (iid pull targets), stale parameters and the senders-first push walk, k = 32 at ResNet-18 size,
    every tile, 6 steps from a common start (the noise spreads the replicas from the first step on)."""
    base = W.CONFIGS["gossip_r18"]
    cfg = W.Config("%s_r18" % rule, rule, base.k, base.d, 6, block_columns=base.block_columns)
    run = _Run(G, oracle, cfg, _block_columns(cfg, layout))
    try:
        run.advance(6)
        run.check()
    finally:
        run.close()


@pytest.fixture(scope="module", params=LAYOUTS)
def metric_run(request, G, oracle):
    cfg = W.CONFIGS["gossip_r50"]
    run = _Run(G, oracle, cfg, _block_columns(cfg, request.param))
    yield run
    run.close()


@pytest.mark.parametrize("until", [5, 12, 20])
def test_gossip_metric_shape_full_arrays(metric_run, until):
    """k = 32, ResNet-50 size, the shape bench.py reports: the run is carried from one checkpoint to the next."""
    assert metric_run.t <= until
    metric_run.advance(until)
    metric_run.check()


@pytest.mark.parametrize("layout", LAYOUTS)
def test_segmented_gossip_k128_one_quad_of_every_tile(G, oracle, layout):
    import torch
    cfg = W.CONFIGS["seg_gossip_r50_k128"]
    k, d = cfg.k, cfg.d
    b = _block_columns(cfg, layout)
    ld = W.round_up(d, b or 1024)
    off, sc, _ = W.resnet_layout(cfg.layout)
    n_tiles = W.round_up(d, 1024) // 1024
    tiles = np.arange(n_tiles, dtype=np.int64)
    lane = (tiles * 37 + 11) % 256                       # a different lane of the workgroup in every tile
    first = tiles * 1024 + lane * 4
    first = np.minimum(first, (d - 4) // 4 * 4)          # the ragged last tile: its last whole quad
    cols = (first[:, None] + np.arange(4)[None, :]).reshape(-1)
    assert cols.max() < d and len(np.unique(cols // 1024)) == n_tiles
    lr_full = oracle.expand_lr(cfg.lr, d, off, sc)
    lr_cols = np.ascontiguousarray(lr_full[cols])
    xstar, h, x0 = _shared(d, ld, seed=4321)
    cols_t = torch.from_numpy(cols).cuda()
    if b:
        # where the blocked layout keeps element (i, col): (col / b) * k * b + i * b + col % b
        flat_t = (torch.from_numpy((cols // b) * k * b + cols % b).cuda()[None, :]
                  + torch.arange(k, device="cuda", dtype=torch.int64)[:, None] * b)
    with G.Context(k, d, ld, lr=cfg.lr, momentum=cfg.momentum, sigma=SIGMA, seed=cfg.seed, noise_kind=G.NOISE_UNIFORM,
                   seg_offsets=off, seg_lr_scale=sc, block_columns=b) as ctx:
        x = torch.empty((k, ld), dtype=torch.float32, device="cuda")
        v = torch.empty_like(x)
        g = torch.empty_like(x)
        dh, dxs, dx0 = (torch.from_numpy(a).cuda() for a in (h, xstar, x0))
        ctx.init_replicas(x, v, None, None, G.INIT_PER_REPLICA)    # a spread start: every row differs

        def gather(t):
            if b:
                return np.ascontiguousarray(torch.take(t, flat_t).cpu().numpy())
            return np.ascontiguousarray(t.index_select(1, cols_t).cpu().numpy())

        for t in range(4):
            ctx.gen_grad(x, dh, dxs, g, t)
            xs_, vs_, gs_ = gather(x), gather(v), gather(g)
            # the generator on the same quads: the oracle draws a quad from its global column
            go = np.zeros((k, 4), np.float32)
            for q in (0, 1, n_tiles // 2, n_tiles - 2, n_tiles - 1):
                c0 = int(first[q])
                oracle.gen_grad(np.ascontiguousarray(xs_[:, 4 * q:4 * q + 4]), h[c0:c0 + 4].copy(), xstar[c0:c0 + 4].copy(),
                                go, SIGMA, cfg.seed, t, 1, col0=c0)
                assert np.array_equal(go.view(np.uint32), gs_[:, 4 * q:4 * q + 4].view(np.uint32)), (t, q)
            perm = G.make_perm(cfg.seed, t, k)
            ctx.step_gossip(x, v, g, perm, cfg.beta)
            oracle.step_gossip(xs_, vs_, gs_, lr_cols, cfg.momentum, cfg.beta, perm)
            gx, gv = gather(x), gather(v)
            for name, got, want in (("x", gx, xs_), ("v", gv, vs_)):
                same = got.view(np.uint32) == want.view(np.uint32)
                if not same.all():
                    i, j = np.argwhere(~same)[0]
                    raise AssertionError("step %d: %s differs in tile %d (replica %d, column %d): %r vs %r; %d quads off"
                                         % (t, name, j // 4, i, cols[j], got[i, j], want[i, j],
                                            len(np.unique(np.argwhere(~same)[:, 1] // 4))))
        ctx.stats(x, dxs)

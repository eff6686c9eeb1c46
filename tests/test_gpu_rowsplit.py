"""The k-way sums with the rows split over the wavefronts of a workgroup and
staged through LDS (the layout short vectors get): all-reduce and elastic
averaging against the oracle and against the serial-order kernels.

The split associates the same fp64 additions differently, so the bar is that of
push-gossip: bit-equal on at least 99.99 % of the elements, adjacent floats
elsewhere; what does not go through the sum (momentum buffers and parameters of
elastic averaging, padding) must be bit-equal."""
import numpy as np
import pytest

from paper_1611_04581_amd import workloads as W
from parity_util import assert_bitwise, assert_ulp_close

pytestmark = pytest.mark.gpu
SEED = W.DEFAULT_SEED
# (k, d, ld): 4 wavefronts per workgroup below k = 48, 16 from there on; ragged tails; fewer rows than wavefronts
SHAPES = [(8, 5 * 1024 + 7, None), (32, 2 * 1024 + 2, 4096), (3, 1, 4), (5, 255, 256), (48, 777, None),
          (128, 1024 + 12, None), (512, 300, None), (17, 4 * 256, None)]


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
    return np.ascontiguousarray(t.cpu().numpy())


@pytest.mark.parametrize("k,d,ld", SHAPES)
@pytest.mark.parametrize("wd,nesterov", [(0.0, False), (1e-4, True)])
def test_row_split_allreduce_and_easgd(G, oracle, k, d, ld, wd, nesterov):
    ld = ld or W.round_up(d, 4)
    inp = W.make_inputs(k, d, ld, seed=700 + k)
    alpha_e = 0.9 / k
    with G.Context(k, d, ld, lr=0.05, momentum=0.9) as ctx:
        ctx.set_local_step(wd, nesterov)
        res = {}
        for mode in (G.ROW_SPLIT_ON, G.ROW_SPLIT_OFF):
            ctx.set_row_split(mode)
            x, v = dev(inp.x), dev(inp.v)
            ctx.step_allreduce(x, v, dev(inp.g))
            xe, ve, ce = dev(inp.x), dev(inp.v), dev(inp.center)
            ctx.step_easgd(xe, ve, dev(inp.g), ce, alpha_e)
            res[mode] = [host(t) for t in (x, v, xe, ve, ce)]
        xo, vo = inp.x.copy(), inp.v.copy()
        oracle.step_allreduce_ext(xo, vo, inp.g, 0.05, 0.9, wd=wd, nesterov=nesterov, n=d)
        xeo, veo, ceo = inp.x.copy(), inp.v.copy(), inp.center.copy()
        oracle.step_easgd_ext(xeo, veo, inp.g, ceo, 0.05, 0.9, alpha_e, wd=wd, nesterov=nesterov, n=d)
        x, v, xe, ve, ce = res[G.ROW_SPLIT_ON]
        assert_ulp_close(x[:, :d], xo[:, :d], "all-reduce x")
        assert_ulp_close(v[:, :d], vo[:, :d], "all-reduce v")
        assert_bitwise(x[:, d:], xo[:, d:], "x padding")
        assert_bitwise(v[:, d:], vo[:, d:], "v padding")
        assert all(np.array_equal(v[0, :d], v[i, :d]) for i in range(1, k))      # every node got the same average
        assert_bitwise(xe, xeo, "elastic averaging x")                           # per-row updates do not see the sum
        assert_bitwise(ve, veo, "elastic averaging v")
        assert_ulp_close(ce[:d], ceo[:d], "centre")
        assert_bitwise(ce[d:], ceo[d:], "centre padding")
        # the serial-order kernels on the same inputs are the oracle bit for bit
        x, v, xe, ve, ce = res[G.ROW_SPLIT_OFF]
        assert_bitwise(x, xo, "serial all-reduce x")
        assert_bitwise(ce, ceo, "serial centre")


def test_row_split_with_segments_and_a_trajectory(G, oracle):
    """Per-layer step sizes, 30 steps of all-reduce from identical rows with
    uniform noise (the layout AUTO picks for this short vector): rows stay
    identical, and the trajectory follows the oracle's."""
    k, d, steps = 64, 9 * 1024 + 5, 30
    ld = W.round_up(d, 1024)
    off, sc = W.random_segments(d, 37, seed=3, align=1)
    lrc = oracle.expand_lr(0.05, d, off, sc)
    inp = W.make_inputs(k, d, ld, seed=701, identical_rows=True)
    xo, vo, go = inp.x.copy(), np.zeros_like(inp.v), inp.g.copy()
    with G.Context(k, d, ld, lr=0.05, momentum=0.9, sigma=0.1, seed=SEED, noise_kind=G.NOISE_UNIFORM,
                   seg_offsets=off, seg_lr_scale=sc) as ctx:
        x, v, g = dev(xo), dev(vo), dev(go)
        h, xs = dev(inp.h), dev(inp.xstar)
        for t in range(steps):
            ctx.gen_grad(x, h, xs, g, t)
            ctx.step_allreduce(x, v, g)                        # AUTO: 10 tiles < compute units, k >= 16 -> row split
            oracle.gen_grad(xo, inp.h, inp.xstar, go, 0.1, SEED, t, 1, n=d)
            oracle.step_allreduce(xo, vo, go, lrc, 0.9, n=d)
        got = host(x)
        assert all(np.array_equal(got[0, :d], got[i, :d]) for i in range(1, k))
        assert np.abs(got[:, :d].astype(np.float64) - xo[:, :d]).max() <= 1e-6 * max(1.0, np.abs(xo[:, :d]).max())
        assert (got[:, :d] == xo[:, :d]).mean() > 0.999
        ctx.stats(x, xs)
    with pytest.raises(G.GsgdError):
        ctx2 = G.Context(2, 16)
        try:
            ctx2.set_row_split(7)
        finally:
            ctx2.close()

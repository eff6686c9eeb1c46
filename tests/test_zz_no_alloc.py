"""The statistics call that allocates nothing (gsgd_stats_static) against the
context's gsgd_stats: same kernels, same order, so the four numbers must be
bit-identical; two calls in a row, the second on a smaller input, share the
library's fixed scratch array."""
import numpy as np
import pytest

from paper_1611_04581_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_stats_static_matches_stats_twice_in_a_row_second_smaller():
    import torch
    from paper_1611_04581_amd import gsgd as G
    assert torch.cuda.is_available()
    out = torch.zeros(4, dtype=torch.float64, device="cuda")
    # 701 tiles over 512 workgroups' partial sums, then 10 tiles; then the same pair on blocked matrices (blocks of
    # 2048 columns)
    for (k, d, b) in [(32, 700 * 1024 + 13, 0), (5, 9 * 1024 + 2, 0), (32, 700 * 1024 + 13, 2048), (5, 9 * 1024 + 2, 2048)]:
        ld = W.round_up(d, b or 1024)
        inp = W.make_inputs(k, d, ld, seed=31 + k)
        x = torch.from_numpy(W.to_blocked(inp.x, b) if b else inp.x).cuda()
        xs = torch.from_numpy(inp.xstar).cuda()
        out.fill_(-1.0)
        G.stats_static(k, d, ld, x, xs, out, block_columns=b)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        with G.Context(k, d, ld, block_columns=b) as ctx:
            want = ctx.stats(x, xs)
        assert np.array_equal(got, want), (k, d, b, got, want)
        # and both are the plain fp64 definition to rounding
        x64 = inp.x[:, :d].astype(np.float64)
        xbar = x64.mean(0)
        ref = np.array([((x64 - xbar) ** 2).sum(), ((x64 - inp.xstar[:d]) ** 2).sum(),
                        ((xbar - inp.xstar[:d]) ** 2).sum(), (xbar ** 2).sum()])
        assert np.allclose(got, ref, rtol=1e-11, atol=0)


def test_stats_static_rejects_what_it_is_not_specified_for():
    import torch
    from paper_1611_04581_amd import gsgd as G
    x = torch.zeros(4096, dtype=torch.float32, device="cuda")
    out = torch.zeros(4, dtype=torch.float64, device="cuda")
    L = G.lib()
    too_big = G.STATS_STATIC_MAX_D + 4
    # sizes beyond the stated maximum are refused before anything is launched (the pointers are never followed)
    assert L.gsgd_stats_static(1, too_big, too_big, 0, x.data_ptr(), x.data_ptr(), out.data_ptr(), None) == G.ERR_TOO_LARGE
    assert "GSGD_STATS_STATIC_MAX_D" in G.strerror(G.ERR_TOO_LARGE)
    assert L.gsgd_stats_static(0, 16, 16, 0, x.data_ptr(), x.data_ptr(), out.data_ptr(), None) == G.ERR_INVALID_ARG
    assert L.gsgd_stats_static(1, 16, 18, 0, x.data_ptr(), x.data_ptr(), out.data_ptr(), None) == G.ERR_INVALID_ARG
    assert L.gsgd_stats_static(1, 16, 16, 0, x.data_ptr(), x.data_ptr(), None, None) == G.ERR_INVALID_ARG
    # a block that is not a power of two, or that does not divide the row length
    assert L.gsgd_stats_static(1, 3000, 3072, 3072, x.data_ptr(), x.data_ptr(), out.data_ptr(), None) == G.ERR_INVALID_ARG
    assert L.gsgd_stats_static(1, 3000, 3072, 2048, x.data_ptr(), x.data_ptr(), out.data_ptr(), None) == G.ERR_INVALID_ARG
    with pytest.raises(ValueError):
        G.stats_static(1, 16, 16, x, x, out.float())

"""Helpers shared by the GPU parity tests: tolerances and array plumbing."""
import numpy as np

# Floating-point bar of the parity tests.  Per replica row a (GPU) vs b (oracle):
#   max_j |a_j - b_j| <= 1e-6 * max(1, ||b||_inf)   and   ||a - b||_2 <= 1e-6 * ||b||_2.
# Near-zero coordinates make a per-element relative error meaningless, hence
# the row-wise norms.  The replica mean must be preserved by the gossip mix to
# 1e-5 * max(1, ||mean||_inf).
PARAM_RTOL = 1e-6
MEAN_RTOL = 1e-5


def assert_rows_close(a, b, what="x", rtol=PARAM_RTOL):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    if a.ndim == 1:
        a, b = a[None], b[None]
    for i in range(a.shape[0]):
        diff = np.abs(a[i] - b[i])
        bound = rtol * max(1.0, np.abs(b[i]).max())
        assert diff.max() <= bound, "%s row %d: max abs diff %.3e > %.3e" % (what, i, diff.max(), bound)
        l2 = np.linalg.norm(a[i] - b[i])
        ref = np.linalg.norm(b[i])
        assert l2 <= rtol * ref + 1e-30, "%s row %d: l2 diff %.3e > %.3e" % (what, i, l2, rtol * ref)


def assert_bitwise(a, b, what="x"):
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    assert a.shape == b.shape and a.dtype == b.dtype
    same = a.view(np.uint32) == b.view(np.uint32) if a.dtype == np.float32 else a == b
    if not same.all():
        idx = np.argwhere(~same)[0]
        raise AssertionError("%s differs bitwise at %s: %r vs %r (%d of %d elements differ)"
                             % (what, tuple(idx), a[tuple(idx)], b[tuple(idx)], (~same).sum(), same.size))


def mean_preserved(before, after, rtol=MEAN_RTOL):
    mb = np.asarray(before, dtype=np.float64).mean(0)
    ma = np.asarray(after, dtype=np.float64).mean(0)
    bound = rtol * max(1.0, np.abs(mb).max())
    assert np.abs(ma - mb).max() <= bound, "replica mean moved by %.3e > %.3e" % (np.abs(ma - mb).max(), bound)


def assert_ulp_close(got, want, what="x", min_equal=0.9999):
    """fp32 arrays bit-equal on at least `min_equal` of the elements and adjacent
    floats elsewhere: the bar for results that round one fp64 sum whose
    additions the two sides associate differently."""
    a = np.ascontiguousarray(got).view(np.int32).astype(np.int64)
    b = np.ascontiguousarray(want).view(np.int32).astype(np.int64)
    # map the sign-magnitude bit patterns to a monotone integer line (so -0 and +0 are neighbours)
    a = np.where(a < 0, -(a & 0x7FFFFFFF) - 1, a)
    b = np.where(b < 0, -(b & 0x7FFFFFFF) - 1, b)
    steps = np.abs(a - b)
    assert steps.max() <= 1, "%s: %d units in the last place apart" % (what, steps.max())
    assert (steps == 0).mean() >= min_equal, "%s: only %.6f bit-equal" % (what, (steps == 0).mean())

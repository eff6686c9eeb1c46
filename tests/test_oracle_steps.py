"""Pins for the oracle's update rules: synthetic gradient, local momentum step,
gossip mix, all-reduce average, elastic averaging, segmented step sizes and the
statistics.  CPU only.

What each rule is tied to:
  * exact replay -- the same operation sequence re-done in pure Python on exact
    rationals with an explicit round-to-nearest-binary32 after each operation;
  * brute force over all permutations of k <= 4 replicas;
  * invariants the paper's analysis rests on (doubly stochastic mixing keeps
    the mean; E[M^T M] = (I + 11^T/k)/2 halves the expected consensus distance,
    Section 6.1.1);
  * closed forms: the heavy-ball linear recurrence, the EASGD centre update,
    the stationary variance from a discrete Lyapunov equation;
  * the convergence bound of the synchronous pull-gossip theorem.
"""
import math
from fractions import Fraction
from itertools import product

import numpy as np
import pytest
from scipy import linalg as sla

import brute
from paper_1611_04581_amd import workloads as W

F = lambda a: Fraction(float(a))
SEED = 0x161104581


def _dyadic(rng, shape, bits=6, scale=8):
    """Small dyadic rationals: exactly representable, sums/halves stay exact."""
    return (rng.integers(-(1 << bits), 1 << bits, shape) / float(scale)).astype(np.float32)


# ----------------------------------------------------------------------------
# synthetic gradient

def test_gen_grad_exact_replay_uniform_noise(oracle):
    k, n, col0, step = 3, 13, 6, 41
    sigma = np.float32(0.3)
    inp = W.make_inputs(k, n, seed=1)
    g = np.zeros_like(inp.x)
    oracle.gen_grad(inp.x, inp.h, inp.xstar, g, sigma, SEED, step, oracle.NOISE_UNIFORM, col0=col0)
    key = (SEED & 0xFFFFFFFF, SEED >> 32)
    for i, j in product(range(k), range(n)):
        gj = col0 + j
        word = brute.philox4((gj // 4, i, step, 0), key)[gj % 4]
        xi = brute.uniform_noise_exact(word)
        t1 = brute.f32_sub(F(inp.x[i, j]), F(inp.xstar[j]))
        t2 = brute.f32_mul(F(sigma), xi)
        assert F(g[i, j]) == brute.f32_fma(F(inp.h[j]), t1, t2)


def test_gen_grad_gaussian_is_quadratic_gradient_plus_noise(oracle):
    k, n = 4, 4096
    inp = W.make_inputs(k, n, seed=2)
    g0 = np.zeros_like(inp.x)
    g1 = np.zeros_like(inp.x)
    oracle.gen_grad(inp.x, inp.h, inp.xstar, g0, 0.0, SEED, 0)
    want = inp.h.astype(np.float64) * (inp.x.astype(np.float64) - inp.xstar.astype(np.float64))
    assert np.allclose(g0, want, rtol=3e-7, atol=1e-7)
    sigma = 0.25
    oracle.gen_grad(inp.x, inp.h, inp.xstar, g1, sigma, SEED, 0)
    z = (g1.astype(np.float64) - want) / sigma
    assert abs(z.mean()) < 4 / math.sqrt(z.size)
    assert abs(z.var() - 1.0) < 0.05
    # independent across replicas and across steps
    assert abs(np.corrcoef(z[0], z[1])[0, 1]) < 0.06
    g2 = np.zeros_like(inp.x)
    oracle.gen_grad(inp.x, inp.h, inp.xstar, g2, sigma, SEED, 1)
    z2 = (g2.astype(np.float64) - want) / sigma
    assert abs(np.corrcoef(z.ravel(), z2.ravel())[0, 1]) < 0.03
    # slice at an unaligned global column == that part of the whole
    gs = np.zeros((k, 100), np.float32)
    oracle.gen_grad(np.ascontiguousarray(inp.x[:, 333:433]), inp.h[333:433].copy(), inp.xstar[333:433].copy(),
                    gs, sigma, SEED, 0, col0=333)
    assert np.array_equal(gs, g1[:, 333:433])


# ----------------------------------------------------------------------------
# local momentum step + gossip mix

def _replay_gossip(x, v, g, lr, mu, beta, peer):
    k, n = x.shape
    xp = [[None] * n for _ in range(k)]
    vn = [[None] * n for _ in range(k)]
    for i, j in product(range(k), range(n)):
        t3 = brute.f32_mul(F(mu), F(v[i, j]))
        vn[i][j] = brute.f32_fma(-F(lr), F(g[i, j]), t3)
        xp[i][j] = brute.f32_add(F(x[i, j]), vn[i][j])
    xn = [[brute.f32_fma(-F(beta), brute.f32_sub(xp[i][j], xp[peer[i]][j]), xp[i][j]) for j in range(n)]
          for i in range(k)]
    return xn, vn


@pytest.mark.parametrize("beta", [0.5, 0.3])
def test_gossip_step_exact_replay(oracle, beta):
    k, n = 4, 9
    lr, mu, beta = np.float32(0.05), np.float32(0.9), np.float32(beta)
    for trial, peer in enumerate([[1, 2, 3, 0], [0, 1, 2, 3], [1, 0, 3, 2], [2, 2, 0, 1]]):
        inp = W.make_inputs(k, n, seed=10 + trial)
        xn, vn = _replay_gossip(inp.x, inp.v, inp.g, lr, mu, beta, peer)
        oracle.step_gossip(inp.x, inp.v, inp.g, lr, mu, beta, peer)
        for i, j in product(range(k), range(n)):
            assert F(inp.x[i, j]) == xn[i][j]
            assert F(inp.v[i, j]) == vn[i][j]


@pytest.mark.parametrize("k", [2, 3, 4])
def test_gossip_mix_brute_force_all_permutations(oracle, k):
    """With lr = 0, mu = 0 the local step is the identity, so the call is the
    pure mix; on dyadic inputs it must equal the exact rational mix."""
    rng = np.random.default_rng(k)
    n = 5
    for beta in (0.5, 0.25):
        for peer in brute.all_permutations(k):
            x = _dyadic(rng, (k, n))
            v = np.zeros((k, n), np.float32)
            g = _dyadic(rng, (k, n))
            want = brute.gossip_mix_exact([[F(t) for t in row] for row in x], peer, Fraction(beta))
            oracle.step_gossip(x, v, g, 0.0, 0.0, beta, peer)
            assert [[F(t) for t in row] for row in x] == want
            assert not v.any()


@pytest.mark.parametrize("k", [2, 3, 4])
def test_expected_consensus_halves_over_uniform_permutations(oracle, k):
    """E[M^T M] = (I + 11^T/k)/2 (Section 6.1.1) holds for a uniformly random
    permutation target as it does for iid targets, because E[P] = 11^T/k:
    averaged over all k! permutations the consensus distance after one pure
    gossip round with beta = 1/2 is exactly half of what it was."""
    rng = np.random.default_rng(100 + k)
    n = 4
    x0 = _dyadic(rng, (k, n))
    before = brute.consensus_distance(x0.tolist())
    total = Fraction(0)
    perms = brute.all_permutations(k)
    for peer in perms:
        x = x0.copy()
        oracle.step_gossip(x, np.zeros_like(x), np.zeros_like(x), 0.0, 0.0, 0.5, peer)
        total += brute.consensus_distance([[F(t) for t in row] for row in x])
    assert total / len(perms) == before / 2


def test_gossip_invariants(oracle):
    k, n = 8, 257
    lr, mu = 0.05, 0.9
    base = W.make_inputs(k, n, seed=21)

    def run(peer, beta):
        x, v = base.x.copy(), base.v.copy()
        oracle.step_gossip(x, v, base.g, lr, mu, beta, peer)
        return x, v

    ident = list(range(k))
    x_id, v_id = run(ident, 0.5)
    x_b0, v_b0 = run([3, 0, 1, 2, 7, 4, 5, 6], 0.0)
    # identity permutation and beta = 0 are both "no mixing": bitwise the local step
    assert np.array_equal(x_id, x_b0) and np.array_equal(v_id, v_b0)
    vn = (np.float32(mu) * base.v)
    assert np.allclose(x_id, base.x + (vn - np.float32(lr) * base.g), rtol=1e-6, atol=1e-6)
    # the momentum buffer is never mixed
    peer = [int(t) for t in oracle.make_perm(SEED, 3, k)]
    x_p, v_p = run(peer, 0.5)
    assert np.array_equal(v_p, v_id)
    # doubly stochastic mix keeps every column's sum (the replica mean)
    assert np.allclose(x_p.astype(np.float64).sum(0), x_id.astype(np.float64).sum(0), rtol=0, atol=1e-5)
    # an involution with beta = 1/2 leaves partners at their common midpoint
    # (each side rounds a - (a-b)/2 on its own, so equal up to the last place)
    inv = [1, 0, 3, 2, 5, 4, 7, 6]
    x_i, _ = run(inv, 0.5)
    for a, b in ((0, 1), (2, 3), (4, 5), (6, 7)):
        mid = 0.5 * (x_id[a].astype(np.float64) + x_id[b].astype(np.float64))
        assert np.allclose(x_i[a], mid, rtol=2e-7, atol=1e-7) and np.allclose(x_i[b], mid, rtol=2e-7, atol=1e-7)
    # row i of the result depends only on rows i and peer[i] of the local step
    for i in range(k):
        want = x_id[i] - np.float32(0.5) * (x_id[i] - x_id[peer[i]])
        assert np.allclose(x_p[i], want, rtol=1e-6, atol=1e-7)
    with pytest.raises(ValueError):
        oracle.step_gossip(base.x.copy(), base.v.copy(), base.g, lr, mu, 0.5, [0, 1, 2, 3, 4, 5, 6, 8])


def _heavy_ball_closed_form(e0, h, lr, mu, steps):
    """Textbook heavy ball on a 1-D quadratic, as the three-term recurrence
    e_{t+1} = (1 + mu - lr h) e_t - mu e_{t-1}, with e_{-1} chosen for v_0 = 0."""
    prev, cur = e0.copy(), e0.copy()      # v_0 = 0  <=>  e_{-1} = e_0
    for _ in range(steps):
        prev, cur = cur, (1.0 + mu - lr * h) * cur - mu * prev
    return cur


def test_local_step_is_heavy_ball(oracle):
    n, steps = 512, 60
    lr, mu = 0.05, 0.9
    inp = W.make_inputs(1, n, seed=30)
    x = inp.x.copy()
    v = np.zeros_like(x)
    g = np.zeros_like(x)
    for t in range(steps):
        oracle.gen_grad(x, inp.h, inp.xstar, g, 0.0, SEED, t)
        oracle.step_gossip(x, v, g, lr, mu, 0.5, [0])
    e0 = inp.x[0].astype(np.float64) - inp.xstar.astype(np.float64)
    want = _heavy_ball_closed_form(e0, inp.h.astype(np.float64), float(np.float32(lr)), float(np.float32(mu)), steps)
    got = x[0].astype(np.float64) - inp.xstar.astype(np.float64)
    assert np.allclose(got, want, rtol=0, atol=2e-5)
    assert np.abs(want).max() > 0.05        # not yet converged: the comparison has teeth


# ----------------------------------------------------------------------------
# all-reduce

def test_allreduce_exact_replay(oracle):
    k, n = 3, 7
    lr, mu = np.float32(0.05), np.float32(0.9)
    inp = W.make_inputs(k, n, seed=40)
    x0, v0, g0 = inp.x.copy(), inp.v.copy(), inp.g.copy()
    oracle.step_allreduce(inp.x, inp.v, inp.g, lr, mu)
    for j in range(n):
        u = [brute.f32_fma(-F(lr), F(g0[i, j]), brute.f32_mul(F(mu), F(v0[i, j]))) for i in range(k)]
        mean = sum(u) / k
        ubar = brute.nearest_f32(mean)
        # the oracle sums in fp64; the correctly rounded mean may differ from it by at
        # most one unit in the last place in rare double-rounding cases
        for i in range(k):
            assert abs(F(inp.v[i, j]) - ubar) <= abs(ubar) * Fraction(1, 1 << 23)
            assert F(inp.x[i, j]) == brute.f32_add(F(x0[i, j]), F(inp.v[i, j]))
        assert len({float(inp.v[i, j]) for i in range(k)}) == 1


def test_allreduce_invariants_and_noise_free_closed_form(oracle):
    k, n, steps = 8, 300, 50
    lr, mu = 0.05, 0.9
    inp = W.make_inputs(k, n, seed=41, identical_rows=True)
    x = inp.x.copy()
    v = np.zeros_like(x)
    g = np.zeros_like(x)
    for t in range(steps):
        oracle.gen_grad(x, inp.h, inp.xstar, g, 0.1, SEED, t, oracle.NOISE_UNIFORM)
        assert np.abs(g - g[0]).max() > 0           # the noise differs per replica ...
        oracle.step_allreduce(x, v, g, lr, mu)
        assert all(np.array_equal(x[0], x[i]) and np.array_equal(v[0], v[i]) for i in range(1, k))  # ... the rows do not
    # rows that start apart keep their differences
    inp2 = W.make_inputs(k, n, seed=42)
    x2, v2 = inp2.x.copy(), inp2.v.copy()
    d_before = x2.astype(np.float64) - x2[0].astype(np.float64)
    oracle.step_allreduce(x2, v2, inp2.g, lr, mu)
    d_after = x2.astype(np.float64) - x2[0].astype(np.float64)
    assert np.allclose(d_before, d_after, rtol=0, atol=1e-6)
    # sigma = 0, identical start: k-fold replicated heavy ball
    x3 = inp.x.copy()
    v3 = np.zeros_like(x3)
    for t in range(steps):
        oracle.gen_grad(x3, inp.h, inp.xstar, g, 0.0, SEED, t)
        oracle.step_allreduce(x3, v3, g, lr, mu)
    e0 = inp.x[0].astype(np.float64) - inp.xstar.astype(np.float64)
    want = _heavy_ball_closed_form(e0, inp.h.astype(np.float64), float(np.float32(lr)), float(np.float32(mu)), steps)
    assert np.allclose(x3[3].astype(np.float64) - inp.xstar, want, rtol=0, atol=2e-5)


def test_gossip_mean_follows_allreduce_trajectory(oracle):
    """The gradient is affine in x and a permutation mix is doubly stochastic,
    so the replica mean under gossip obeys the all-reduce recursion started at
    the mean, driven by the same per-replica noise."""
    k, n, steps = 8, 400, 40
    lr, mu, sigma = 0.05, 0.9, 0.1
    inp = W.make_inputs(k, n, seed=50)
    xg, vg = inp.x.copy(), np.zeros_like(inp.x)
    mean0 = inp.x.astype(np.float64).mean(0).astype(np.float32)
    xa = np.tile(mean0, (k, 1))
    va = np.zeros_like(xa)
    g = np.zeros_like(xg)
    for t in range(steps):
        oracle.gen_grad(xg, inp.h, inp.xstar, g, sigma, SEED, t)
        oracle.step_gossip(xg, vg, g, lr, mu, 0.5, oracle.make_perm(SEED, t, k))
        oracle.gen_grad(xa, inp.h, inp.xstar, g, sigma, SEED, t)
        oracle.step_allreduce(xa, va, g, lr, mu)
    assert np.allclose(xg.astype(np.float64).mean(0), xa[0], rtol=0, atol=2e-5)
    assert np.abs(xg - xg[0]).max() > 1e-3       # the replicas themselves still differ


# ----------------------------------------------------------------------------
# elastic averaging

@pytest.mark.parametrize("k", [2, 3, 4])
def test_easgd_exact_on_dyadic_inputs(oracle, k):
    rng = np.random.default_rng(60 + k)
    n = 6
    x = _dyadic(rng, (k, n))
    c = _dyadic(rng, (n,))
    v = np.zeros((k, n), np.float32)
    g = _dyadic(rng, (k, n))
    alpha = 0.125
    x0, c0 = x.copy(), c.copy()
    oracle.step_easgd(x, v, g, c, 0.0, 0.0, alpha)      # lr = 0: the exchange alone, all exact
    for j in range(n):
        e = [Fraction(alpha) * (F(x0[i, j]) - F(c0[j])) for i in range(k)]
        for i in range(k):
            assert F(x[i, j]) == F(x0[i, j]) - e[i]
        assert F(c[j]) == F(c0[j]) + sum(e)


def test_easgd_exact_replay_and_invariants(oracle):
    k, n = 4, 11
    lr, mu, alpha = np.float32(0.05), np.float32(0.9), np.float32(0.9 / 4)
    inp = W.make_inputs(k, n, seed=70)
    x0, v0, c0 = inp.x.copy(), inp.v.copy(), inp.center.copy()
    oracle.step_easgd(inp.x, inp.v, inp.g, inp.center, lr, mu, alpha)
    for j in range(n):
        tot = Fraction(0)
        xps = []
        for i in range(k):
            vn = brute.f32_fma(-F(lr), F(inp.g[i, j]), brute.f32_mul(F(mu), F(v0[i, j])))
            xp = brute.f32_add(F(x0[i, j]), vn)
            e = brute.f32_mul(F(alpha), brute.f32_sub(xp, F(c0[j])))
            assert F(inp.v[i, j]) == vn
            assert F(inp.x[i, j]) == brute.f32_sub(xp, e)
            tot += e
            xps.append(xp)
        # fp64 accumulation of k fp32 terms is exact here, so the centre is the
        # correctly rounded sum
        assert F(inp.center[j]) == brute.nearest_f32(F(c0[j]) + tot)
        # closed form of the synchronous round: c <- (1 - k a) c + k a mean(x')
        closed = (1 - k * F(alpha)) * F(c0[j]) + k * F(alpha) * (sum(xps) / k)
        assert abs(float(F(inp.center[j]) - closed)) < 1e-6
        # conservation: sum_i x_i + c is what it was after the local step
        assert abs(float(sum(F(inp.x[i, j]) for i in range(k)) + F(inp.center[j]) - sum(xps) - F(c0[j]))) < 2e-6
    # alpha_e = 0: k independent local steps, centre untouched
    inp2 = W.make_inputs(k, n, seed=71)
    xa, va, ca = inp2.x.copy(), inp2.v.copy(), inp2.center.copy()
    xb, vb = inp2.x.copy(), inp2.v.copy()
    oracle.step_easgd(xa, va, inp2.g, ca, lr, mu, 0.0)
    oracle.step_gossip(xb, vb, inp2.g, lr, mu, 0.0, list(range(k)))
    assert np.array_equal(xa, xb) and np.array_equal(va, vb) and np.array_equal(ca, inp2.center)


# ----------------------------------------------------------------------------
# convergence on the noisy quadratic

def _stationary_var(h, lr, mu, s2):
    """Var(x - x*) of heavy ball driven by gradient noise of variance s2:
    state (e, v), e' = e + v', v' = mu v - lr h e - lr n;  P = A P A^T + Q."""
    A = np.array([[1.0 - lr * h, mu], [-lr * h, mu]])
    Q = lr * lr * s2 * np.ones((2, 2))
    return sla.solve_discrete_lyapunov(A, Q)[0, 0]


@pytest.mark.parametrize("rule", ["allreduce", "gossip"])
def test_converges_to_xstar_with_predicted_noise_floor(oracle, rule):
    k, n, steps = 8, 6000, 320
    lr, mu, sigma = 0.05, 0.9, 0.5
    inp = W.make_inputs(k, n, seed=80, identical_rows=True)
    x, v, g = inp.x.copy(), np.zeros_like(inp.x), np.zeros_like(inp.x)
    d0 = ((x[0].astype(np.float64) - inp.xstar) ** 2).mean()
    for t in range(steps):
        oracle.gen_grad(x, inp.h, inp.xstar, g, sigma, SEED, t)
        if rule == "allreduce":
            oracle.step_allreduce(x, v, g, lr, mu)
        else:
            oracle.step_gossip(x, v, g, lr, mu, 0.5, oracle.make_perm(SEED, t, k))
    xbar = x.astype(np.float64).mean(0)
    got = ((xbar - inp.xstar) ** 2).mean()
    hs = np.linspace(0.1, 1.0, 91)
    want = np.mean([_stationary_var(h, lr, mu, sigma ** 2 / k) for h in hs])
    assert 0.85 * want < got < 1.15 * want
    assert got < 0.05 * d0


def test_sync_pull_gossip_bound_holds(oracle):
    """Theorem (synchronous pull-gossip, Section 6.1.1), mu = 0, iid uniform
    targets: E||theta_t - theta* 1||^2 <= (1 - 2 a mL/(m+L))^t ||theta_0 - theta* 1||^2
    + p a sigma^2 (m+L)/(2mL), with sigma^2 the noise variance summed over the
    coordinates."""
    k, n = 8, 2000
    lr, sigma = 0.5, 0.2
    m_, L_ = 0.1, 1.0
    assert lr <= 2.0 / (m_ + L_)
    inp = W.make_inputs(k, n, seed=90, identical_rows=True)
    x, v, g = inp.x.copy(), np.zeros_like(inp.x), np.zeros_like(inp.x)
    rng = np.random.default_rng(91)
    d0 = float(((x.astype(np.float64) - inp.xstar) ** 2).sum())
    rate = 1.0 - 2.0 * lr * m_ * L_ / (m_ + L_)
    floor = k * lr * (sigma ** 2 * n) * (m_ + L_) / (2 * m_ * L_)
    for t in range(1, 61):
        oracle.gen_grad(x, inp.h, inp.xstar, g, sigma, SEED, t)
        oracle.step_gossip(x, v, g, lr, 0.0, 0.5, rng.integers(0, k, k))
        dist = oracle.stats(x, inp.xstar)[1]
        assert dist <= 1.05 * (rate ** t * d0 + floor)
    assert dist < 0.01 * d0


def test_consensus_distance_plateau_from_both_sides(oracle):
    k, n, steps = 8, 3000, 150
    lr, mu, sigma = 0.05, 0.9, 0.1
    inp = W.make_inputs(k, n, seed=95)
    out = {}
    for mode in (0, 1):
        x, v, c = np.zeros_like(inp.x), np.ones_like(inp.x), np.zeros(n, np.float32)
        oracle.init_replicas(x, v, c, inp.x0, SEED, mode)
        assert not v.any()
        hist = []
        g = np.zeros_like(x)
        for t in range(steps):
            oracle.gen_grad(x, inp.h, inp.xstar, g, sigma, SEED, t)
            oracle.step_gossip(x, v, g, lr, mu, 0.5, oracle.make_perm(SEED, t, k))
            hist.append(oracle.stats(x, inp.xstar)[0])
        out[mode] = hist
    assert out[0][0] > 0 and out[0][-1] > 3 * out[0][0]           # identical start: rises to the floor
    assert out[1][-1] < 1e-2 * out[1][0]                          # spread start: shrinks by orders of magnitude
    assert 0.6 < out[0][-1] / out[1][-1] < 1.6                    # same plateau


# ----------------------------------------------------------------------------
# init, segments, statistics

def test_init_replicas(oracle):
    k, n = 5, 1000
    inp = W.make_inputs(k, n, seed=96)
    x, v, c = np.zeros_like(inp.x), np.ones_like(inp.x), np.zeros(n, np.float32)
    oracle.init_replicas(x, v, c, inp.x0, SEED, 0)
    assert all(np.array_equal(x[i], inp.x0) for i in range(k)) and np.array_equal(c, inp.x0) and not v.any()
    oracle.init_replicas(x, v, c, None, SEED, 1)
    assert abs(x.mean()) < 0.06 and abs(x.var() - 1) < 0.06
    assert abs(np.corrcoef(x[0], x[1])[0, 1]) < 0.1
    assert np.allclose(c, x.astype(np.float64).mean(0), rtol=0, atol=1e-7)
    xs = np.zeros((k, 64), np.float32)
    oracle.init_replicas(xs, np.zeros_like(xs), None, None, SEED, 1, col0=130)
    assert np.array_equal(xs, x[:, 130:194])
    with pytest.raises(ValueError):
        oracle.init_replicas(x, v, c, None, SEED, 0)


def test_expand_lr_matches_searchsorted(oracle):
    d = 5000
    off, sc = W.random_segments(d, 37, seed=3)
    lr = np.float32(0.05)
    got = oracle.expand_lr(lr, d, off, sc)
    seg = np.searchsorted(off, np.arange(d), side="right") - 1
    assert np.array_equal(got, lr * sc[seg])
    assert np.array_equal(oracle.expand_lr(lr, 300, off, sc, col0=1234), got[1234:1534])
    assert np.array_equal(oracle.expand_lr(lr, d), np.full(d, lr, np.float32))
    with pytest.raises(ValueError):
        oracle.expand_lr(lr, d + 1, off, sc)


def test_segmented_step_equals_flat_when_scales_are_one(oracle):
    k, d = 4, 999
    off, sc = W.random_segments(d, 20, seed=4)
    inp = W.make_inputs(k, d, seed=97)
    peer = oracle.make_perm(SEED, 0, k)
    xa, va = inp.x.copy(), inp.v.copy()
    xb, vb = inp.x.copy(), inp.v.copy()
    oracle.step_gossip(xa, va, inp.g, 0.05, 0.9, 0.5, peer)
    oracle.step_gossip(xb, vb, inp.g, oracle.expand_lr(0.05, d, off, np.ones_like(sc)), 0.9, 0.5, peer)
    assert np.array_equal(xa, xb) and np.array_equal(va, vb)
    # and with real scales, a segment's columns move exactly as a flat run at that step size would
    xc, vc = inp.x.copy(), inp.v.copy()
    oracle.step_gossip(xc, vc, inp.g, oracle.expand_lr(0.05, d, off, sc), 0.9, 0.5, peer)
    for s in (0, 7, 19):
        lo, hi = int(off[s]), int(off[s + 1])
        xd, vd = inp.x.copy(), inp.v.copy()
        oracle.step_gossip(xd, vd, inp.g, np.float32(0.05) * sc[s], 0.9, 0.5, peer)
        assert np.array_equal(xc[:, lo:hi], xd[:, lo:hi]) and np.array_equal(vc[:, lo:hi], vd[:, lo:hi])


def test_stats_against_numpy(oracle):
    k, n = 6, 777
    inp = W.make_inputs(k, n, ld=800, seed=98)
    got = oracle.stats(inp.x, inp.xstar, n=n)
    x = inp.x[:, :n].astype(np.float64)
    xs = inp.xstar[:n].astype(np.float64)
    xbar = x.mean(0)
    want = [((x - xbar) ** 2).sum(), ((x - xs) ** 2).sum(), ((xbar - xs) ** 2).sum(), (xbar ** 2).sum()]
    assert np.allclose(got, want, rtol=1e-12)
    # decomposition: sum_i |x_i - x*|^2 = consensus + k |xbar - x*|^2
    assert got[1] == pytest.approx(got[0] + k * got[2], rel=1e-12)


def test_strided_rows_leave_padding_untouched(oracle):
    k, d, ld = 3, 50, 64
    inp = W.make_inputs(k, d, ld=ld, seed=99)
    x, v = inp.x.copy(), inp.v.copy()
    oracle.step_gossip(x, v, inp.g, 0.05, 0.9, 0.5, [1, 2, 0], n=d)
    assert (x[:, d:] == 777.0).all() and (v[:, d:] == 777.0).all()
    xt, vt = np.ascontiguousarray(inp.x[:, :d]), np.ascontiguousarray(inp.v[:, :d])
    oracle.step_gossip(xt, vt, np.ascontiguousarray(inp.g[:, :d]), 0.05, 0.9, 0.5, [1, 2, 0])
    assert np.array_equal(x[:, :d], xt) and np.array_equal(v[:, :d], vt)

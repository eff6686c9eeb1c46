"""Pins for gossip with targets that are not a permutation: iid pull targets
(Algorithm 3 / Section 3.1), push-gossip with a variable number of received
messages (Algorithm 4), the target generator, and the host-side visiting order
the pull kernel uses for such maps.  CPU only.

Tied to: big-integer restatement of the generator and chi-square uniformity;
exact rationals on dyadic inputs over *all* k^k maps for small k; the second
moment E[M^T M] = (I + 11^T/k)/2 that the synchronous pull-gossip analysis
(Section 6.1.1) derives for iid targets; special maps whose result is known in
closed form (everyone to one node = that node gets the global mean, a
derangement = pairwise averaging); a Python replay of the walk machine against
the plain definition.
"""
from fractions import Fraction
from itertools import product

import numpy as np
import pytest

import brute
from paper_1611_04581_amd import gsgd
from paper_1611_04581_amd import workloads as W

SEED = 0x161104581
F = lambda a: Fraction(float(a))


# ----------------------------------------------------------------------------
# target generator

def _targets_bigint(seed, step, k, exclude_self):
    key = (seed & 0xFFFFFFFF, seed >> 32)
    out = []
    for i in range(k):
        r = brute.philox4((i, 1, step, 5), key)[0]
        if exclude_self:
            j = (r * (k - 1)) >> 32
            out.append(j + 1 if j >= i else j)
        else:
            out.append((r * k) >> 32)
    return out


@pytest.mark.parametrize("exclude_self", [False, True])
def test_targets_match_restatement_and_library(oracle, exclude_self):
    for k in (2, 3, 8, 32, 128, 512):
        for step in (0, 1, 199, 2**32 - 1):
            want = _targets_bigint(SEED, step, k, exclude_self)
            assert list(oracle.make_targets(SEED, step, k, exclude_self)) == want
            assert list(gsgd.make_targets(SEED, step, k, exclude_self)) == want
    assert list(oracle.make_targets(SEED, 0, 1, False)) == [0]
    with pytest.raises(ValueError):
        oracle.make_targets(SEED, 0, 1, True)
    with pytest.raises(gsgd.GsgdError):
        gsgd.make_targets(SEED, 0, 1, True)


def test_targets_are_uniform_and_independent(oracle):
    k, steps = 8, 40000
    t = np.stack([oracle.make_targets(SEED, s, k, False) for s in range(steps)])
    assert t.min() == 0 and t.max() == k - 1
    for i in range(k):                                   # each node: uniform over all k nodes, itself included
        cnt = np.bincount(t[:, i], minlength=k)
        chi2 = ((cnt - steps / k) ** 2 / (steps / k)).sum()
        assert chi2 < 30.0, (i, chi2)                    # 7 dof: 30 is beyond the 1e-4 tail
    joint = np.bincount(t[:, 0] * k + t[:, 1], minlength=k * k)
    chi2 = ((joint - steps / k**2) ** 2 / (steps / k**2)).sum()
    assert chi2 < 120.0                                  # 63 dof
    te = np.stack([oracle.make_targets(SEED, s, k, True) for s in range(steps)])
    for i in range(k):                                   # never itself, uniform over the others
        cnt = np.bincount(te[:, i], minlength=k)
        assert cnt[i] == 0
        others = np.delete(cnt, i)
        chi2 = ((others - steps / (k - 1)) ** 2 / (steps / (k - 1))).sum()
        assert chi2 < 28.0, (i, chi2)


# ----------------------------------------------------------------------------
# pull-gossip on arbitrary maps

def _dyadic(k, n, seed):
    rng = np.random.default_rng(seed)
    return (rng.integers(-64, 64, size=(k, n)) / 8.0).astype(np.float32)


@pytest.mark.parametrize("k", [2, 3, 4])
def test_pull_mix_brute_force_over_all_maps(oracle, k):
    """lr = 0, mu = 0: the step is the mix alone; on dyadic inputs with
    beta = 1/2 or 1/4 every value is exact."""
    n = 5
    x0 = _dyadic(k, n, 7)
    zeros = np.zeros_like(x0)
    for beta in (0.5, 0.25):
        for peer in product(range(k), repeat=k):
            x, v = x0.copy(), zeros.copy()
            oracle.step_gossip(x, v, zeros, 0.0, 0.0, beta, list(peer))
            want = brute.gossip_mix_exact([[F(a) for a in row] for row in x0], list(peer), beta)
            for i in range(k):
                for j in range(n):
                    assert F(x[i, j]) == want[i][j], (peer, i, j)


@pytest.mark.parametrize("k", [2, 3, 4])
def test_second_moment_of_the_iid_pull_matrix(oracle, k):
    """Section 6.1.1: with M_I = (1/2) sum_i e_i (e_i + e_{j_i})^T and iid
    uniform j_i, E[M_I^T M_I] = (I + 11^T/k)/2.  Averaged over all k^k maps the
    oracle's mix must reproduce it exactly: y^T E[M^T M] y = E ||M y||^2."""
    n = 3
    y = _dyadic(k, n, 11)
    zeros = np.zeros_like(y)
    total = Fraction(0)
    for peer in product(range(k), repeat=k):
        x, v = y.copy(), zeros.copy()
        oracle.step_gossip(x, v, zeros, 0.0, 0.0, 0.5, list(peer))
        total += sum(F(a) ** 2 for a in x.ravel())
    mean_sq = total / k**k
    yy = [[F(a) for a in row] for row in y]
    norm2 = sum(a * a for row in yy for a in row)
    colsum2 = sum(sum(yy[i][j] for i in range(k)) ** 2 for j in range(n))
    assert mean_sq == (norm2 + colsum2 / k) / 2


def test_pull_map_special_cases(oracle):
    k, n = 6, 40
    inp = W.make_inputs(k, n, seed=3)
    # everyone pulls from node 2: node 2 keeps x', the others move halfway to it
    peer = [2] * k
    x, v = inp.x.copy(), inp.v.copy()
    oracle.step_gossip(x, v, inp.g, 0.05, 0.9, 0.5, peer)
    xl, vl = inp.x.copy(), inp.v.copy()
    oracle.step_gossip(xl, vl, inp.g, 0.05, 0.9, 0.5, list(range(k)))      # local step only
    assert np.array_equal(x[2], xl[2])
    for i in (0, 1, 3, 4, 5):
        assert np.allclose(x[i], 0.5 * (xl[i].astype(np.float64) + xl[2]), rtol=0, atol=1e-6)
    assert np.array_equal(v, vl)


# ----------------------------------------------------------------------------
# push-gossip

def _push_exact(xp, target):
    k = len(xp)
    out = []
    for r in range(k):
        got = [xp[r]] + [xp[i] for i in range(k) if i != r and target[i] == r]
        out.append([sum(col) / len(got) for col in zip(*got)])
    return out


@pytest.mark.parametrize("k", [2, 3, 4])
def test_push_brute_force_over_all_maps(oracle, k):
    """lr = 0, mu = 0: the step is the averaging alone.  Exact rationals say
    what the average is; the oracle's fp64 sum of dyadic values is exact, so
    its result is the correctly rounded quotient."""
    n = 4
    x0 = _dyadic(k, n, 13)
    zeros = np.zeros_like(x0)
    for target in product(range(k), repeat=k):
        x, v = x0.copy(), zeros.copy()
        oracle.step_gossip_push(x, v, zeros, 0.0, 0.0, list(target))
        want = _push_exact([[F(a) for a in row] for row in x0], list(target))
        for r in range(k):
            for j in range(n):
                assert F(x[r, j]) == brute.nearest_f32(want[r][j]), (target, r, j)


def test_push_special_cases(oracle):
    k, n = 6, 50
    inp = W.make_inputs(k, n, seed=5)
    xl, vl = inp.x.copy(), inp.v.copy()
    oracle.step_gossip(xl, vl, inp.g, 0.05, 0.9, 0.5, list(range(k)))      # x' of every node
    xl64 = xl.astype(np.float64)
    # everyone pushes to node 0: node 0 ends at the global mean of x', the others keep their own x'
    x, v = inp.x.copy(), inp.v.copy()
    oracle.step_gossip_push(x, v, inp.g, 0.05, 0.9, [0] * k)
    assert np.array_equal(x[0], xl64.mean(0).astype(np.float32))
    assert np.array_equal(x[1:], xl[1:]) and np.array_equal(v, vl)
    # own target: nothing is sent, nothing changes
    x, v = inp.x.copy(), inp.v.copy()
    oracle.step_gossip_push(x, v, inp.g, 0.05, 0.9, list(range(k)))
    assert np.array_equal(x, xl)
    # a derangement: everyone receives exactly one message, so push = pairwise averaging with the sender,
    # which is pull-gossip at beta = 1/2 on the inverse map (up to the last place: different rounding points)
    target = [1, 2, 3, 4, 5, 0]
    inverse = [5, 0, 1, 2, 3, 4]
    x, v = inp.x.copy(), inp.v.copy()
    oracle.step_gossip_push(x, v, inp.g, 0.05, 0.9, target)
    xq, vq = inp.x.copy(), inp.v.copy()
    oracle.step_gossip(xq, vq, inp.g, 0.05, 0.9, 0.5, inverse)
    assert np.allclose(x, xq, rtol=0, atol=2.5e-7)
    assert np.allclose(x.astype(np.float64).sum(0), xl64.sum(0), rtol=0, atol=1e-5)   # column sums kept
    # weight decay / Nesterov go through the same local step as the other rules
    x, v = inp.x.copy(), inp.v.copy()
    oracle.step_gossip_push(x, v, inp.g, 0.05, 0.9, list(range(k)), wd=1e-3, nesterov=True)
    xe, ve = inp.x.copy(), inp.v.copy()
    oracle.step_gossip_ext(xe, ve, inp.g, 0.05, 0.9, 0.5, list(range(k)), wd=1e-3, nesterov=True)
    assert np.array_equal(x, xe) and np.array_equal(v, ve)


def test_push_gossip_contracts_towards_consensus(oracle):
    """Pure push rounds (no gradient) on uniformly drawn targets shrink the
    consensus distance geometrically, as the simplified push-sum step the paper
    describes should (Section 3.1)."""
    k, n = 16, 2000
    inp = W.make_inputs(k, n, seed=8)
    x, v, zeros = inp.x.copy(), np.zeros_like(inp.x), np.zeros_like(inp.x)
    c0 = oracle.stats(x, inp.xstar)[0]
    for t in range(12):
        oracle.step_gossip_push(x, v, zeros, 0.0, 0.0, oracle.make_targets(SEED, t, k, True))
    c1 = oracle.stats(x, inp.xstar)[0]
    assert c1 < c0 * 1e-2


# ----------------------------------------------------------------------------
# the pull kernel's visiting order, replayed

def _replay_pull_walk(walk, post, key, beta):
    """Runs the kernel's register machine on Python floats.  post[i] = x'_i,
    key[i] = what replica i contributes to whoever pulls from it."""
    k = len(post)
    out = [None] * k
    stack = [None] * gsgd.WALK_SLOTS
    first_key = prev_key = prev_post = prev_row = par = None
    for wd in walk:
        wd = int(wd)
        row = wd & gsgd.WALK_ROW_MASK
        slot = (wd >> gsgd.WALK_SLOT_SHIFT) & 0xF
        if wd & gsgd.WALK_TREE:
            restore = (wd >> gsgd.WALK_RESTORE_SHIFT) & 3
            if restore == 1:
                par = prev_key
            elif restore == 2:
                par = stack[slot]
                assert par is not None
            assert par is not None
            assert out[row] is None
            out[row] = post[row] - beta * (key[row] - par)
            if wd & gsgd.WALK_SAVE:
                stack[slot] = par
            if wd & gsgd.WALK_DESCEND:
                par = key[row]
        else:
            if wd & gsgd.WALK_FIRST:
                first_key = key[row]
            else:
                out[prev_row] = prev_post - beta * (prev_key - key[row])
            if wd & gsgd.WALK_LAST:
                out[row] = post[row] - beta * (key[row] - first_key)
            prev_key, prev_post, prev_row = key[row], post[row], row
    return out


def _maps_for(k, rng):
    maps = [[0] * k, [max(i - 1, 0) for i in range(k)], [(i + 1) % k for i in range(k)], list(range(k)),
            [i // 2 for i in range(k)], [(i - 1) // 3 if i else 0 for i in range(k)]]
    maps += [list(rng.integers(0, k, size=k)) for _ in range(12)]
    return maps


@pytest.mark.parametrize("k", [1, 2, 5, 32, 33, 128, 512])
def test_pull_walk_realises_the_definition(k):
    rng = np.random.default_rng(k)
    post = list(rng.standard_normal(k))
    old = list(rng.standard_normal(k))
    worst = 0
    for peer in _maps_for(k, rng):
        peer = [int(p) for p in peer]
        walk, slots = gsgd.pull_walk(peer)
        worst = max(worst, slots)
        assert 0 <= slots <= gsgd.WALK_SLOTS
        assert sorted(int(w) & gsgd.WALK_ROW_MASK for w in walk) == list(range(k))
        for key in (post, old):                                    # fresh and stale parameters
            got = _replay_pull_walk(walk, post, key, 0.5)
            for i in range(k):
                assert got[i] == post[i] - 0.5 * (key[i] - key[peer[i]]), (peer, i)
    if k == 512:
        # a 512-long chain needs no slot at all; a complete binary tree needs about log2(k)
        assert gsgd.pull_walk([max(i - 1, 0) for i in range(k)])[1] == 0
        assert 1 <= gsgd.pull_walk([(i - 1) // 2 if i else 0 for i in range(k)])[1] <= 8


def test_pull_walk_of_a_permutation_is_the_cycle_walk():
    rng = np.random.default_rng(1)
    for k in (1, 7, 32, 512):
        perm = [int(p) for p in rng.permutation(k)]
        walk, slots = gsgd.pull_walk(perm)
        assert slots == 0
        assert [int(w) for w in walk] == [int(w) for w in gsgd.perm_walk(perm)]
    with pytest.raises(gsgd.GsgdError) as e:
        gsgd.pull_walk([0, 3, 1])
    assert e.value.code == gsgd.ERR_BAD_PERM


# ----------------------------------------------------------------------------
# the push kernel's visiting order, replayed

def _replay_push_walk(walk, post):
    """Runs the push kernel's register machine on exact rationals."""
    k = len(post)
    out = [None] * k
    stack = [None] * gsgd.WALK_SLOTS
    acc = first_sum = first_count = first_row = prev = None
    for wd in walk:
        wd = int(wd)
        row = wd & gsgd.WALK_ROW_MASK
        count = wd >> gsgd.PUSH_COUNT_SHIFT
        slot = (wd >> gsgd.PUSH_SLOT_SHIFT) & 7
        total = post[row]
        if wd & gsgd.PUSH_HAS_SENDERS:
            assert acc is not None
            total = acc + post[row]
        assert out[row] is None
        if wd & gsgd.WALK_TREE:
            out[row] = total / count
            mode = (wd >> gsgd.PUSH_MODE_SHIFT) & 3
            assert mode in (1, 2, 3)
            if mode == 1:
                acc = post[row]
            elif mode == 2:
                acc = acc + post[row]
            else:
                acc = stack[slot] + post[row]
            if wd & gsgd.PUSH_SAVE_AFTER:
                stack[slot] = acc
        elif wd & gsgd.WALK_FIRST:
            if wd & gsgd.WALK_LAST:
                out[row] = total / count
            else:
                first_sum, first_count, first_row = total, count, row
            prev = post[row]
        else:
            out[row] = (total + prev) / count
            if wd & gsgd.WALK_LAST:
                out[first_row] = (first_sum + post[row]) / first_count
            prev = post[row]
    return out


@pytest.mark.parametrize("k", [1, 2, 5, 32, 33, 128, 512])
def test_push_walk_realises_the_definition(k):
    rng = np.random.default_rng(1000 + k)
    post = [Fraction(int(a), 16) for a in rng.integers(-1000, 1000, size=k)]
    for target in _maps_for(k, rng):
        target = [int(p) for p in target]
        walk, slots = gsgd.push_walk(target)
        assert 0 <= slots <= gsgd.WALK_SLOTS
        assert sorted(int(w) & gsgd.WALK_ROW_MASK for w in walk) == list(range(k))
        got = _replay_push_walk(walk, post)
        want = _push_exact([[p] for p in post], target)
        for r in range(k):
            assert got[r] == want[r][0], (target, r)
    if k == 512:
        assert gsgd.push_walk([max(i - 1, 0) for i in range(k)])[1] == 0
        assert 1 <= gsgd.push_walk([(i - 1) // 2 if i else 0 for i in range(k)])[1] <= 8
    with pytest.raises(gsgd.GsgdError):
        gsgd.push_walk([k] * k)


# ----------------------------------------------------------------------------
# diffusion potential (Section 3.1)

def test_diffusion_potential_special_cases(oracle):
    rng = np.random.default_rng(3)
    p, n = 6, 40
    theta = rng.standard_normal((p, n))
    # before any round V = I: each node holds only its own vector
    assert np.isclose(oracle.diffusion_potential(theta, np.eye(p)), (1 - 1 / p) * (theta ** 2).sum(), rtol=1e-12)
    # identical starting vectors: Phi = ||theta||^2 sum_ij (v_ij - 1/p)^2, zero once every weight is 1/p
    same = np.tile(theta[0], (p, 1))
    V = rng.dirichlet(np.ones(p), size=p)
    assert np.isclose(oracle.diffusion_potential(same, V), (theta[0] ** 2).sum() * ((V - 1 / p) ** 2).sum(), rtol=1e-12)
    assert abs(oracle.diffusion_potential(same, np.full((p, p), 1 / p))) < 1e-20


def test_mixing_matrices_are_the_brute_forced_step_rules(oracle):
    """Pin of oracle.mixing_matrix_pull / mixing_matrix_push: with no gradient
    step (lr = 0, mu = 0, v = 0) a gossip round is theta' = M theta, so for
    every one of the k^k maps (k <= 3) M @ theta0 on dyadic theta0 must equal,
    exactly, what oracle.step_gossip / step_gossip_push return -- and those two
    are themselves pinned by exact-rational brute force over all maps above.
    A transposed M, a self-target counted twice or a wrong weight fails here.
    Dyadic inputs keep every product with 1/2 exact in fp32 and fp64; thirds
    (push with two senders) are compared through the correctly rounded
    quotient of the exact rational."""
    rng = np.random.default_rng(11)
    for k in (1, 2, 3):
        n = 5
        theta0 = (rng.integers(-64, 64, size=(k, n)) / 8.0).astype(np.float32)
        zeros = np.zeros((k, n), np.float32)
        for m in product(range(k), repeat=k):
            # pull: row i <- (1 - beta) theta_i + beta theta_m[i]
            for beta in (0.5, 0.25, 1.0, 0.0):
                x = theta0.copy()
                oracle.step_gossip(x, zeros.copy(), zeros.copy(), 0.0, 0.0, beta, list(m))
                M = oracle.mixing_matrix_pull(list(m), beta)
                assert np.array_equal(M @ theta0.astype(np.float64), x.astype(np.float64)), (m, beta)
                assert np.allclose(M.sum(1), 1.0, rtol=0, atol=0)
            # push: row r <- average of theta_r and every theta_i (i != r) with m[i] == r
            x = theta0.copy()
            oracle.step_gossip_push(x, zeros.copy(), zeros.copy(), 0.0, 0.0, list(m))
            M = oracle.mixing_matrix_push(list(m))
            for r in range(k):
                got = [r] + [i for i in range(k) if i != r and m[i] == r]
                for j in range(n):
                    exact = sum(Fraction(float(theta0[i, j])) for i in got) / len(got)
                    assert Fraction(float(x[r, j])) == Fraction(float(np.float32(float(exact)))), (m, r, j)
                    # M's row, applied in exact rationals, is that same average
                    row = sum(Fraction(M[r, i]).limit_denominator(6) * Fraction(float(theta0[i, j])) for i in range(k))
                    assert row == exact, (m, r, j)
            assert np.allclose(M.sum(1), 1.0, rtol=0, atol=1e-15)
    # orientation: in a pull round from the map (1, 1, 0), node 0 takes from node 1 and not the other way round
    M = oracle.mixing_matrix_pull([1, 1, 0], 0.25)
    assert M[0, 1] == 0.25 and M[1, 0] == 0.0 and M[1, 1] == 1.0 and M[2, 0] == 0.25 and M[2, 2] == 0.75
    # push with targets (1, 1, 0): node 1 receives from 0 (its own target is itself), node 0 from 2, node 2 from nobody
    M = oracle.mixing_matrix_push([1, 1, 0])
    assert np.array_equal(M, np.array([[0.5, 0, 0.5], [0.5, 0.5, 0], [0, 0, 1.0]]))


def test_weight_matrices_and_library_potential(oracle):
    """The library's host-side weight updates are the oracle's mixing matrices
    applied from the left, and its closed form of the potential (from row
    norms) equals the term-by-term definition."""
    rng = np.random.default_rng(4)
    for k in (1, 2, 5, 16):
        theta = rng.standard_normal((k, 30))
        V = np.eye(k)
        Vo = np.eye(k)
        for r in range(6):
            if r % 2 == 0:
                peer = [int(a) for a in oracle.make_targets(SEED, r, k)]
                gsgd.weights_pull(V, peer, 0.5)
                Vo = oracle.mixing_matrix_pull(peer, 0.5) @ Vo
            else:
                target = [int(a) for a in rng.integers(0, k, size=k)]
                gsgd.weights_push(V, target)
                Vo = oracle.mixing_matrix_push(target) @ Vo
            assert np.allclose(V, Vo, rtol=0, atol=1e-15)
            assert np.allclose(V.sum(1), 1.0, rtol=0, atol=1e-14)          # rows stay weighted averages
            now = Vo @ theta
            got = gsgd.diffusion_potential(V, (theta ** 2).sum(1), (now ** 2).sum(1))
            assert np.isclose(got, oracle.diffusion_potential(theta, Vo), rtol=1e-10, atol=1e-12)
    with pytest.raises(gsgd.GsgdError):
        gsgd.weights_pull(np.eye(3), [0, 1, 3], 0.5)


def test_diffusion_potential_decays_under_uniform_gossip(oracle):
    """Repeated rounds of uniform gossip shrink the potential at a steady rate
    (the property the paper quotes from the push-sum analysis).  With one
    common starting vector the potential is ||theta||^2 sum_ij (v_ij - 1/p)^2,
    the weight potential of that analysis, and decays geometrically towards
    zero for push-gossip with its near-uniform weights; with distinct starting
    vectors it falls to the spread the contributions keep at consensus."""
    k, n = 16, 50
    theta = np.random.default_rng(5).standard_normal((k, n))
    same = np.tile(theta[0], (k, 1))
    for kind in ("pull", "push"):
        V = np.eye(k)
        phi, phi_same = [oracle.diffusion_potential(theta, V)], [oracle.diffusion_potential(same, V)]
        for r in range(24):
            if kind == "pull":
                V = oracle.mixing_matrix_pull(oracle.make_targets(SEED, r, k), 0.5) @ V
            else:
                V = oracle.mixing_matrix_push(oracle.make_targets(SEED, r, k, True)) @ V
            phi.append(oracle.diffusion_potential(theta, V))
            phi_same.append(oracle.diffusion_potential(same, V))
        assert phi[8] < 0.2 * phi[0] and phi[-1] <= phi[8]
        spread = V.max(0) - V.min(0)                       # near consensus: every node holds almost the same weights
        assert spread.max() < 2e-2
        # the first rounds, before the weights settle, shrink the common-vector potential geometrically
        ratios = np.array(phi_same[1:7]) / np.array(phi_same[:6])
        assert np.exp(np.log(ratios).mean()) < 0.75
        assert phi_same[-1] < 0.05 * phi_same[0]

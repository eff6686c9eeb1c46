"""The predicted consensus floor of gossiping SGD (paper_1611_04581_amd.theory)
against the oracle, on the CPU: a closed form at mu = 0, and seeded runs with
the experiments' local step (Nesterov 0.9, weight decay 1e-4) through a
step-size schedule annealed by 0.1 twice (Section 4.2): after each anneal the
consensus distance settles on a floor about 100 times lower, i.e. it moves
with the step size (the observation of Section 4.3), and the prediction
follows it."""
import numpy as np

from paper_1611_04581_amd import theory, workloads as W

SEED = W.DEFAULT_SEED


def test_floor_closed_form_without_momentum():
    h = np.linspace(0.1, 1.0, 7)
    lr, sigma, k = 0.05, 0.3, 8
    got = theory.gossip_consensus_floor(h, lr, 0.0, sigma, k)
    # mu = 0, beta = 1/2:  a = 1/2 [ (1 - lr h)^2 a + lr^2 sigma^2 (1 - 1/k) ]
    want = 0.5 * lr ** 2 * sigma ** 2 * (1 - 1 / k) / (1 - 0.5 * (1 - lr * h) ** 2)
    assert np.allclose(got, want, rtol=1e-12)
    # Nesterov and heavy ball coincide when there is no momentum
    assert np.allclose(theory.gossip_consensus_floor(h, lr, 0.0, sigma, k, nesterov=True), want, rtol=1e-12)
    # beta = 0: no exchange, the floor is that of k independent runs about their mean
    free = theory.gossip_consensus_floor(h, lr, 0.0, sigma, k, beta=0.0)
    assert np.allclose(free, lr ** 2 * sigma ** 2 * (1 - 1 / k) / (1 - (1 - lr * h) ** 2), rtol=1e-12)


def test_floor_follows_the_oracle_through_annealing(oracle):
    k, d = 8, 12000
    mu, sigma, wd = 0.9, 0.1, 1e-4
    rng = np.random.default_rng(1)
    h = rng.uniform(0.1, 1.0, d).astype(np.float32)
    xs = rng.standard_normal(d).astype(np.float32)
    x = np.tile(rng.standard_normal(d).astype(np.float32), (k, 1)).copy()      # identical start, as in the algorithm boxes
    v, g = np.zeros_like(x), np.zeros_like(x)
    t, floors, preds = 0, [], []
    for lr in (0.1, 0.01, 0.001):
        cons = []
        for s in range(170):
            oracle.gen_grad(x, h, xs, g, sigma, SEED, t, 0)
            oracle.step_gossip_ext(x, v, g, lr, mu, 0.5, oracle.make_perm(SEED, t, k), wd=wd, nesterov=True)
            t += 1
            if s >= 140:
                cons.append(oracle.stats(x, xs)[0])
        floors.append(np.mean(cons))
        preds.append(k * theory.gossip_consensus_floor(h, lr, mu, sigma, k, 0.5, wd, True).sum())
    for f, p in zip(floors, preds):
        assert abs(f / p - 1.0) < 0.1, (floors, preds)
    # the floor moves with the step size: two orders of magnitude per anneal, as predicted
    for a in (0, 1):
        assert 40 < floors[a] / floors[a + 1] < 160
        assert abs((floors[a] / floors[a + 1]) / (preds[a] / preds[a + 1]) - 1.0) < 0.15
    # heavy ball, no weight decay, at one step size
    x = np.tile(xs * 0, (k, 1)).copy()
    v[:] = 0
    cons = []
    for s in range(200):
        oracle.gen_grad(x, h, xs, g, sigma, SEED, t, 1)
        oracle.step_gossip(x, v, g, 0.05, mu, 0.5, oracle.make_perm(SEED, t, k))
        t += 1
        if s >= 150:
            cons.append(oracle.stats(x, xs)[0])
    pred = k * theory.gossip_consensus_floor(h, 0.05, mu, sigma, k).sum()
    assert abs(np.mean(cons) / pred - 1.0) < 0.1

"""What the analysis predicts for runs on the noisy quadratic (numpy, fp64).

Not part of the computing path: these are closed-form expectations a user can
hold a run against (tests and bench.py do).

Stationary consensus distance of gossiping SGD with one uniformly random
permutation of peers per step (the setting of the synchronous analysis,
Section 6.1.1, with momentum added).  Per coordinate with curvature h the
deviation of a node from the node mean, d_i = theta_i - mean, and of its
momentum buffer, w_i, follow the local step linearly,

    heavy ball:  w' = mu w - a (H d + sigma n),  d' = d + w'
    Nesterov  :  w' = mu w - a (H d + sigma n),  d' = d - a (H d + sigma n) + mu w'

with H = h + weight decay, a the step size, n the node's noise minus the mean
noise (variance 1 - 1/p), and the mix d_i <- (1 - beta) d'_i + beta d'_pi(i)
touches d only.  Because sum_i d_i = 0 and pi(i) is uniform over all nodes,
E[d'_i d'_pi(i)] = 0 and E[d'_pi(i) w'_i] = 0, so the second moments
(E d^2, E d w, E w^2) obey a closed 3 x 3 linear recursion: the local step's
A S A^T + noise, then E d^2 scaled by (1 - beta)^2 + beta^2 (one half at
beta = 1/2, the factor of E[M^T M] in Section 6.1.1 away from the consensus
direction) and E d w by (1 - beta).  Its fixed point is the floor the
consensus distance settles on; it scales like the square of the step size,
which is why annealing the step size moves gossip's consensus floor with it
(the observation of Section 4.3), while all-reduce keeps the nodes identical.
"""
import numpy as np


def gossip_consensus_floor(h, lr, mu, sigma, k, beta=0.5, weight_decay=0.0, nesterov=False):
    """Stationary E[(theta_i - mean)^2] per coordinate, right after the mix, for curvatures `h` (array).
    Sum it over the coordinates and multiply by k for sum_i ||theta_i - mean||^2."""
    H = np.asarray(h, np.float64) + float(weight_decay)
    a = float(lr)
    if nesterov:
        A00, A01 = 1.0 - a * H * (1.0 + mu), np.full_like(H, mu * mu)
        b0 = -a * sigma * (1.0 + mu)
    else:
        A00, A01 = 1.0 - a * H, np.full_like(H, float(mu))
        b0 = -a * sigma
    A10, A11 = -a * H, np.full_like(H, float(mu))
    b1 = -a * sigma
    s2 = 1.0 - 1.0 / k
    # local step on the moments z = (E d^2, E d w, E w^2):  z' = L z + s2 r
    L = np.empty(H.shape + (3, 3))
    L[..., 0, 0], L[..., 0, 1], L[..., 0, 2] = A00 * A00, 2 * A00 * A01, A01 * A01
    L[..., 1, 0], L[..., 1, 1], L[..., 1, 2] = A00 * A10, A00 * A11 + A01 * A10, A01 * A11
    L[..., 2, 0], L[..., 2, 1], L[..., 2, 2] = A10 * A10, 2 * A10 * A11, A11 * A11
    r = np.array([b0 * b0, b0 * b1, b1 * b1])
    D = np.diag([(1.0 - beta) ** 2 + beta ** 2, 1.0 - beta, 1.0])          # the mix
    M = np.eye(3) - D @ L
    z = np.linalg.solve(M, np.broadcast_to(s2 * (D @ r), H.shape + (3,))[..., None])[..., 0]
    return z[..., 0]

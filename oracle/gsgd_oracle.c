/*
 * gsgd_oracle.c -- plain CPU oracle for the per-step parameter-aggregation
 * update of "How to scale distributed deep learning?" (arXiv 1611.04581).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the slow, scalar, obviously-correct
 * statement of what the GPU library must compute.  Only the test-suite, the
 * smoke check and the CPU-baseline leg of the benchmark may call it.  It shares
 * no code, header, table or constant generator with the HIP path and the
 * product never links or imports it.
 *
 * Conventions (the paper's notation, Section 2 "Background"):
 *   k replicas (the paper's p nodes), d parameters, row stride ld >= n.
 *   x = theta (parameters), v = Delta-theta (momentum / update buffer),
 *   g = stochastic gradient, c = theta-tilde (EASGD centre), lr = alpha,
 *   mu = momentum, beta = gossip mixing weight, alpha_e = EASGD moving rate.
 *   Arrays are row-major fp32, one row per replica: a[i*ld + j].
 *
 * Every routine works on a column slice: local column j stands for global
 * column col0 + j.  All three aggregation rules are independent per column, so
 * a slice of the full problem is computed exactly as the full problem would
 * compute it (the random streams are indexed by the global column).
 *
 * Arithmetic: state is fp32 (the paper trains in fp32); element-wise
 * operations are written out one rounding at a time with fmaf where a fused
 * multiply-add is meant (compile with -ffp-contract=off so nothing else is
 * fused); k-way sums (all-reduce average, EASGD centre) and the statistics
 * are accumulated in fp64 in ascending replica order; the Gaussian noise
 * transform is evaluated in fp64 and rounded once to fp32.
 *
 * Pins (tests that tie this file to something other than itself) live in
 * tests/test_oracle_*.py; every function below has at least one, so nothing
 * here is "parity unpinned".  The one caveat: the Philox known-answer vectors
 * in tests/golden/ are the generator authors' published ones, recalled rather
 * than downloaded; a second pin (the same round structure at 64-bit width
 * against numpy's Philox) guards the wiring independently.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11, "Parallel random
 * numbers: as easy as 1, 2, 3", Section 3.3 / Table 2 constants).
 * One round: two 32x32->64 products; the high halves are xored with the
 * neighbouring counter words and the round key, the low halves pass through
 * permuted.  The key is bumped by the Weyl constants between rounds.        */

static void philox_round(uint32_t c[4], uint32_t k0, uint32_t k1)
{
    const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c[0];
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c[2];
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    const uint32_t n0 = hi1 ^ c[1] ^ k0;
    const uint32_t n1 = lo1;
    const uint32_t n2 = hi0 ^ c[3] ^ k1;
    const uint32_t n3 = lo0;
    c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
}

void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c[4] = { ctr[0], ctr[1], ctr[2], ctr[3] };
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        if (r > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
        philox_round(c, k0, k1);
    }
    out[0] = c[0]; out[1] = c[1]; out[2] = c[2]; out[3] = c[3];
}

/* Stream ids: the fourth counter word says what the numbers are for. */
enum { STREAM_GRAD = 0, STREAM_INIT = 1, STREAM_XSTAR = 2, STREAM_H = 3, STREAM_X0 = 4, STREAM_PERM = 5 };

/* counter = (quad, replica, step, stream), key = (seed low, seed high) */
static void philox_at(uint64_t seed, uint32_t quad, uint32_t replica, uint32_t step,
                      uint32_t stream, uint32_t out[4])
{
    const uint32_t ctr[4] = { quad, replica, step, stream };
    const uint32_t key[2] = { (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32) };
    oracle_philox4x32_10(ctr, key, out);
}

/* ------------------------------------------------------------------------ */
/* u32 -> open-interval uniform.  The top 23 bits b give u = (2b+1)/2^24, a
 * 24-bit odd numerator, so u is exactly representable in fp32, never 0 or 1,
 * and symmetric about 1/2.                                                   */
float oracle_u01(uint32_t r)
{
    return (float)(r >> 9) * 0x1.0p-23f + 0x1.0p-24f;
}

/* Four unit-variance zero-mean noise values from four words (the analysis
 * only asks for zero mean and bounded variance, Theorem 1 / Section 6.1;
 * Gaussian noise is the example it names).
 *   kind 0: Box-Muller in fp64 on (u0,u1) -> (z0,z1) and (u2,u3) -> (z2,z3),
 *           z_even = rho cos(2 pi u'), z_odd = rho sin(2 pi u'), rho = sqrt(-2 ln u)
 *   kind 1: sqrt(3) (2u - 1), all in fp32 with one rounding (2u-1 is exact)  */
void oracle_noise4(const uint32_t r[4], int kind, float xi[4])
{
    if (kind == 1) {
        const float sqrt3 = 1.7320508075688772f;
        for (int m = 0; m < 4; ++m) {
            const float u = oracle_u01(r[m]);
            const float w = fmaf(2.0f, u, -1.0f);
            xi[m] = sqrt3 * w;
        }
        return;
    }
    const double two_pi = 6.283185307179586476925286766559;
    for (int pair = 0; pair < 2; ++pair) {
        const double ua = (double)oracle_u01(r[2 * pair]);
        const double ub = (double)oracle_u01(r[2 * pair + 1]);
        const double rho = sqrt(-2.0 * log(ua));
        xi[2 * pair]     = (float)(rho * cos(two_pi * ub));
        xi[2 * pair + 1] = (float)(rho * sin(two_pi * ub));
    }
}

/* Noise for global column j of replica `replica` at step `step` on `stream`. */
static float noise_at(uint64_t seed, int64_t j, uint32_t replica, uint32_t step,
                      uint32_t stream, int kind)
{
    uint32_t r[4];
    float xi[4];
    philox_at(seed, (uint32_t)(j >> 2), replica, step, stream, r);
    oracle_noise4(r, kind, xi);
    return xi[j & 3];
}

static float uniform_at(uint64_t seed, int64_t j, uint32_t replica, uint32_t step, uint32_t stream)
{
    uint32_t r[4];
    philox_at(seed, (uint32_t)(j >> 2), replica, step, stream, r);
    return oracle_u01(r[j & 3]);
}

/* ------------------------------------------------------------------------ */
/* Shared synthetic vectors of the noisy quadratic f(x) = 1/2 sum_j h_j (x_j - x*_j)^2
 * (strongly convex with m = min h, L = max h, the setting of Theorem 1):
 *   which 2: x* ~ N(0,1);  which 3: h ~ U(0.1, 1) as fma(0.9, u, 0.1);  which 4: x0 ~ N(0,1). */
int oracle_fill(float* dst, int64_t col0, int64_t n, uint64_t seed, int which)
{
    if (which != STREAM_XSTAR && which != STREAM_H && which != STREAM_X0) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; ++j) {
        const int64_t gj = col0 + j;
        if (which == STREAM_H)
            dst[j] = fmaf(0.9f, uniform_at(seed, gj, 0u, 0u, STREAM_H), 0.1f);
        else
            dst[j] = noise_at(seed, gj, 0u, 0u, (uint32_t)which, 0);
    }
    return 0;
}

/* Initialisation (first line of Algorithms 1-4: every node starts from the
 * same theta_0; the EASGD server starts its centre there too).
 *   mode 0: x_i <- x0 for all i, centre <- x0
 *   mode 1: x_i <- N(0,1) per replica (stream INIT), centre <- mean_i x_i
 *           (an extension so that a run can start from non-zero consensus distance)
 * v <- 0 in both modes.  centre may be NULL.                                 */
int oracle_init_replicas(float* x, float* v, float* center, const float* x0,
                         int32_t k, int64_t col0, int64_t n, int64_t ld, uint64_t seed, int mode)
{
    if (mode != 0 && mode != 1) return -1;
    if (mode == 0 && !x0) return -1;
    for (int32_t i = 0; i < k; ++i) {
        #pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            x[i * ld + j] = mode == 0 ? x0[j] : noise_at(seed, col0 + j, (uint32_t)i, 0u, STREAM_INIT, 0);
            v[i * ld + j] = 0.0f;
        }
    }
    if (center) {
        #pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            if (mode == 0) { center[j] = x0[j]; continue; }
            double s = 0.0;
            for (int32_t i = 0; i < k; ++i) s += (double)x[i * ld + j];
            center[j] = (float)(s / (double)k);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Synthetic stochastic gradient g_i = h (.) (x_i - x*) + sigma xi_i : the
 * gradient of the quadratic plus additive zero-mean noise, the sampling model
 * of Theorem 1.                                                              */
void oracle_gen_grad(const float* x, const float* h, const float* xstar, float* g,
                     int32_t k, int64_t col0, int64_t n, int64_t ld,
                     float sigma, uint64_t seed, uint32_t step, int noise_kind)
{
    for (int32_t i = 0; i < k; ++i) {
        #pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            const float xi = noise_at(seed, col0 + j, (uint32_t)i, step, STREAM_GRAD, noise_kind);
            const float t1 = x[i * ld + j] - xstar[j];
            const float t2 = sigma * xi;
            g[i * ld + j] = fmaf(h[j], t1, t2);
        }
    }
}

/* Per-column step size for a segmented (per-layer-tensor) layout: column gj
 * lies in segment s when seg_offsets[s] <= gj < seg_offsets[s+1]; its step
 * size is lr * seg_lr_scale[s] (one fp32 product).  n_seg == 0 means flat.  */
int oracle_expand_lr(float lr, int32_t n_seg, const int64_t* seg_offsets, const float* seg_lr_scale,
                     int64_t col0, int64_t n, float* lr_col)
{
    if (n_seg == 0) { for (int64_t j = 0; j < n; ++j) lr_col[j] = lr; return 0; }
    for (int64_t j = 0; j < n; ++j) {
        const int64_t gj = col0 + j;
        int32_t s = -1;
        for (int32_t t = 0; t < n_seg; ++t)
            if (seg_offsets[t] <= gj && gj < seg_offsets[t + 1]) { s = t; break; }
        if (s < 0) return -1;
        lr_col[j] = lr * seg_lr_scale[s];
    }
    return 0;
}

/* Local momentum step, identical in Algorithms 2, 3 and 4:
 *   Delta-theta_{t,i} <- -alpha grad + mu Delta-theta_{t-1,i};  theta' <- theta + Delta-theta. */
static inline float momentum_update(float v, float g, float lr, float mu)
{
    const float t3 = mu * v;
    return fmaf(-lr, g, t3);
}

/* Gossip step (Section 3.1; the variant of Section 6.2.2 that mixes post-step parameters):
 *   theta'_i = local momentum step of replica i
 *   theta_{t+1,i} = theta'_i - beta (theta'_i - theta'_{peer[i]})
 * peer[] may be any map into 0..k-1 (a permutation is the case where pull-
 * and push-gossip coincide); peer[i] == i is a no-op mix.                    */
int oracle_step_gossip(float* x, float* v, const float* g, int32_t k, int64_t n, int64_t ld,
                       const float* lr_col, float mu, float beta, const int32_t* peer)
{
    for (int32_t i = 0; i < k; ++i) if (peer[i] < 0 || peer[i] >= k) return -1;
    float* xp = (float*)malloc(sizeof(float) * (size_t)k * (size_t)n);
    if (!xp) return -2;
    for (int32_t i = 0; i < k; ++i) {
        #pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            const float vn = momentum_update(v[i * ld + j], g[i * ld + j], lr_col[j], mu);
            v[i * ld + j] = vn;
            xp[(int64_t)i * n + j] = x[i * ld + j] + vn;
        }
    }
    for (int32_t i = 0; i < k; ++i) {
        const int32_t p = peer[i];
        #pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            const float mine = xp[(int64_t)i * n + j];
            const float theirs = xp[(int64_t)p * n + j];
            x[i * ld + j] = fmaf(-beta, mine - theirs, mine);
        }
    }
    free(xp);
    return 0;
}

/* Synchronous all-reduce step (Algorithm 1):
 *   Delta-theta_{t,i} = -alpha grad_i + mu Delta-theta_{t-1}   (each node's own copy of the last averaged update)
 *   Delta-theta_t = average over i;  theta_{t+1,i} = theta_{t,i} + Delta-theta_t;  every node keeps Delta-theta_t. */
int oracle_step_allreduce(float* x, float* v, const float* g, int32_t k, int64_t n, int64_t ld,
                          const float* lr_col, float mu)
{
    double* acc = (double*)calloc((size_t)n, sizeof(double));
    if (!acc) return -2;
    for (int32_t i = 0; i < k; ++i) {
        #pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j)
            acc[j] += (double)momentum_update(v[i * ld + j], g[i * ld + j], lr_col[j], mu);
    }
    for (int32_t i = 0; i < k; ++i) {
        #pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            const float ubar = (float)(acc[j] / (double)k);
            v[i * ld + j] = ubar;
            x[i * ld + j] = x[i * ld + j] + ubar;
        }
    }
    free(acc);
    return 0;
}

/* Elastic-averaging step (Algorithm 2, communication period 1, all clients
 * exchanging with the same centre value in one synchronous round):
 *   theta'_i = local momentum step
 *   e_i = alpha_e (theta'_i - c);  theta_i <- theta'_i - e_i;  c <- c + sum_i e_i            */
int oracle_step_easgd(float* x, float* v, const float* g, float* center, int32_t k, int64_t n, int64_t ld,
                      const float* lr_col, float mu, float alpha_e)
{
    double* acc = (double*)calloc((size_t)n, sizeof(double));
    if (!acc) return -2;
    for (int32_t i = 0; i < k; ++i) {
        #pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            const float vn = momentum_update(v[i * ld + j], g[i * ld + j], lr_col[j], mu);
            const float xp = x[i * ld + j] + vn;
            const float e = alpha_e * (xp - center[j]);
            v[i * ld + j] = vn;
            x[i * ld + j] = xp - e;
            acc[j] += (double)e;
        }
    }
    #pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; ++j)
        center[j] = (float)((double)center[j] + acc[j]);
    free(acc);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Variants the paper's experiments and appendix use beyond the algorithm boxes
 * (Section 4.2: Nesterov momentum 0.9 and weight decay 1e-4; Section 6.2.1:
 * gossip with stale parameters).  The functions above are the special case
 * wd = 0, nesterov = 0, stale = 0 of the ones below (a test checks bit equality).
 *
 * Local step with weight decay and optional Nesterov momentum, in the usual
 * "momentum buffer" form:
 *   gt = g + wd x  (gt = g when wd is zero);   v' = mu v - lr gt;
 *   heavy ball: x' = x + v'        Nesterov: x' = (x - lr gt) + mu v'           */
static inline void local_step_ext(float x, float v, float g, float lr, float mu, float wd, int nesterov,
                                  float* v_new, float* x_post)
{
    /* A weight decay of zero means the decay term is absent (the algorithm boxes have none), not "+ 0 * x":
     * the gradient then enters as it stands, the sign of a zero included, and the step is the boxed one bit for bit. */
    const float gt = wd != 0.0f ? fmaf(wd, x, g) : g;
    const float t3 = mu * v;
    const float vn = fmaf(-lr, gt, t3);
    *v_new = vn;
    if (nesterov) {
        const float t4 = fmaf(-lr, gt, x);
        *x_post = fmaf(mu, vn, t4);
    } else {
        *x_post = x + vn;
    }
}

/* Gossip with fresh (stale = 0, Section 6.2.2) or stale (stale = 1, Section
 * 6.2.1) parameters.  Stale: the mixing term uses the parameters from before
 * the local step, theta_{t+1,i} = theta'_i - beta (theta_{t,i} - theta_{t,peer}). */
int oracle_step_gossip_ext(float* x, float* v, const float* g, int32_t k, int64_t n, int64_t ld,
                           const float* lr_col, float mu, float wd, int nesterov, float beta,
                           const int32_t* peer, int stale)
{
    for (int32_t i = 0; i < k; ++i) if (peer[i] < 0 || peer[i] >= k) return -1;
    float* xp = (float*)malloc(sizeof(float) * (size_t)k * (size_t)n);
    float* xo = (float*)malloc(sizeof(float) * (size_t)k * (size_t)n);
    if (!xp || !xo) { free(xp); free(xo); return -2; }
    for (int32_t i = 0; i < k; ++i) {
        #pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            float vn, xpost;
            local_step_ext(x[i * ld + j], v[i * ld + j], g[i * ld + j], lr_col[j], mu, wd, nesterov, &vn, &xpost);
            xo[(int64_t)i * n + j] = x[i * ld + j];
            v[i * ld + j] = vn;
            xp[(int64_t)i * n + j] = xpost;
        }
    }
    const float* mixed = stale ? xo : xp;
    for (int32_t i = 0; i < k; ++i) {
        const int32_t p = peer[i];
        #pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            const float diff = mixed[(int64_t)i * n + j] - mixed[(int64_t)p * n + j];
            x[i * ld + j] = fmaf(-beta, diff, xp[(int64_t)i * n + j]);
        }
    }
    free(xp); free(xo);
    return 0;
}

/* All-reduce (Algorithm 1) with the extended local step: every node's momentum
 * buffer and the update it applies to theta are both averaged over the nodes.
 *   heavy ball: applied update d_i = v'_i;  Nesterov: d_i = mu v'_i - lr gt_i
 *   v_i <- mean_i v'_i;  theta_i <- theta_i + mean_i d_i                          */
int oracle_step_allreduce_ext(float* x, float* v, const float* g, int32_t k, int64_t n, int64_t ld,
                              const float* lr_col, float mu, float wd, int nesterov)
{
    double* acc_v = (double*)calloc((size_t)n, sizeof(double));
    double* acc_d = (double*)calloc((size_t)n, sizeof(double));
    if (!acc_v || !acc_d) { free(acc_v); free(acc_d); return -2; }
    for (int32_t i = 0; i < k; ++i) {
        #pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            const float xi = x[i * ld + j];
            const float gt = wd != 0.0f ? fmaf(wd, xi, g[i * ld + j]) : g[i * ld + j];   /* as in local_step_ext */
            const float t3 = mu * v[i * ld + j];
            const float vn = fmaf(-lr_col[j], gt, t3);
            float di = vn;
            if (nesterov) { const float t5 = mu * vn; di = fmaf(-lr_col[j], gt, t5); }
            acc_v[j] += (double)vn;
            acc_d[j] += (double)di;
        }
    }
    for (int32_t i = 0; i < k; ++i) {
        #pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            const float vbar = (float)(acc_v[j] / (double)k);
            const float dbar = (float)(acc_d[j] / (double)k);
            v[i * ld + j] = vbar;
            x[i * ld + j] = x[i * ld + j] + dbar;
        }
    }
    free(acc_v); free(acc_d);
    return 0;
}

/* Elastic averaging (Algorithm 2) with the extended local step. */
int oracle_step_easgd_ext(float* x, float* v, const float* g, float* center, int32_t k, int64_t n, int64_t ld,
                          const float* lr_col, float mu, float wd, int nesterov, float alpha_e)
{
    double* acc = (double*)calloc((size_t)n, sizeof(double));
    if (!acc) return -2;
    for (int32_t i = 0; i < k; ++i) {
        #pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            float vn, xp;
            local_step_ext(x[i * ld + j], v[i * ld + j], g[i * ld + j], lr_col[j], mu, wd, nesterov, &vn, &xp);
            const float e = alpha_e * (xp - center[j]);
            v[i * ld + j] = vn;
            x[i * ld + j] = xp - e;
            acc[j] += (double)e;
        }
    }
    #pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; ++j)
        center[j] = (float)((double)center[j] + acc[j]);
    free(acc);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Peer permutation for one step: Fisher-Yates driven by Philox stream PERM.
 * For i = k-1 .. 1: r = word 0 of Philox(counter (i, 0, step, PERM), seed);
 * j = floor(r (i+1) / 2^32); swap p[i], p[j].  Integer only.                 */
int oracle_make_perm(uint64_t seed, uint32_t step, int32_t k, int32_t* out)
{
    if (k < 1) return -1;
    for (int32_t i = 0; i < k; ++i) out[i] = i;
    for (int32_t i = k - 1; i >= 1; --i) {
        uint32_t r[4];
        philox_at(seed, (uint32_t)i, 0u, step, STREAM_PERM, r);
        const int32_t j = (int32_t)(((uint64_t)r[0] * (uint64_t)(i + 1)) >> 32);
        const int32_t t = out[i]; out[i] = out[j]; out[j] = t;
    }
    return 0;
}

/* Independent uniform targets for one step (Section 3.1: every node draws
 * j ~ Uniform over the nodes): node i uses word 0 of Philox(counter
 * (i, 1, step, PERM), seed).  exclude_self = 0: j = floor(r k / 2^32), the node
 * itself included (pull-gossip).  exclude_self = 1: a uniform draw among the
 * k-1 other nodes, j = floor(r (k-1) / 2^32), stepped over i (push-gossip sends to
 * a node other than itself); needs k >= 2.                                          */
int oracle_make_targets(uint64_t seed, uint32_t step, int32_t k, int exclude_self, int32_t* out)
{
    if (k < 1 || (exclude_self && k < 2)) return -1;
    for (int32_t i = 0; i < k; ++i) {
        uint32_t r[4];
        philox_at(seed, (uint32_t)i, 1u, step, STREAM_PERM, r);
        if (!exclude_self) {
            out[i] = (int32_t)(((uint64_t)r[0] * (uint64_t)k) >> 32);
        } else {
            const int32_t j = (int32_t)(((uint64_t)r[0] * (uint64_t)(k - 1)) >> 32);
            out[i] = j >= i ? j + 1 : j;
        }
    }
    return 0;
}

/* Push-gossip step (Algorithm 4): after the local step every node sends its
 * parameters to itself and to its target; a node's new parameters are the
 * average of what it received,
 *   theta_r <- ( theta'_r + sum over { i != r : target[i] = r } of theta'_i ) / (1 + number of such i).
 * A node whose target is itself sends nothing beyond its own copy.  The sum
 * runs in fp64 (own value first, then senders in ascending index) and the
 * average is rounded once to fp32.                                            */
int oracle_step_gossip_push(float* x, float* v, const float* g, int32_t k, int64_t n, int64_t ld,
                            const float* lr_col, float mu, float wd, int nesterov, const int32_t* target)
{
    for (int32_t i = 0; i < k; ++i) if (target[i] < 0 || target[i] >= k) return -1;
    float* xp = (float*)malloc(sizeof(float) * (size_t)k * (size_t)n);
    if (!xp) return -2;
    for (int32_t i = 0; i < k; ++i) {
        #pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            float vn, xpost;
            local_step_ext(x[i * ld + j], v[i * ld + j], g[i * ld + j], lr_col[j], mu, wd, nesterov, &vn, &xpost);
            v[i * ld + j] = vn;
            xp[(int64_t)i * n + j] = xpost;
        }
    }
    for (int32_t r = 0; r < k; ++r) {
        int32_t received = 1;
        for (int32_t i = 0; i < k; ++i) if (i != r && target[i] == r) ++received;
        #pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            double s = (double)xp[(int64_t)r * n + j];
            for (int32_t i = 0; i < k; ++i)
                if (i != r && target[i] == r) s += (double)xp[(int64_t)i * n + j];
            x[r * ld + j] = (float)(s / (double)received);
        }
    }
    free(xp);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Asynchronous pull-gossip, one tick of the master clock (Section 6.1.2): the
 * node i whose clock ticked takes its local step and pulls from node j,
 *   theta_{t+1,i} = (1 - beta)(theta_{t,i} - alpha g_{t,i}) + beta theta_{t,j},   theta_{t+1,m} = theta_{t,m} for m != i,
 * i.e. theta_{t+1} = D (theta_t - alpha g_t) with D = I + beta e_i (e_j - e_i)^T.  j is read as it stands
 * (node j takes no step in this tick); j == i leaves theta'_i.  g_row is node i's gradient (n values).
 * The local step is the same as everywhere else (momentum / weight decay / Nesterov optional); the mix is written
 * theta' - beta (theta' - theta_j) as in Section 3.1.                                                              */
int oracle_async_tick(float* x, float* v, const float* g_row, int32_t k, int64_t n, int64_t ld,
                      const float* lr_col, float mu, float wd, int nesterov, float beta, int32_t i, int32_t j)
{
    if (i < 0 || i >= k || j < 0 || j >= k) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < n; ++c) {
        float vn, xp;
        local_step_ext(x[i * ld + c], v[i * ld + c], g_row[c], lr_col[c], mu, wd, nesterov, &vn, &xp);
        const float theirs = (j == i) ? xp : x[j * ld + c];
        v[i * ld + c] = vn;
        x[i * ld + c] = fmaf(-beta, xp - theirs, xp);
    }
    return 0;
}

/* Elastic averaging as Algorithm 2 states it, one client at a time: client i takes its local step and exchanges
 * with the server, which applies that one client's update immediately (the asynchronous parameter-server form):
 *   theta'_i = local step;  e = alpha_e (theta'_i - c);  theta_i <- theta'_i - e;  c <- c + e.
 * The other clients and their view of the centre are untouched; they meet the moved centre at their own exchange. */
int oracle_easgd_tick(float* x, float* v, const float* g_row, float* center, int32_t k, int64_t n, int64_t ld,
                      const float* lr_col, float mu, float wd, int nesterov, float alpha_e, int32_t i)
{
    if (i < 0 || i >= k) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < n; ++c) {
        float vn, xp;
        local_step_ext(x[i * ld + c], v[i * ld + c], g_row[c], lr_col[c], mu, wd, nesterov, &vn, &xp);
        const float e = alpha_e * (xp - center[c]);
        v[i * ld + c] = vn;
        x[i * ld + c] = xp - e;
        center[c] = center[c] + e;
    }
    return 0;
}

/* Synthetic gradient of one node for one tick: as oracle_gen_grad, for row i only, the noise drawn at counter
 * (column / 4, i, tick, GRAD).                                                                                    */
void oracle_gen_grad_row(const float* x, const float* h, const float* xstar, float* g_row,
                         int32_t i, int64_t col0, int64_t n, int64_t ld,
                         float sigma, uint64_t seed, uint32_t tick, int noise_kind)
{
    #pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < n; ++c) {
        const float xi = noise_at(seed, col0 + c, (uint32_t)i, tick, STREAM_GRAD, noise_kind);
        const float t1 = x[i * ld + c] - xstar[c];
        const float t2 = sigma * xi;
        g_row[c] = fmaf(h[c], t1, t2);
    }
}

/* Which node ticks and whom it pulls from (Section 6.1.2: the ticking clock is uniform over the nodes, and so is
 * the node pulled from): words 0 and 1 of Philox(counter (tick, 2, 0, PERM), seed), each mapped by floor(r k / 2^32). */
int oracle_make_tick(uint64_t seed, uint32_t tick, int32_t k, int32_t* i_out, int32_t* j_out)
{
    if (k < 1) return -1;
    uint32_t r[4];
    philox_at(seed, tick, 2u, 0u, STREAM_PERM, r);
    *i_out = (int32_t)(((uint64_t)r[0] * (uint64_t)k) >> 32);
    *j_out = (int32_t)(((uint64_t)r[1] * (uint64_t)k) >> 32);
    return 0;
}

/* The two quantities the analysis bounds (Section 6.1) plus the mean's own
 * distance, all over the slice, in fp64:
 *   out[0] = sum_i ||x_i - xbar||^2   (agent consensus)
 *   out[1] = sum_i ||x_i - x*||^2     (distance to the optimum)
 *   out[2] = ||xbar - x*||^2
 *   out[3] = ||xbar||^2                                                       */
void oracle_stats(const float* x, const float* xstar, int32_t k, int64_t n, int64_t ld, double out[4])
{
    double cons = 0.0, dist = 0.0, mdist = 0.0, mnorm = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        double s = 0.0;
        for (int32_t i = 0; i < k; ++i) s += (double)x[i * ld + j];
        const double xbar = s / (double)k;
        for (int32_t i = 0; i < k; ++i) {
            const double a = (double)x[i * ld + j] - xbar;
            const double b = (double)x[i * ld + j] - (double)xstar[j];
            cons += a * a;
            dist += b * b;
        }
        const double c = xbar - (double)xstar[j];
        mdist += c * c;
        mnorm += xbar * xbar;
    }
    out[0] = cons; out[1] = dist; out[2] = mdist; out[3] = mnorm;
}

/* Limit the threads of the parallel loops above (for the benchmark's one-thread figure); n < 1 is ignored. */
void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    extern void omp_set_num_threads(int);
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* How many threads the parallel loops above use (for the benchmark's report). */
int oracle_num_threads(void)
{
    int n = 1;
    #pragma omp parallel
    {
        #pragma omp single
        {
#ifdef _OPENMP
            extern int omp_get_num_threads(void);
            n = omp_get_num_threads();
#endif
        }
    }
    return n;
}

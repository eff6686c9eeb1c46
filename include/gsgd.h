/*
 * gsgd.h -- C ABI of libgsgd, the MI355X (gfx950) library for the per-step
 * parameter-aggregation update of "How to scale distributed deep learning?"
 * (Jin, Yuan, Iandola, Keutzer; arXiv 1611.04581): a local momentum-SGD step
 * fused with gossip pairwise averaging (the paper's Section 3), and the two
 * rules it is compared with, synchronous all-reduce averaging (Algorithm 1)
 * and elastic averaging (Algorithm 2).
 *
 * The k "nodes" of the paper are k replica rows that all live in one GPU's
 * memory.  Notation follows the paper's Section 2: theta -> x (parameters),
 * Delta-theta -> v (momentum / update buffer), grad f_i -> g, theta-tilde ->
 * center, alpha -> lr, mu -> momentum, p -> k.  The gossip mixing weight is
 * beta (Section 3.1; the authors' runs use 1/2).  The elastic-averaging
 * "moving rate", which Algorithm 2 also calls beta, is alpha_e here.
 *
 * Memory model
 *   - x, v, g are row-major fp32 matrices of k rows with a row stride of ld
 *     elements (ld >= d, ld % 4 == 0); element (i, j) is at base[i*ld + j].
 *     Only columns 0..d-1 are read or written.  center, h, xstar, x0 are fp32
 *     vectors of at least d elements.
 *   - Blocked layout (gsgd_config.block_columns = B > 0, a power of two >= 1024,
 *     ld a multiple of B): the same k * ld elements hold the columns in blocks
 *     of B, each block with its k row pieces back to back; element (i, j) is at
 *     base[(j / B) * k * B + i * B + j % B].  A replica's vector is then a
 *     sequence of B-element pieces k * B apart, and the k values of a column
 *     lie B elements apart instead of ld, which is what the kernels that walk
 *     a column's replicas stream fastest.  Every entry point that takes a
 *     context follows the context's layout; vectors are plain in both.
 *   - Every pointer named "device" is GPU memory owned by the caller, 16-byte
 *     aligned, valid until the stream has run the call.  The library never
 *     frees or reallocates caller memory.  x, v, g, center must not overlap,
 *     and h, xstar, x0 must not overlap anything a call writes: the address
 *     ranges are compared, and an overlap is GSGD_ERR_INVALID_ARG.
 *   - Pointers named "host" are ordinary host memory, read (or written, for
 *     outputs) before the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Step calls only enqueue kernels; they do not synchronise, allocate or
 *     clear memory, so a caller may record a run of them into a HIP graph
 *     (peer maps, step numbers and hyper-parameters are baked in as kernel
 *     arguments at record time).  gsgd_stats and gsgd_row_sqnorms wait for
 *     the stream and must stay outside a capture.
 *   - One context may be used from several streams at once (at most 32 over
 *     its lifetime; a 33rd gets GSGD_ERR_UNSUPPORTED): every stream hands out
 *     tiles through a counter pair of its own.  A recorded graph keeps the
 *     pair of the stream it was captured on, so it must not replay while
 *     eager calls or another replay of the same context run on that stream's
 *     pair from a different stream.
 *
 * Errors: every function returns GSGD_OK (0) or a negative code; nothing
 * throws, aborts or prints.  A gsgd_ctx is not thread-safe; distinct contexts
 * are independent.
 */
#ifndef GSGD_H
#define GSGD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GSGD_MAX_K 512              /* most replicas one context can hold */

enum {
    GSGD_OK               =  0,
    GSGD_ERR_INVALID_ARG  = -1,    /* null pointer, k/d/ld out of range, misaligned pointer, bad enum */
    GSGD_ERR_BAD_PERM     = -2,    /* peer entry outside 0..k-1, or peer_perm not a bijection where one is required */
    GSGD_ERR_BAD_SEGMENTS = -3,    /* segment table not ascending from 0 to d */
    GSGD_ERR_HIP          = -4,    /* a HIP runtime call failed; see gsgd_last_hip_error */
    GSGD_ERR_UNSUPPORTED  = -5,    /* the context has launched on 32 distinct streams already */
    GSGD_ERR_NO_MEMORY    = -6,
    GSGD_ERR_BAD_STATE    = -7,    /* a tile counter was found non-zero on a drained stream; see gsgd_stats */
    GSGD_ERR_TOO_LARGE    = -8     /* input beyond the stated maximum of gsgd_stats_static */
};

enum { GSGD_NOISE_GAUSSIAN = 0, GSGD_NOISE_UNIFORM = 1 };
enum { GSGD_INIT_BROADCAST = 0, GSGD_INIT_PER_REPLICA = 1 };
enum { GSGD_FILL_XSTAR = 2, GSGD_FILL_H = 3, GSGD_FILL_X0 = 4 };
enum { GSGD_ROW_SPLIT_AUTO = 0, GSGD_ROW_SPLIT_OFF = 1, GSGD_ROW_SPLIT_ON = 2 };
enum { GSGD_GOSSIP_AUTO = 0, GSGD_GOSSIP_WALK = 1, GSGD_GOSSIP_SWEEP = 2, GSGD_GOSSIP_SWEEP_SPLIT = 3 };
/* the streaming kernels, for gsgd_set_launch_width.  The local step and the gradient generator are plain grids on
 * row-major matrices (and the generator below 12 replicas): there the number is the 1024-column tiles per band of
 * the grid; on blocked matrices they are persistent workgroups like the others and the number counts those. */
enum { GSGD_KERNEL_GOSSIP = 0, GSGD_KERNEL_ALLREDUCE = 1, GSGD_KERNEL_EASGD = 2, GSGD_KERNEL_GEN_GRAD = 3,
       GSGD_KERNEL_GOSSIP_FUSED = 4, GSGD_KERNEL_LOCAL = 5, GSGD_KERNEL_COUNT = 6 };

typedef struct gsgd_ctx gsgd_ctx;   /* opaque; owns the segment tables and a small scratch for gsgd_stats */

typedef struct gsgd_config {
    int32_t  k;                     /* replicas, 1..GSGD_MAX_K (the paper's p) */
    int64_t  d;                     /* parameters per replica, >= 1 */
    int64_t  ld;                    /* row stride in elements, >= d, multiple of 4 */
    float    lr;                    /* step size alpha (Section 2) */
    float    momentum;              /* mu (Section 2) */
    float    sigma;                 /* std-dev of the additive gradient noise (Theorem 1's xi) */
    uint64_t seed;                  /* Philox key */
    int32_t  noise_kind;            /* GSGD_NOISE_*: both are zero-mean unit-variance (Theorem 1's assumption) */
    int32_t  n_seg;                 /* 0 = flat vector; else number of per-layer tensors laid back to back */
    const int64_t* seg_offsets;     /* host, n_seg+1 entries, [0] = 0, strictly ascending, [n_seg] = d; copied */
    const float*   seg_lr_scale;    /* host, n_seg entries; segment s steps with lr * seg_lr_scale[s]; copied */
    int64_t  block_columns;         /* 0 = row-major matrices; else the blocked layout's B (see "Memory model") */
} gsgd_config;

/* Create / destroy a context.  gsgd_create validates the configuration, copies
 * the segment tables to the current device and allocates the scratch that
 * gsgd_stats reduces into.  The current HIP device at creation is the device
 * every later call must run on. */
int gsgd_create(const gsgd_config* cfg, gsgd_ctx** out);
int gsgd_destroy(gsgd_ctx* ctx);

/* Change the base step size (the paper anneals alpha, Section 4.2).  Host only. */
int gsgd_set_lr(gsgd_ctx* ctx, float lr);

/* The local step the experiments use (Section 4.2: Nesterov momentum 0.9 and
 * weight decay 1e-4) in place of the plain heavy-ball step of the algorithm
 * boxes.  With gt = g + weight_decay * x, every step rule below computes
 *   v_i <- momentum * v_i - lr_s * gt_i;
 *   x'_i = x_i + v_i                          (nesterov = 0)
 *   x'_i = (x_i - lr_s * gt_i) + momentum * v_i   (nesterov = 1)
 * and then communicates as documented.  Under all-reduce the momentum buffers
 * and the applied updates x'_i - x_i are averaged separately (they differ when
 * nesterov = 1).  weight_decay >= 0; (0, 0) restores the default.  Host only. */
int gsgd_set_local_step(gsgd_ctx* ctx, float weight_decay, int nesterov);

/* Tuning knob.  The streaming kernels run as a fixed number of persistent
 * workgroups that pull 1024-column tiles from a ticket counter owned by the
 * context; `workgroups` sets that number for one GSGD_KERNEL_*, 0 restores the
 * default (a small multiple of the device's compute-unit count).  Results do
 * not depend on it.  Host only. */
int gsgd_set_launch_width(gsgd_ctx* ctx, int kernel, int workgroups);

/* Which kernel form the gossip calls (gsgd_step_gossip, _stale, _pull, _push and their generator-fused variants)
 * take.  Both forms compute the same update bit for bit (Section 3.1's mix of post-step parameters; Section 6.2.1's
 * with stale ones), read x, v, g once and write x, v once:
 *   GSGD_GOSSIP_WALK         rows visited along the cycles (and trees) of the peer map, values handed from row to
 *                            row in registers;
 *   GSGD_GOSSIP_SWEEP        rows visited in ascending order twice, the values a row's mix needs parked in LDS in
 *                            between; a workgroup owns 1024 columns (at most 36 replicas);
 *   GSGD_GOSSIP_SWEEP_SPLIT  the same with 256 columns per workgroup and the rows split over its wavefronts (four;
 *                            eight or twelve beyond 64 replicas) (at most 144 replicas);
 *   GSGD_GOSSIP_AUTO         (default) the walk on row-major matrices, the sweeps on blocked ones: the memory system
 *                            serves the row pieces of a block fastest in address order; in either layout the
 *                            split sweeps for vectors too short to fill the chip with 1024-column tiles.
 *                            Push-gossip runs with twice the workgroups where two fit a compute unit (up to 16
 *                            replicas in whole tiles, 37 to 64 in split ones) unless gsgd_set_launch_width has set
 *                            their number.
 * Push-gossip's fp64 sums are taken own value first, then the senders in ascending index by the sweep forms, and in
 * visiting order by the walk (the two can differ in the last place of the rounded average).
 * A sweep form asked for with more replicas than it can park falls back (SWEEP -> SWEEP_SPLIT -> WALK).  Host only. */
int gsgd_set_gossip_form(gsgd_ctx* ctx, int form);

/* How the k-way sums of gsgd_step_allreduce (the average of Algorithm 1) and
 * gsgd_step_easgd (the server's sum of Algorithm 2) are laid out.
 *   GSGD_ROW_SPLIT_OFF : one thread per four columns adds all k rows in fp64 in
 *                        ascending order (bit-identical to a serial sum);
 *   GSGD_ROW_SPLIT_ON  : the rows are split into blocks over the wavefronts of
 *                        a workgroup, each block summed in ascending order, the
 *                        block sums staged through LDS and added in ascending
 *                        block order.  Same fp64 additions, associated
 *                        differently: a result can differ from OFF in the last
 *                        place where the fp64 sum is itself inexact.  Faster
 *                        when d is too short to fill the GPU with d/4 threads;
 *   GSGD_ROW_SPLIT_AUTO: ON when d has fewer 1024-column tiles than the device
 *                        has compute units and k >= 16, else OFF (the default).
 * Host only. */
int gsgd_set_row_split(gsgd_ctx* ctx, int mode);

/* Initialisation: first line of Algorithms 1-4 (every node starts at the same
 * theta_0; the elastic-averaging server's centre starts there too).
 *   mode GSGD_INIT_BROADCAST   : x_i <- x0 for all i; center <- x0
 *   mode GSGD_INIT_PER_REPLICA : x_i <- N(0,1) drawn per replica from the
 *        context's Philox stream 1 (lets a run start from non-zero consensus
 *        distance); center <- mean_i x_i;  x0 is ignored and may be NULL
 * v <- 0 in both modes.  x, v: device k x ld.  center: device d, may be NULL.
 * x0: device d. */
int gsgd_init_replicas(gsgd_ctx* ctx, float* x, float* v, float* center, const float* x0, int mode, void* stream);

/* Copy a k x d matrix from one layout of the memory model into another (row-major with any row stride, blocked with
 * any block width), e.g. replicas loaded as flat vectors into the blocked layout the kernels stream fastest, or back.
 * Needs no context.  src, dst: device, k x src_ld / k x dst_ld elements, not overlapping; padding columns of dst are
 * left as they are.  Asynchronous on `stream`. */
int gsgd_relayout(int32_t k, int64_t d, int64_t src_ld, int64_t src_block_columns, const float* src,
                  int64_t dst_ld, int64_t dst_block_columns, float* dst, void* stream);

/* Fill a device vector of d elements with one of the shared synthetic vectors
 * of the noisy quadratic f(x) = 1/2 sum_j h_j (x_j - xstar_j)^2, which is
 * m-strongly convex with L-Lipschitz gradient for m = min h, L = max h
 * (the function class of Theorem 1):
 *   GSGD_FILL_XSTAR ~ N(0,1), GSGD_FILL_H ~ U(0.1, 1), GSGD_FILL_X0 ~ N(0,1). */
int gsgd_fill(gsgd_ctx* ctx, float* dst, int which, void* stream);

/* Synthetic stochastic gradient, the sampling model of Theorem 1
 * (g = grad f + xi, E xi = 0, bounded variance):
 *   g_i = h (.) (x_i - xstar) + sigma xi_i,   xi from Philox stream 0 at
 *   counter (column/4, replica i, step, 0).  step < 2^32.
 * x: device k x ld (read).  h, xstar: device d.  g: device k x ld (written). */
int gsgd_gen_grad(gsgd_ctx* ctx, const float* x, const float* h, const float* xstar, float* g,
                  uint64_t step, void* stream);

/* Synchronous all-reduce step, Algorithm 1:
 *   u_i = momentum * v_i - lr_s * g_i;  ubar = (1/k) sum_i u_i;
 *   v_i <- ubar;  x_i <- x_i + ubar          for every replica i.
 * The k-way sum runs in fp64 in ascending i and is rounded once to fp32
 * (for short vectors in blocks of rows, see gsgd_set_row_split).
 * x, v: device k x ld, updated in place.  g: device k x ld, read. */
int gsgd_step_allreduce(gsgd_ctx* ctx, float* x, float* v, const float* g, void* stream);

/* Gossip step: local momentum step (the two lines shared by Algorithms 2-4)
 * followed by the pairwise mix of Section 3.1 / 6.2.2 (the mix of post-step parameters):
 *   v_i <- momentum * v_i - lr_s * g_i;   x'_i = x_i + v_i;
 *   x_i <- x'_i - beta * (x'_i - x'_{peer_perm[i]}).
 * peer_perm: host, k entries, a bijection on 0..k-1 (each node is pulled from
 * exactly once, so pull- and push-gossip coincide); peer_perm[i] == i mixes a
 * replica with itself, i.e. leaves x'_i.  The array is consumed before the
 * call returns.  Everything happens in place in one pass over x, v and g. */
int gsgd_step_gossip(gsgd_ctx* ctx, float* x, float* v, const float* g,
                     const int32_t* peer_perm, float beta, void* stream);

/* Gossip with stale parameters (Section 6.2.1): the mix uses both nodes'
 * parameters from before the local step.  As gsgd_step_gossip, but
 *   x_i <- x'_i - beta * (x_i - x_{peer_perm[i]}). */
int gsgd_step_gossip_stale(gsgd_ctx* ctx, float* x, float* v, const float* g,
                           const int32_t* peer_perm, float beta, void* stream);

/* Pull-gossip with arbitrary targets (Algorithm 3; Section 3.1: every node
 * pulls from one node chosen uniformly at random, so several may pull from the
 * same node and a node may pull from itself).  The update is that of
 * gsgd_step_gossip (stale = 0) or of gsgd_step_gossip_stale (stale = 1), but
 * peer may be any map into 0..k-1.  The mixing matrix is then only
 * row-stochastic (Section 6.1.1): the replica mean is preserved in
 * expectation, not exactly.  Still one in-place pass over x, v and g.
 * peer: host, k entries, consumed before the call returns; GSGD_ERR_BAD_PERM
 * for an entry outside 0..k-1. */
int gsgd_step_gossip_pull(gsgd_ctx* ctx, float* x, float* v, const float* g,
                          const int32_t* peer, float beta, int stale, void* stream);

/* Push-gossip step (Algorithm 4): after the local step every node sends its
 * parameters to itself and to target[i]; a node's new parameters are the
 * average of what it received,
 *   x_r <- ( x'_r + sum over { i != r : target[i] = r } of x'_i ) / (1 + number of such i).
 * target may be any map into 0..k-1 (a node may receive from none or from
 * many); target[i] == i sends nothing beyond the node's own copy.  The sum is
 * accumulated in fp64 and the average rounded once.  One in-place pass over x,
 * v and g.  target: host, k entries, consumed before the call returns;
 * GSGD_ERR_BAD_PERM for an entry outside 0..k-1. */
int gsgd_step_gossip_push(gsgd_ctx* ctx, float* x, float* v, const float* g,
                          const int32_t* target, void* stream);

/* Asynchronous pull-gossip, one tick of the master clock (Section 6.1.2): node
 * i, whose clock ticked, takes its local step and mixes with node j as j
 * stands; every other node is left alone:
 *   v_i <- momentum * v_i - lr_s * g_i;  x'_i = x_i + v_i;  x_i <- x'_i - beta * (x'_i - x_j)
 * (x_j is j's current value, j takes no step; j == i leaves x'_i).  In the
 * paper's matrix form x <- D (x - lr g e_i), D = I + beta e_i (e_j - e_i)^T.
 * Only row i of g is read.  0 <= i, j < k, else GSGD_ERR_INVALID_ARG. */
int gsgd_step_async_tick(gsgd_ctx* ctx, float* x, float* v, const float* g, int32_t i, int32_t j,
                         float beta, void* stream);

/* Elastic averaging, one client's exchange with the server (Algorithm 2 as a
 * client/server protocol: the server applies each client's update as it
 * arrives).  Client i takes its local step and exchanges; nobody else moves:
 *   v_i <- momentum * v_i - lr_s * g_i;  x'_i = x_i + v_i;
 *   e = alpha_e * (x'_i - center);  x_i <- x'_i - e;  center <- center + e.
 * Only row i of g is read.  center: device d, updated in place. */
int gsgd_step_easgd_tick(gsgd_ctx* ctx, float* x, float* v, const float* g, float* center, int32_t i,
                         float alpha_e, void* stream);

/* The asynchronous pull-gossip tick with node i's synthetic gradient generated on the fly:
 * g_i = h (.) (x_i - xstar) + sigma xi, xi from Philox stream 0 at counter
 * (column/4, i, tick, 0).  tick < 2^32. */
int gsgd_step_async_tick_fused(gsgd_ctx* ctx, float* x, float* v, const float* h, const float* xstar,
                               int32_t i, int32_t j, float beta, uint64_t tick, void* stream);

/* Who ticks and whom it pulls from at tick number `tick`: i and j uniform over
 * the k nodes and independent (the Poisson-clock model of Section 6.1.2),
 * words 0 and 1 of Philox stream 5 at counter (tick, 2, 0, 5), each mapped by
 * floor(r k / 2^32).  Pure host code. */
int gsgd_make_tick(uint64_t seed, uint64_t tick, int32_t k, int32_t* i_out, int32_t* j_out);

/* n_ticks consecutive ticks first_tick, first_tick+1, ... of the asynchronous
 * model, each drawn with gsgd_make_tick under the context's seed and run with
 * gsgd_step_async_tick_fused.  Enqueues n_ticks kernels; does not wait. */
int gsgd_run_async_ticks(gsgd_ctx* ctx, float* x, float* v, const float* h, const float* xstar,
                         float beta, uint64_t first_tick, uint64_t n_ticks, void* stream);

/* The local step alone (v_i and x_i <- x'_i, no exchange): what every node
 * does in the iterations between two exchanges when the communication period
 * tau of Algorithms 2-4 is larger than 1. */
int gsgd_step_local(gsgd_ctx* ctx, float* x, float* v, const float* g, void* stream);

/* Communication schedule of Algorithms 2-4 (an exchange opens every iteration
 * whose index is a positive multiple of the period tau).  The step calls here run the local step
 * first and the exchange after it, so the exchange of iteration t+1 is the
 * tail of step call t: returns 1 when step call number `step` (0-based) should
 * be an exchanging call, 0 when it should be gsgd_step_local, and
 * GSGD_ERR_INVALID_ARG for tau = 0.  Pure host code. */
int gsgd_comm_due(uint64_t step, uint32_t tau);

/* Elastic-averaging step, Algorithm 2 with communication period 1, all k
 * clients exchanging with the same centre value in one synchronous round:
 *   v_i <- momentum * v_i - lr_s * g_i;   x'_i = x_i + v_i;
 *   e_i = alpha_e * (x'_i - center);  x_i <- x'_i - e_i;  center <- center + sum_i e_i.
 * The sum runs in fp64 in ascending i.  center: device d, updated in place. */
int gsgd_step_easgd(gsgd_ctx* ctx, float* x, float* v, const float* g,
                    float* center, float alpha_e, void* stream);

/* Gossip step with the synthetic gradient generated on the fly (g never
 * touches memory): equivalent to gsgd_gen_grad followed by gsgd_step_gossip. */
int gsgd_step_gossip_fused(gsgd_ctx* ctx, float* x, float* v, const float* h, const float* xstar,
                           const int32_t* peer_perm, float beta, uint64_t step, void* stream);

/* The same for pull-gossip on an arbitrary peer map (fresh or stale parameters)
 * and for push-gossip: gsgd_gen_grad at `step` followed by gsgd_step_gossip_pull
 * / gsgd_step_gossip_push, with g never written to memory. */
int gsgd_step_gossip_pull_fused(gsgd_ctx* ctx, float* x, float* v, const float* h, const float* xstar,
                                const int32_t* peer, float beta, int stale, uint64_t step, void* stream);
int gsgd_step_gossip_push_fused(gsgd_ctx* ctx, float* x, float* v, const float* h, const float* xstar,
                                const int32_t* target, uint64_t step, void* stream);

/* Raw Philox4x32-10 output for counters (q, c1, c2, c3), q = 0..n_blocks-1,
 * under the context's key: out[4q .. 4q+3] are the four words of block q.
 * The generator is the one of Salmon, Moraes, Dror and Shaw (SC'11); this
 * entry point exists so that the device stream can be compared word for word.
 * out: device, 4 * n_blocks uint32. */
int gsgd_philox_raw(gsgd_ctx* ctx, uint32_t c1, uint32_t c2, uint32_t c3, int64_t n_blocks, uint32_t* out,
                    void* stream);

/* Measurement hook for the ALU side of the generator's roofline: `workgroups`
 * workgroups of 256 threads each draw `iters` Philox blocks per thread and turn
 * them into the context's kind of noise (the device functions gsgd_gen_grad and
 * the fused steps use), keeping everything in registers; thread t stores one
 * float to out[t].  Timed by the caller, it gives the generator's cost per
 * block of four values with no memory traffic in the way.
 * out: device, workgroups * 256 floats. */
int gsgd_noise_alu_probe(gsgd_ctx* ctx, int32_t workgroups, uint32_t iters, float* out, void* stream);

/* Uniformly random peer permutation for one step (the target choice of
 * Algorithms 3-4, with every node chosen once): Fisher-Yates from the top, driven
 * by Philox stream 5 at counter (i, 0, step, 5), index floor(r (i+1) / 2^32).
 * Pure host code, deterministic.  out: host, k entries. */
int gsgd_make_perm(uint64_t seed, uint64_t step, int32_t k, int32_t* out);

/* Independent uniform targets for one step (Section 3.1, j ~ Uniform over the
 * nodes): node i takes word 0 of Philox stream 5 at counter (i, 1, step, 5).
 *   exclude_self = 0: target floor(r k / 2^32), the node itself included
 *                     (pull-gossip; a self-target is a no-op mix);
 *   exclude_self = 1: a uniform draw among the k-1 other nodes (push-gossip sends to
 *                     a node other than itself), floor(r (k-1) / 2^32) stepped
 *                     over i; needs k >= 2.
 * Pure host code, deterministic.  out: host, k entries. */
int gsgd_make_targets(uint64_t seed, uint64_t step, int32_t k, int exclude_self, int32_t* out);

/* Visiting order of the pull-gossip kernel for an arbitrary peer map, exported
 * for tests.  walk[t] holds the replica index in its low 12 bits.  Replicas on
 * a cycle of the map carry bit 14 (first of its cycle) / bit 15 (last), as in
 * gsgd_perm_walk.  The others (bit 13 set) follow the cycle replica they hang
 * off, parents before children, and say how the kernel's parent register is
 * kept: bits 16..17 = 1 reload it from the last cycle replica, = 2 reload it
 * from stack slot bits 20..23; bit 12 = this replica becomes the parent of what
 * follows; bit 18 = the old parent is first saved to stack slot bits 20..23.
 * *slots_used = stack slots the walk needs (at most 8 for k <= GSGD_MAX_K).
 * Pure host code.  walk: host, k entries. */
int gsgd_pull_walk(const int32_t* peer, int32_t k, uint32_t* walk, int32_t* slots_used);

/* Visiting order of the push-gossip kernel, exported for tests: senders before
 * receivers.  walk[t]: replica in the low 12 bits; bits 22..31 = how many
 * values its average takes (1 + senders); bit 12 = the running sum holds its
 * senders' values; bit 13 = not on a cycle of the map, and then bits 16..17 say
 * how its own value joins its receiver's running sum (1 start it, 2 add, 3 add
 * to what stack slot bits 19..21 holds) and bit 18 that the running sum is
 * then parked in that slot; cycle replicas carry bits 14 / 15 (first / last of
 * the cycle, walked in the direction of sending).  *slots_used <= 8.
 * Pure host code.  walk: host, k entries. */
int gsgd_push_walk(const int32_t* target, int32_t k, uint32_t* walk, int32_t* slots_used);

/* Order in which the gossip kernel visits replicas: the cycles of peer_perm,
 * each walked i, perm[i], perm[perm[i]], ...  walk[t] holds the replica index
 * in its low 12 bits, bit 14 set on the first member of a cycle and bit 15 on
 * the last.  Pure host code (exported for tests).  walk: host, k entries.
 * Returns GSGD_ERR_BAD_PERM when peer_perm is not a bijection. */
int gsgd_perm_walk(const int32_t* peer_perm, int32_t k, uint16_t* walk);

/* The two quantities the analysis bounds (Section 6.1) and the mean's own
 * distance, over columns 0..d-1, accumulated in fp64:
 *   out[0] = sum_i ||x_i - xbar||^2, out[1] = sum_i ||x_i - xstar||^2,
 *   out[2] = ||xbar - xstar||^2,     out[3] = ||xbar||^2.
 * Waits for the stream.  out: host.
 * With the stream drained, the tile counter pair of that stream must read
 * zero; if it does not (a launch was cut short, or launches on different
 * streams were forced onto one pair by replaying a graph elsewhere), out is
 * still filled, the pair is cleared so that later launches visit every tile
 * again, and GSGD_ERR_BAD_STATE is returned: results of step calls since the
 * last clean check on this stream are suspect.  gsgd_row_sqnorms checks the
 * same way. */
int gsgd_stats(gsgd_ctx* ctx, const float* x, const float* xstar, double out[4], void* stream);

/* gsgd_stats for callers that cannot allocate or wait: code recorded into a
 * HIP graph, tight loops that must not call hipMalloc, harnesses that forbid
 * it.  Needs no context.  Computes the same four numbers with the same
 * kernels in the same order (bit-identical to gsgd_stats), writes them to
 * out_device (device memory, 4 doubles, 8-byte aligned, caller-owned) and
 * returns without waiting for the stream.  It calls no hipMalloc / hipFree and
 * nothing else that allocates: the partial sums of the pass (one set per
 * workgroup, at most 2048 sets = 64 KiB) go to a fixed array in device memory
 * that the library holds on every GPU it runs on until the process ends.  The
 * entry point is specified for
 *   d <= GSGD_STATS_STATIC_MAX_D columns;
 * a larger d is refused with GSGD_ERR_TOO_LARGE.  All calls on one GPU share
 * that array: calls that overlap in time on one GPU (different streams, or a
 * graph replaying beside eager calls) race on it and give garbage; calls that
 * follow one another on a stream are fine, whatever their sizes (every partial
 * a call reads it has written itself).  The array's device address is looked
 * up on the first call on a device (and by gsgd_create); make that first call
 * outside a stream capture.  k, d, ld, block_columns as in gsgd_config (there is
 * no context to take the layout from).  x: device k x ld.  xstar: device d. */
#define GSGD_STATS_STATIC_MAX_D ((int64_t)1 << 26)
int gsgd_stats_static(int32_t k, int64_t d, int64_t ld, int64_t block_columns, const float* x, const float* xstar,
                      double* out_device, void* stream);

/* Squared Euclidean norm of every replica row over columns 0..d-1, in fp64:
 * out[i] = ||x_i||^2.  Waits for the stream.  out: host, k doubles. */
int gsgd_row_sqnorms(gsgd_ctx* ctx, const float* x, double* out, void* stream);

/* The diffusion potential of Section 3.1.  Under rounds of gossip alone (no
 * gradient steps) every node's parameters stay a weighted average of the
 * starting ones, theta_i(r) = sum_j v_ij theta_j(0), and
 *   Phi = sum_i sum_j || v_ij theta_j(0) - (1/p) sum_j' v_ij' theta_j'(0) ||^2
 *       = sum_i [ sum_j v_ij^2 ||theta_j(0)||^2 - (1/p) ||theta_i(r)||^2 ].
 * V is the k x k row-major matrix of the v_ij, the identity before the first
 * round; gsgd_weights_pull / gsgd_weights_push advance it by one round of
 * pull-gossip (v_i <- v_i - beta (v_i - v_peer[i])) or push-gossip (v_r <-
 * average of v_r and the v_i sent to r), the same maps the step calls take.
 * gsgd_diffusion_potential evaluates the second form from the row norms at the
 * start (sqnorm_start) and now (sqnorm_now), both from gsgd_row_sqnorms.
 * All three are pure host code; V, the norms and out are host memory. */
int gsgd_weights_pull(double* V, int32_t k, const int32_t* peer, double beta);
int gsgd_weights_push(double* V, int32_t k, const int32_t* target);
int gsgd_diffusion_potential(const double* V, int32_t k, const double* sqnorm_start, const double* sqnorm_now,
                             double* out);

/* Test hook: set the tile counter pair of `stream` to (next_tile, finished)
 * once the stream has drained.  (0, 0) is the only state step calls may start
 * from; anything else makes the next gsgd_stats on that stream report
 * GSGD_ERR_BAD_STATE. */
int gsgd_poke_tickets(gsgd_ctx* ctx, uint32_t next_tile, uint32_t finished, void* stream);

const char* gsgd_strerror(int code);
int gsgd_last_hip_error(const gsgd_ctx* ctx);   /* raw hipError_t of the last GSGD_ERR_HIP */

#ifdef __cplusplus
}
#endif
#endif /* GSGD_H */

// The aggregation-step kernels: gossip in its pull, push and stale-parameter
// forms (Section 3.1, Algorithms 3-4, Section 6.2 of the paper), all-reduce
// average (Algorithm 1), elastic averaging (Algorithm 2), and the local step
// alone.
//
// Every exchanging rule couples only the k values of one column, so a thread owns four
// adjacent columns (one 128-bit lane) of all k replica rows and walks the rows.
// A wavefront reads or writes 1 KiB contiguous per access; x, v and g are each
// read once and x, v written once: 20 bytes per replica-element, the minimum.
//
// The order the rows are visited in is what the memory system feels.  On
// row-major matrices (rows tens of MB apart) it does not matter, and gossip
// follows the peer map so that values can be handed from row to row in
// registers (gossip_step_kernel, push_step_kernel).  On blocked matrices the
// k row pieces of a tile are neighbours, ascending order is address order, and
// every kernel visits them that way: gossip in two sweeps with the values a
// mix needs parked in LDS (gossip_sweep_kernel, push_sweep_kernel, in
// kernels_sweep.hip), the local step as a row walk (local_walk_kernel);
// all-reduce and elastic averaging sum in ascending order anyway.
//
// Rows are fetched in batches of U: all loads of a batch are issued before the
// first dependent instruction, the batch loop has no conditionals around the
// loads (the k % U leftover rows run through a batch of one; in the sweeps
// through batches of 4, 2 and 1), and the row order comes from scalar
// registers, so nothing waits on the vector-memory counter except the uses
// of the loaded rows themselves.
#include "device_common.hpp"

namespace gsgd {

#ifndef GSGD_ROWS_IN_FLIGHT
#define GSGD_ROWS_IN_FLIGHT 4
#endif
#ifndef GSGD_WALK_ROWS_IN_FLIGHT
#define GSGD_WALK_ROWS_IN_FLIGHT 3
#endif

// ---------------------------------------------------------------------------
// Gossip.  x_new[i] needs the post-step parameters of replica i and of its
// peer.  Rows are visited along the cycles of the peer map,
// i -> peer[i] -> peer[peer[i]] ..., so the peer of the row visited last time
// is the row visited now: keeping `first`, `prev` and the current x' in
// registers is enough to finish every row in place, in one pass, without a
// second buffer and without two replicas ever racing on a row.
//
// What a row contributes to the mix of the row pulling from it is called its
// "key" below: x' for the fresh-parameter rule of Sections 3.1 / 6.2.2, and
// the x from before the local step for the stale-parameter rule of Section
// 6.2.1 (STALE), x_i <- x'_i - beta (x_i - x_peer).
//
// TREE: the peer map is not a bijection (iid pull targets).  Rows that are on
// no cycle follow the cycle row they hang off, parents before children; each
// is finished as soon as it is loaded, against its parent's key, which the
// walk keeps in `par` (see the WALK_* flags) with an LDS stack lane per thread
// for the few keys that must outlive a sibling subtree.
typedef f32x4 KeyStack[WALK_SLOTS][BLOCK];

template <bool FULL, int U, bool FUSED_GEN, int NOISE, bool EXT, bool STALE, bool TREE>
__device__ __forceinline__
void gossip_step_body(const Geom& geo, const Hyper& hp, const SegTable& seg, const SegLds& lds, const Quad& qd,
                      float neg_beta, const Walk& walk, KeyStack* stack,
                      float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                      const float* __restrict__ h, const float* __restrict__ xstar,
                      float sigma, RngKey key, uint32_t step)
{
    const int valid = FULL ? 4 : qd.valid;
    const f32x4 neg_lr = -quad_lr(seg, lds, qd.col, valid, hp.lr);
    f32x4 h4 = {0.f, 0.f, 0.f, 0.f}, xs4 = {0.f, 0.f, 0.f, 0.f};
    if constexpr (FUSED_GEN) {
        h4 = load_quad_cached<FULL>(h + qd.col, valid);
        xs4 = load_quad_cached<FULL>(xstar + qd.col, valid);
    }
    const uint32_t quad_index = static_cast<uint32_t>(qd.col >> 2);

    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    f32x4 first_key = zero, prev_key = zero, prev_post = zero, par = zero;
    int64_t prev_off = 0;                      // uniform: row offset of the cycle row visited last

    for_row_batches<U>(geo.k, [&](auto n, int t0) {
        constexpr int N = decltype(n)::value;
        f32x4 X[N], V[N], G[N];
        uint32_t w[N];
#pragma unroll
        for (int u = 0; u < N; ++u) {
            w[u] = walk.seq[t0 + u];
            const int64_t off = static_cast<int64_t>(w[u] & WALK_ROW_MASK) * geo.rs + qd.mat;
            X[u] = load_quad<FULL>(x + off + qd.lane_col, valid);
            V[u] = load_quad<FULL>(v + off + qd.lane_col, valid);
            if constexpr (!FUSED_GEN) G[u] = load_quad<FULL>(g + off + qd.lane_col, valid);
        }
#pragma unroll
        for (int u = 0; u < N; ++u) {
            const uint32_t row = w[u] & WALK_ROW_MASK;
            const int64_t off = static_cast<int64_t>(row) * geo.rs + qd.mat;
            if constexpr (FUSED_GEN) {
                const f32x4 xi = noise4<NOISE>(philox4x32_10(quad_index, row, step, STREAM_GRAD, key.k0, key.k1));
                const f32x4 t1 = X[u] - xs4;
                const f32x4 t2 = sigma * xi;
                G[u] = fma4(h4, t1, t2);
            }
            f32x4 vn, post;
            local_step<EXT>(X[u], V[u], G[u], neg_lr, hp, vn, post);
            store_quad<FULL>(v + off + qd.lane_col, vn, valid);
            const f32x4 mine = STALE ? X[u] : post;
            if (TREE && (w[u] & WALK_TREE)) {
                const uint32_t slot = (w[u] & WALK_SLOT_MASK) >> WALK_SLOT_SHIFT;
                const uint32_t restore = w[u] & WALK_RESTORE_MASK;
                if (restore == WALK_RESTORE_PREV) par = prev_key;
                else if (restore == WALK_RESTORE_SLOT) par = (*stack)[slot][threadIdx.x];
                store_quad<FULL>(x + off + qd.lane_col, mix_keys(post, mine, par, neg_beta), valid);
                if (w[u] & WALK_SAVE) (*stack)[slot][threadIdx.x] = par;
                if (w[u] & WALK_DESCEND) par = mine;
            } else {
                if (w[u] & WALK_FIRST) first_key = mine;
                else store_quad<FULL>(x + prev_off + qd.lane_col, mix_keys(prev_post, prev_key, mine, neg_beta), valid);
                if (w[u] & WALK_LAST)
                    store_quad<FULL>(x + off + qd.lane_col, mix_keys(post, mine, first_key, neg_beta), valid);
                prev_key = mine;
                prev_post = post;
                prev_off = off;
            }
        }
    });
}

template <int U, bool FUSED_GEN, int NOISE, bool EXT = false, bool STALE = false, bool TREE = false>
__global__ __launch_bounds__(BLOCK)
void gossip_step_kernel(Geom geo, Hyper hp, SegTable seg, float neg_beta, Walk walk,
                        float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                        const float* __restrict__ h, const float* __restrict__ xstar,
                        float sigma, RngKey key, uint32_t step, Persist pst, uint32_t n_tiles)
{
    __shared__ SegLds lds;
    __shared__ f32x4 stack_mem[TREE ? WALK_SLOTS : 1][TREE ? BLOCK : 1];
    KeyStack* stack = reinterpret_cast<KeyStack*>(&stack_mem[0][0]);     // only dereferenced when TREE
    stage_segments(seg, lds);
    for_each_tile(pst, n_tiles, [&](uint32_t tile) {
        const Quad qd = quad_of_tile(tile, geo);
        if (tile_is_full(qd, geo.d))
            gossip_step_body<true, U, FUSED_GEN, NOISE, EXT, STALE, TREE>(geo, hp, seg, lds, qd, neg_beta, walk, stack,
                                                                          x, v, g, h, xstar, sigma, key, step);
        else if (qd.valid > 0)
            gossip_step_body<false, U, FUSED_GEN, NOISE, EXT, STALE, TREE>(geo, hp, seg, lds, qd, neg_beta, walk, stack,
                                                                           x, v, g, h, xstar, sigma, key, step);
    });
}

// ---------------------------------------------------------------------------
// Push-gossip (Algorithm 4): every node sends x' to itself and to its target;
// a node's new parameters are the average of what it received.  Rows are
// visited senders first (see build_push_walk), so when a row is loaded the
// fp64 sum of everything sent to it through tree edges is in `acc`; the x' of
// a cycle row's cycle predecessor rides in `prev`, and the first row of a
// cycle waits in `first_sum` for the last.  One in-place pass, as for pull.
typedef f64x4 SumStack[WALK_SLOTS][BLOCK];

template <bool FULL, int U, bool EXT, bool FUSED_GEN, int NOISE>
__device__ __forceinline__
void push_step_body(const Geom& geo, const Hyper& hp, const SegTable& seg, const SegLds& lds, const Quad& qd,
                    const Walk& walk, SumStack* stack,
                    float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                    const float* __restrict__ h, const float* __restrict__ xstar,
                    float sigma, RngKey key, uint32_t step)
{
    const int valid = FULL ? 4 : qd.valid;
    const f32x4 neg_lr = -quad_lr(seg, lds, qd.col, valid, hp.lr);
    f32x4 h4 = {0.f, 0.f, 0.f, 0.f}, xs4 = {0.f, 0.f, 0.f, 0.f};
    if constexpr (FUSED_GEN) {
        h4 = load_quad_cached<FULL>(h + qd.col, valid);
        xs4 = load_quad_cached<FULL>(xstar + qd.col, valid);
    }
    const uint32_t quad_index = static_cast<uint32_t>(qd.col >> 2);

    f64x4 acc = {0.0, 0.0, 0.0, 0.0}, first_sum = {0.0, 0.0, 0.0, 0.0};
    f32x4 prev = {0.f, 0.f, 0.f, 0.f};
    uint32_t first_count = 1;                  // uniform
    int64_t first_off = 0;                     // uniform

    for_row_batches<U>(geo.k, [&](auto n, int t0) {
        constexpr int N = decltype(n)::value;
        f32x4 X[N], V[N], G[N];
        uint32_t w[N];
#pragma unroll
        for (int u = 0; u < N; ++u) {
            w[u] = walk.seq[t0 + u];
            const int64_t off = static_cast<int64_t>(w[u] & WALK_ROW_MASK) * geo.rs + qd.mat;
            X[u] = load_quad<FULL>(x + off + qd.lane_col, valid);
            V[u] = load_quad<FULL>(v + off + qd.lane_col, valid);
            if constexpr (!FUSED_GEN) G[u] = load_quad<FULL>(g + off + qd.lane_col, valid);
        }
#pragma unroll
        for (int u = 0; u < N; ++u) {
            const uint32_t row = w[u] & WALK_ROW_MASK;
            const int64_t off = static_cast<int64_t>(row) * geo.rs + qd.mat;
            const uint32_t count = w[u] >> PUSH_COUNT_SHIFT;
            const uint32_t slot = (w[u] & PUSH_SLOT_MASK) >> PUSH_SLOT_SHIFT;
            if constexpr (FUSED_GEN) {
                const f32x4 xi = noise4<NOISE>(philox4x32_10(quad_index, row, step, STREAM_GRAD, key.k0, key.k1));
                const f32x4 t1 = X[u] - xs4;
                const f32x4 t2 = sigma * xi;
                G[u] = fma4(h4, t1, t2);
            }
            f32x4 vn, post;
            local_step<EXT>(X[u], V[u], G[u], neg_lr, hp, vn, post);
            store_quad<FULL>(v + off + qd.lane_col, vn, valid);
            const f64x4 post64 = widen(post);
            f64x4 sum = post64;
            if (w[u] & PUSH_HAS_SENDERS) sum = acc + post64;
            if (w[u] & WALK_TREE) {
                store_quad<FULL>(x + off + qd.lane_col, count == 1 ? post : average(sum, count), valid);
                const uint32_t mode = w[u] & PUSH_MODE_MASK;
                if (mode == PUSH_START) acc = post64;
                else if (mode == PUSH_ADD) acc = acc + post64;
                else acc = (*stack)[slot][threadIdx.x] + post64;
                if (w[u] & PUSH_SAVE_AFTER) (*stack)[slot][threadIdx.x] = acc;
            } else if (w[u] & WALK_FIRST) {
                if (w[u] & WALK_LAST) {        // a node that sends to nobody but itself
                    store_quad<FULL>(x + off + qd.lane_col, count == 1 ? post : average(sum, count), valid);
                } else {
                    first_sum = sum;
                    first_count = count;
                    first_off = off;
                }
                prev = post;
            } else {
                store_quad<FULL>(x + off + qd.lane_col, average(sum + widen(prev), count), valid);
                if (w[u] & WALK_LAST)
                    store_quad<FULL>(x + first_off + qd.lane_col, average(first_sum + post64, first_count), valid);
                prev = post;
            }
        }
    });
}

template <int U, bool EXT, bool FUSED_GEN = false, int NOISE = 0>
__global__ __launch_bounds__(BLOCK)
void push_step_kernel(Geom geo, Hyper hp, SegTable seg, Walk walk,
                      float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                      const float* __restrict__ h, const float* __restrict__ xstar,
                      float sigma, RngKey key, uint32_t step, Persist pst, uint32_t n_tiles)
{
    __shared__ SegLds lds;
    __shared__ SumStack stack;
    stage_segments(seg, lds);
    for_each_tile(pst, n_tiles, [&](uint32_t tile) {
        const Quad qd = quad_of_tile(tile, geo);
        if (tile_is_full(qd, geo.d))
            push_step_body<true, U, EXT, FUSED_GEN, NOISE>(geo, hp, seg, lds, qd, walk, &stack, x, v, g, h, xstar, sigma,
                                                           key, step);
        else if (qd.valid > 0)
            push_step_body<false, U, EXT, FUSED_GEN, NOISE>(geo, hp, seg, lds, qd, walk, &stack, x, v, g, h, xstar, sigma,
                                                            key, step);
    });
}

// ---------------------------------------------------------------------------
// All-reduce average (Algorithm 1).  Pass 1 reads v and g of every row and
// accumulates u_i = mu v_i - lr g_i in fp64 in ascending i; pass 2 adds the
// rounded mean to every row of x and leaves it in every row of v.
// EXT (weight decay / Nesterov, Section 4.2): the momentum buffers and the
// applied updates are averaged separately (they differ under Nesterov), and
// pass 1 also reads x when the weight decay is non-zero.
template <bool FULL, int U, bool EXT>
__device__ __forceinline__
void allreduce_step_body(const Geom& geo, const Hyper& hp, const SegTable& seg, const SegLds& lds, const Quad& qd,
                         float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g)
{
    const int valid = FULL ? 4 : qd.valid;
    const f32x4 neg_lr = -quad_lr(seg, lds, qd.col, valid, hp.lr);
    const int k = geo.k;
    const bool need_x = EXT && hp.wd != 0.0f;       // uniform
    const bool nesterov = EXT && hp.nesterov != 0;   // uniform

    f64x4 acc_v = {0.0, 0.0, 0.0, 0.0}, acc_d = {0.0, 0.0, 0.0, 0.0};
    for_row_batches<2 * U>(k, [&](auto n, int i0) {
        constexpr int N = decltype(n)::value;
        f32x4 X[N], V[N], G[N];
#pragma unroll
        for (int u = 0; u < N; ++u) {
            const int64_t off = static_cast<int64_t>(i0 + u) * geo.rs + qd.mat;
            V[u] = load_quad<FULL>(v + off + qd.lane_col, valid);
            G[u] = load_quad<FULL>(g + off + qd.lane_col, valid);
            X[u] = f32x4{0.f, 0.f, 0.f, 0.f};
            if constexpr (EXT) { if (need_x) X[u] = load_quad_cached<FULL>(x + off + qd.lane_col, valid); }
        }
#pragma unroll
        for (int u = 0; u < N; ++u) {
            f32x4 un, xp_unused, gt;
            local_step<EXT>(X[u], V[u], G[u], neg_lr, hp, un, xp_unused, &gt);
            acc_v.x += static_cast<double>(un.x);
            acc_v.y += static_cast<double>(un.y);
            acc_v.z += static_cast<double>(un.z);
            acc_v.w += static_cast<double>(un.w);
            if constexpr (EXT) {
                if (nesterov) {
                    const f32x4 t5 = hp.mu * un;
                    const f32x4 di = fma4(neg_lr, gt, t5);
                    acc_d.x += static_cast<double>(di.x);
                    acc_d.y += static_cast<double>(di.y);
                    acc_d.z += static_cast<double>(di.z);
                    acc_d.w += static_cast<double>(di.w);
                }
            }
        }
    });
    const double kd = static_cast<double>(k);
    const f32x4 ubar = {static_cast<float>(acc_v.x / kd), static_cast<float>(acc_v.y / kd),
                        static_cast<float>(acc_v.z / kd), static_cast<float>(acc_v.w / kd)};
    f32x4 dbar = ubar;
    if constexpr (EXT) {
        if (nesterov)
            dbar = f32x4{static_cast<float>(acc_d.x / kd), static_cast<float>(acc_d.y / kd),
                         static_cast<float>(acc_d.z / kd), static_cast<float>(acc_d.w / kd)};
    }
    for_row_batches<2 * U>(k, [&](auto n, int i0) {
        constexpr int N = decltype(n)::value;
        f32x4 X[N];
#pragma unroll
        for (int u = 0; u < N; ++u)
            X[u] = load_quad<FULL>(x + static_cast<int64_t>(i0 + u) * geo.rs + qd.mat + qd.lane_col, valid);
#pragma unroll
        for (int u = 0; u < N; ++u) {
            const int64_t off = static_cast<int64_t>(i0 + u) * geo.rs + qd.mat;
            store_quad<FULL>(v + off + qd.lane_col, ubar, valid);
            store_quad<FULL>(x + off + qd.lane_col, X[u] + dbar, valid);
        }
    });
}

template <int U, bool EXT = false>
__global__ __launch_bounds__(BLOCK)
void allreduce_step_kernel(Geom geo, Hyper hp, SegTable seg,
                           float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                           Persist pst, uint32_t n_tiles)
{
    __shared__ SegLds lds;
    stage_segments(seg, lds);
    for_each_tile(pst, n_tiles, [&](uint32_t tile) {
        const Quad qd = quad_of_tile(tile, geo);
        if (tile_is_full(qd, geo.d)) allreduce_step_body<true, U, EXT>(geo, hp, seg, lds, qd, x, v, g);
        else if (qd.valid > 0) allreduce_step_body<false, U, EXT>(geo, hp, seg, lds, qd, x, v, g);
    });
}

// ---------------------------------------------------------------------------
// Elastic averaging (Algorithm 2, period 1, one synchronous round):
// every client moves towards the same centre value, the centre moves by the
// sum of what the clients gave up.
template <bool FULL, int U, bool EXT>
__device__ __forceinline__
void easgd_step_body(const Geom& geo, const Hyper& hp, const SegTable& seg, const SegLds& lds, const Quad& qd,
                     float alpha_e, float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                     float* __restrict__ center)
{
    const int valid = FULL ? 4 : qd.valid;
    const f32x4 neg_lr = -quad_lr(seg, lds, qd.col, valid, hp.lr);
    const f32x4 c4 = load_quad_cached<FULL>(center + qd.col, valid);

    f64x4 acc = {0.0, 0.0, 0.0, 0.0};
    for_row_batches<U>(geo.k, [&](auto n, int i0) {
        constexpr int N = decltype(n)::value;
        f32x4 X[N], V[N], G[N];
#pragma unroll
        for (int u = 0; u < N; ++u) {
            const int64_t off = static_cast<int64_t>(i0 + u) * geo.rs + qd.mat;
            X[u] = load_quad<FULL>(x + off + qd.lane_col, valid);
            V[u] = load_quad<FULL>(v + off + qd.lane_col, valid);
            G[u] = load_quad<FULL>(g + off + qd.lane_col, valid);
        }
#pragma unroll
        for (int u = 0; u < N; ++u) {
            const int64_t off = static_cast<int64_t>(i0 + u) * geo.rs + qd.mat;
            f32x4 vn, xp;
            local_step<EXT>(X[u], V[u], G[u], neg_lr, hp, vn, xp);
            const f32x4 e = alpha_e * (xp - c4);
            store_quad<FULL>(v + off + qd.lane_col, vn, valid);
            store_quad<FULL>(x + off + qd.lane_col, xp - e, valid);
            acc.x += static_cast<double>(e.x);
            acc.y += static_cast<double>(e.y);
            acc.z += static_cast<double>(e.z);
            acc.w += static_cast<double>(e.w);
        }
    });
    const f32x4 cn = {static_cast<float>(static_cast<double>(c4.x) + acc.x),
                      static_cast<float>(static_cast<double>(c4.y) + acc.y),
                      static_cast<float>(static_cast<double>(c4.z) + acc.z),
                      static_cast<float>(static_cast<double>(c4.w) + acc.w)};
    store_quad<FULL>(center + qd.col, cn, valid);
}

template <int U, bool EXT = false>
__global__ __launch_bounds__(BLOCK)
void easgd_step_kernel(Geom geo, Hyper hp, SegTable seg, float alpha_e,
                       float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                       float* __restrict__ center, Persist pst, uint32_t n_tiles)
{
    __shared__ SegLds lds;
    stage_segments(seg, lds);
    for_each_tile(pst, n_tiles, [&](uint32_t tile) {
        const Quad qd = quad_of_tile(tile, geo);
        if (tile_is_full(qd, geo.d)) easgd_step_body<true, U, EXT>(geo, hp, seg, lds, qd, alpha_e, x, v, g, center);
        else if (qd.valid > 0) easgd_step_body<false, U, EXT>(geo, hp, seg, lds, qd, alpha_e, x, v, g, center);
    });
}

// ---------------------------------------------------------------------------
// The k-way sums with the rows split over the wavefronts of a workgroup, for vectors too short to fill the chip
// with one thread per four columns walking all k rows (fewer 1024-column tiles than compute units).  A workgroup of
// WAVES wavefronts owns a tile of 64 quads (256 columns); wavefront w takes the w-th block of ceil(k / WAVES)
// consecutive rows, accumulates its part of the sum in fp64 in ascending row order and parks it in LDS; after one
// barrier every wavefront adds the WAVES partial sums in ascending w and finishes its own rows.  The chip sees 4 x
// as many workgroups and WAVES x as many rows in flight per column, which is what a latency-bound walk needs.
// The sum is the same set of fp64 additions associated differently ((rows of wave 0) + (rows of wave 1) + ...
// instead of one ascending chain), so a result can differ from the serial kernels' in the last place where the fp64
// sum is itself inexact; everything else (local step, per-row updates) is the same arithmetic.
constexpr int SPLIT_QUADS = 64;                    // quads (lanes) per tile: one wavefront wide
constexpr int SPLIT_COLUMNS = SPLIT_QUADS * 4;

__device__ __forceinline__ void store_quad_cached(float* p, f32x4 r, int valid)
{
    if (valid == 4) { *reinterpret_cast<f32x4*>(p) = r; return; }
    if (valid > 0) p[0] = r.x;
    if (valid > 1) p[1] = r.y;
    if (valid > 2) p[2] = r.z;
}

__device__ __forceinline__ void add_into(f64x4& acc, f32x4 a)
{
    acc.x += static_cast<double>(a.x);
    acc.y += static_cast<double>(a.y);
    acc.z += static_cast<double>(a.z);
    acc.w += static_cast<double>(a.w);
}

template <int WAVES, bool EXT>
__global__ __launch_bounds__(WAVES * 64)
void allreduce_rowsplit_kernel(Geom geo, Hyper hp, SegTable seg,
                               float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g)
{
    __shared__ SegLds lds;
    __shared__ f64x4 part_v[WAVES][SPLIT_QUADS];
    __shared__ f64x4 part_d[EXT ? WAVES : 1][EXT ? SPLIT_QUADS : 1];
    stage_segments(seg, lds);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t col = static_cast<int64_t>(blockIdx.x) * SPLIT_COLUMNS + lane * 4;
    const int64_t mcol = column_origin(geo, col);       // a quad never straddles a block
    const int64_t left = geo.d - col;
    const int valid = left >= 4 ? 4 : (left > 0 ? static_cast<int>(left) : 0);
    const int k = geo.k;
    const int rows_per_wave = (k + WAVES - 1) / WAVES;
    const int r0 = wave * rows_per_wave < k ? wave * rows_per_wave : k;
    const int r1 = r0 + rows_per_wave < k ? r0 + rows_per_wave : k;
    const bool need_x = EXT && hp.wd != 0.0f;
    const bool nesterov = EXT && hp.nesterov != 0;
    const f32x4 neg_lr = valid > 0 ? -quad_lr(seg, lds, col, valid, hp.lr) : f32x4{0.f, 0.f, 0.f, 0.f};

    f64x4 acc_v = {0.0, 0.0, 0.0, 0.0}, acc_d = {0.0, 0.0, 0.0, 0.0};
    if (valid > 0) {
        for (int i = r0; i < r1; ++i) {
            const int64_t off = static_cast<int64_t>(i) * geo.rs + mcol;
            const f32x4 V = load_quad_cached(v + off, valid);
            const f32x4 G = load_quad_cached(g + off, valid);
            f32x4 X = {0.f, 0.f, 0.f, 0.f};
            if constexpr (EXT) { if (need_x) X = load_quad_cached(x + off, valid); }
            f32x4 un, xp_unused, gt;
            local_step<EXT>(X, V, G, neg_lr, hp, un, xp_unused, &gt);
            add_into(acc_v, un);
            if constexpr (EXT) {
                if (nesterov) {
                    const f32x4 t5 = hp.mu * un;
                    add_into(acc_d, fma4(neg_lr, gt, t5));
                }
            }
        }
    }
    part_v[wave][lane] = acc_v;
    if constexpr (EXT) part_d[wave][lane] = acc_d;
    __syncthreads();
    if (valid == 0) return;
    f64x4 sum_v = part_v[0][lane];
    for (int w = 1; w < WAVES; ++w) sum_v += part_v[w][lane];
    const double kd = static_cast<double>(k);
    const f32x4 ubar = {static_cast<float>(sum_v.x / kd), static_cast<float>(sum_v.y / kd),
                        static_cast<float>(sum_v.z / kd), static_cast<float>(sum_v.w / kd)};
    f32x4 dbar = ubar;
    if constexpr (EXT) {
        if (nesterov) {
            f64x4 sum_d = part_d[0][lane];
            for (int w = 1; w < WAVES; ++w) sum_d += part_d[w][lane];
            dbar = f32x4{static_cast<float>(sum_d.x / kd), static_cast<float>(sum_d.y / kd),
                         static_cast<float>(sum_d.z / kd), static_cast<float>(sum_d.w / kd)};
        }
    }
    for (int i = r0; i < r1; ++i) {
        const int64_t off = static_cast<int64_t>(i) * geo.rs + mcol;
        const f32x4 X = load_quad_cached(x + off, valid);
        store_quad_cached(v + off, ubar, valid);
        store_quad_cached(x + off, X + dbar, valid);
    }
}

template <int WAVES, bool EXT>
__global__ __launch_bounds__(WAVES * 64)
void easgd_rowsplit_kernel(Geom geo, Hyper hp, SegTable seg, float alpha_e,
                           float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                           float* __restrict__ center)
{
    __shared__ SegLds lds;
    __shared__ f64x4 part[WAVES][SPLIT_QUADS];
    stage_segments(seg, lds);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t col = static_cast<int64_t>(blockIdx.x) * SPLIT_COLUMNS + lane * 4;
    const int64_t mcol = column_origin(geo, col);       // a quad never straddles a block
    const int64_t left = geo.d - col;
    const int valid = left >= 4 ? 4 : (left > 0 ? static_cast<int>(left) : 0);
    const int k = geo.k;
    const int rows_per_wave = (k + WAVES - 1) / WAVES;
    const int r0 = wave * rows_per_wave < k ? wave * rows_per_wave : k;
    const int r1 = r0 + rows_per_wave < k ? r0 + rows_per_wave : k;

    f64x4 acc = {0.0, 0.0, 0.0, 0.0};
    f32x4 c4 = {0.f, 0.f, 0.f, 0.f};
    if (valid > 0) {
        const f32x4 neg_lr = -quad_lr(seg, lds, col, valid, hp.lr);
        c4 = load_quad_cached(center + col, valid);
        for (int i = r0; i < r1; ++i) {
            const int64_t off = static_cast<int64_t>(i) * geo.rs + mcol;
            const f32x4 X = load_quad_cached(x + off, valid);
            const f32x4 V = load_quad_cached(v + off, valid);
            const f32x4 G = load_quad_cached(g + off, valid);
            f32x4 vn, xp;
            local_step<EXT>(X, V, G, neg_lr, hp, vn, xp);
            const f32x4 e = alpha_e * (xp - c4);
            store_quad_cached(v + off, vn, valid);
            store_quad_cached(x + off, xp - e, valid);
            add_into(acc, e);
        }
    }
    part[wave][lane] = acc;
    __syncthreads();                                  // also orders every wave's read of the centre before its update
    if (valid == 0 || wave != 0) return;
    f64x4 sum = part[0][lane];
    for (int w = 1; w < WAVES; ++w) sum += part[w][lane];
    const f32x4 cn = {static_cast<float>(static_cast<double>(c4.x) + sum.x),
                      static_cast<float>(static_cast<double>(c4.y) + sum.y),
                      static_cast<float>(static_cast<double>(c4.z) + sum.z),
                      static_cast<float>(static_cast<double>(c4.w) + sum.w)};
    store_quad_cached(center + col, cn, valid);
}

// ---------------------------------------------------------------------------
// Local step alone: what a node does in the iterations between two exchanges
// when the communication period tau of Algorithms 2-4 is larger than 1.
// Nothing couples the rows here, so this is a flat kernel: one workgroup per
// (tile, replica), dispatched row by row, each row streamed once front to
// back.  On MI355X that access order sustains about 79 % of the HBM peak where
// the k-rows-per-tile walk of the coupled rules reaches 72 %.  The per-layer
// table is searched in global memory (it is small and stays in L2); staging
// it in LDS per workgroup would cost as much as the tile itself.
template <bool FULL, bool EXT>
__device__ __forceinline__
void local_step_body(const Geom& geo, const Hyper& hp, const SegTable& seg, const Quad& qd, int row,
                     float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g)
{
    const int valid = FULL ? 4 : qd.valid;
    const int64_t off = static_cast<int64_t>(row) * geo.rs + qd.mat;
    const f32x4 X = load_quad<FULL>(x + off + qd.lane_col, valid);
    const f32x4 V = load_quad<FULL>(v + off + qd.lane_col, valid);
    const f32x4 G = load_quad<FULL>(g + off + qd.lane_col, valid);
    f32x4 lr4 = {hp.lr, hp.lr, hp.lr, hp.lr};
    if (seg.n_seg > 0) lr4 = seg_lookup(seg.offsets, seg.scales, seg.n_seg, qd.col, valid, hp.lr);
    f32x4 vn, xp;
    local_step<EXT>(X, V, G, -lr4, hp, vn, xp);
    store_quad<FULL>(v + off + qd.lane_col, vn, valid);
    store_quad<FULL>(x + off + qd.lane_col, xp, valid);
}

template <bool EXT>
__global__ __launch_bounds__(BLOCK)
void local_step_kernel(Geom geo, Hyper hp, SegTable seg,
                       float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                       uint32_t band_tiles, uint32_t n_tiles)
{
    const uint32_t tile = blockIdx.z * band_tiles + blockIdx.x;
    if (tile >= n_tiles) return;
    const Quad qd = quad_of_tile(tile, geo);
    const int row = static_cast<int>(blockIdx.y);
    if (tile_is_full(qd, geo.d)) local_step_body<true, EXT>(geo, hp, seg, qd, row, x, v, g);
    else if (qd.valid > 0) local_step_body<false, EXT>(geo, hp, seg, qd, row, x, v, g);
}

// The local step as persistent workgroups that walk the k rows of a tile in ascending order: the form for blocked
// matrices, where that order is the address order of a block (the plain grid above is the form for row-major ones).
template <bool FULL, int U, bool EXT>
__device__ __forceinline__
void local_walk_body(const Geom& geo, const Hyper& hp, const SegTable& seg, const SegLds& lds, const Quad& qd,
                     float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g)
{
    const int valid = FULL ? 4 : qd.valid;
    const f32x4 neg_lr = -quad_lr(seg, lds, qd.col, valid, hp.lr);
    for_row_batches<U>(geo.k, [&](auto n, int i0) {
        constexpr int N = decltype(n)::value;
        f32x4 X[N], V[N], G[N];
#pragma unroll
        for (int u = 0; u < N; ++u) {
            const int64_t off = static_cast<int64_t>(i0 + u) * geo.rs + qd.mat;
            X[u] = load_quad<FULL>(x + off + qd.lane_col, valid);
            V[u] = load_quad<FULL>(v + off + qd.lane_col, valid);
            G[u] = load_quad<FULL>(g + off + qd.lane_col, valid);
        }
#pragma unroll
        for (int u = 0; u < N; ++u) {
            const int64_t off = static_cast<int64_t>(i0 + u) * geo.rs + qd.mat;
            f32x4 vn, xp;
            local_step<EXT>(X[u], V[u], G[u], neg_lr, hp, vn, xp);
            store_quad<FULL>(v + off + qd.lane_col, vn, valid);
            store_quad<FULL>(x + off + qd.lane_col, xp, valid);
        }
    });
}

template <int U, bool EXT>
__global__ __launch_bounds__(BLOCK)
void local_walk_kernel(Geom geo, Hyper hp, SegTable seg,
                       float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                       Persist pst, uint32_t n_tiles)
{
    __shared__ SegLds lds;
    stage_segments(seg, lds);
    for_each_tile(pst, n_tiles, [&](uint32_t tile) {
        const Quad qd = quad_of_tile(tile, geo);
        if (tile_is_full(qd, geo.d)) local_walk_body<true, U, EXT>(geo, hp, seg, lds, qd, x, v, g);
        else if (qd.valid > 0) local_walk_body<false, U, EXT>(geo, hp, seg, lds, qd, x, v, g);
    });
}

// ---------------------------------------------------------------------------
#ifndef GSGD_NO_LAUNCHERS
constexpr int RIF = GSGD_ROWS_IN_FLIGHT;
constexpr int RIF_BLOCKED = 2;           // all-reduce on blocked matrices (see launch_step_allreduce)
// Rows in flight for the kernels that walk a peer map.  Measured on MI355X at k = 32 and both ResNet sizes with
// a fresh permutation per launch: 3 rows sustain 71.3-72.0 % of the HBM peak, 2 rows 70.6-71.4 %, 4-6 rows
// 69.9-70.7 %; at k = 128 all sit within 0.3 % of each other.
constexpr int WALK_RIF = GSGD_WALK_ROWS_IN_FLIGHT;

// Persistent launch: never more workgroups than tiles.
static inline unsigned width_for(const Geom& geo, const Persist& p)
{
    const unsigned tiles = grid_for(geo.d);
    return p.workgroups < tiles ? (p.workgroups ? p.workgroups : 1u) : tiles;
}

// The kernels without the extras of Section 4.2 are the ones the benchmark
// times; the extended ones are picked only when weight decay or Nesterov
// momentum is switched on (or, for gossip, the stale variant is asked for).
#define GSGD_LAUNCH(KERNEL, ...) \
    hipLaunchKernelGGL(KERNEL, dim3(width_for(geo, p)), dim3(BLOCK), 0, stream, __VA_ARGS__)

hipError_t launch_step_gossip(const Geom& geo, const Hyper& hp, const SegTable& seg, float beta, const Walk& walk,
                              bool stale, bool has_trees, float* x, float* v, const float* g, Persist p,
                              hipStream_t stream)
{
    const RngKey no_key{0u, 0u};
    const uint32_t tiles = grid_for(geo.d);
    if (has_trees && stale)
        GSGD_LAUNCH((gossip_step_kernel<WALK_RIF, false, 0, true, true, true>), geo, hp, seg, -beta, walk, x, v, g, nullptr,
                    nullptr, 0.0f, no_key, 0u, p, tiles);
    else if (has_trees && hp.extended())
        GSGD_LAUNCH((gossip_step_kernel<WALK_RIF, false, 0, true, false, true>), geo, hp, seg, -beta, walk, x, v, g, nullptr,
                    nullptr, 0.0f, no_key, 0u, p, tiles);
    else if (has_trees)
        GSGD_LAUNCH((gossip_step_kernel<WALK_RIF, false, 0, false, false, true>), geo, hp, seg, -beta, walk, x, v, g,
                    nullptr, nullptr, 0.0f, no_key, 0u, p, tiles);
    else if (stale)
        GSGD_LAUNCH((gossip_step_kernel<WALK_RIF, false, 0, true, true>), geo, hp, seg, -beta, walk, x, v, g, nullptr,
                    nullptr, 0.0f, no_key, 0u, p, tiles);
    else if (hp.extended())
        GSGD_LAUNCH((gossip_step_kernel<WALK_RIF, false, 0, true, false>), geo, hp, seg, -beta, walk, x, v, g, nullptr,
                    nullptr, 0.0f, no_key, 0u, p, tiles);
    else
        GSGD_LAUNCH((gossip_step_kernel<WALK_RIF, false, 0>), geo, hp, seg, -beta, walk, x, v, g, nullptr, nullptr,
                    0.0f, no_key, 0u, p, tiles);
    return hipGetLastError();
}

hipError_t launch_step_gossip_push(const Geom& geo, const Hyper& hp, const SegTable& seg, const Walk& walk,
                                   float* x, float* v, const float* g, Persist p, hipStream_t stream)
{
    const RngKey no_key{0u, 0u};
    if (hp.extended())
        GSGD_LAUNCH((push_step_kernel<WALK_RIF, true>), geo, hp, seg, walk, x, v, g, nullptr, nullptr, 0.0f, no_key, 0u,
                    p, grid_for(geo.d));
    else
        GSGD_LAUNCH((push_step_kernel<WALK_RIF, false>), geo, hp, seg, walk, x, v, g, nullptr, nullptr, 0.0f, no_key,
                    0u, p, grid_for(geo.d));
    return hipGetLastError();
}

// Generator-fused push-gossip (the extended local step covers the plain one: weight decay 0, heavy ball).
hipError_t launch_step_gossip_push_fused(const Geom& geo, const Hyper& hp, const SegTable& seg, const Walk& walk,
                                         float* x, float* v, const float* h, const float* xstar,
                                         float sigma, RngKey key, uint32_t step, int noise_kind, Persist p,
                                         hipStream_t stream)
{
    if (noise_kind == GSGD_NOISE_UNIFORM)
        GSGD_LAUNCH((push_step_kernel<WALK_RIF, true, true, GSGD_NOISE_UNIFORM>), geo, hp, seg, walk, x, v, nullptr, h,
                    xstar, sigma, key, step, p, grid_for(geo.d));
    else
        GSGD_LAUNCH((push_step_kernel<WALK_RIF, true, true, GSGD_NOISE_GAUSSIAN>), geo, hp, seg, walk, x, v, nullptr, h,
                    xstar, sigma, key, step, p, grid_for(geo.d));
    return hipGetLastError();
}

// The local row walk: two rows in flight a point ahead of four at k = 32, level at k = 16; one loses 8-10 points.
constexpr int LOCAL_WALK_RIF = 2;

hipError_t launch_step_local(const Geom& geo, const Hyper& hp, const SegTable& seg,
                             float* x, float* v, const float* g, unsigned band_tiles, Persist p, hipStream_t stream)
{
    if (p.tickets) {                                 // persistent workgroups walking the rows (blocked matrices)
        if (hp.extended()) GSGD_LAUNCH((local_walk_kernel<LOCAL_WALK_RIF, true>), geo, hp, seg, x, v, g, p, grid_for(geo.d));
        else GSGD_LAUNCH((local_walk_kernel<LOCAL_WALK_RIF, false>), geo, hp, seg, x, v, g, p, grid_for(geo.d));
        return hipGetLastError();
    }
    const FlatGrid fg = flat_grid(geo, band_tiles);
    const unsigned tiles = grid_for(geo.d);
    if (hp.extended())
        hipLaunchKernelGGL(local_step_kernel<true>, fg.grid, dim3(BLOCK), 0, stream, geo, hp, seg, x, v, g, fg.band, tiles);
    else
        hipLaunchKernelGGL(local_step_kernel<false>, fg.grid, dim3(BLOCK), 0, stream, geo, hp, seg, x, v, g, fg.band, tiles);
    return hipGetLastError();
}

hipError_t launch_step_gossip_fused(const Geom& geo, const Hyper& hp, const SegTable& seg, float beta,
                                    const Walk& walk, bool stale, bool has_trees, float* x, float* v, const float* h,
                                    const float* xstar, float sigma, RngKey key, uint32_t step, int noise_kind,
                                    Persist p, hipStream_t stream)
{
    const uint32_t tiles = grid_for(geo.d);
    const bool uniform = noise_kind == GSGD_NOISE_UNIFORM;
#define GSGD_FUSED(NOISE, STALE, TREE) \
    GSGD_LAUNCH((gossip_step_kernel<WALK_RIF, true, NOISE, true, STALE, TREE>), geo, hp, seg, -beta, walk, x, v, nullptr, \
                h, xstar, sigma, key, step, p, tiles)
    if (stale || has_trees) {                 // the extended local step covers the plain one here
        if (uniform) {
            if (stale && has_trees) GSGD_FUSED(GSGD_NOISE_UNIFORM, true, true);
            else if (stale) GSGD_FUSED(GSGD_NOISE_UNIFORM, true, false);
            else GSGD_FUSED(GSGD_NOISE_UNIFORM, false, true);
        } else {
            if (stale && has_trees) GSGD_FUSED(GSGD_NOISE_GAUSSIAN, true, true);
            else if (stale) GSGD_FUSED(GSGD_NOISE_GAUSSIAN, true, false);
            else GSGD_FUSED(GSGD_NOISE_GAUSSIAN, false, true);
        }
        return hipGetLastError();
    }
#undef GSGD_FUSED
    if (hp.extended()) {
        if (uniform)
            GSGD_LAUNCH((gossip_step_kernel<WALK_RIF, true, GSGD_NOISE_UNIFORM, true>), geo, hp, seg, -beta, walk, x, v,
                        nullptr, h, xstar, sigma, key, step, p, tiles);
        else
            GSGD_LAUNCH((gossip_step_kernel<WALK_RIF, true, GSGD_NOISE_GAUSSIAN, true>), geo, hp, seg, -beta, walk, x, v,
                        nullptr, h, xstar, sigma, key, step, p, tiles);
    } else {
        if (uniform)
            GSGD_LAUNCH((gossip_step_kernel<WALK_RIF, true, GSGD_NOISE_UNIFORM>), geo, hp, seg, -beta, walk, x, v,
                        nullptr, h, xstar, sigma, key, step, p, tiles);
        else
            GSGD_LAUNCH((gossip_step_kernel<WALK_RIF, true, GSGD_NOISE_GAUSSIAN>), geo, hp, seg, -beta, walk, x, v,
                        nullptr, h, xstar, sigma, key, step, p, tiles);
    }
    return hipGetLastError();
}

// Wavefronts per workgroup of the row-split kernels: enough that a wavefront's share is a handful of rows.
static inline int split_waves(int k) { return k >= 48 ? 16 : 4; }

static inline unsigned split_grid(const Geom& geo)
{
    return static_cast<unsigned>((geo.d + SPLIT_COLUMNS - 1) / SPLIT_COLUMNS);
}

hipError_t launch_step_allreduce(const Geom& geo, const Hyper& hp, const SegTable& seg,
                                 float* x, float* v, const float* g, Persist p, bool row_split, hipStream_t stream)
{
    if (row_split) {
        const dim3 grid(split_grid(geo));
        if (split_waves(geo.k) == 16) {
            if (hp.extended())
                hipLaunchKernelGGL((allreduce_rowsplit_kernel<16, true>), grid, dim3(1024), 0, stream, geo, hp, seg, x, v, g);
            else
                hipLaunchKernelGGL((allreduce_rowsplit_kernel<16, false>), grid, dim3(1024), 0, stream, geo, hp, seg, x, v, g);
        } else {
            if (hp.extended())
                hipLaunchKernelGGL((allreduce_rowsplit_kernel<4, true>), grid, dim3(256), 0, stream, geo, hp, seg, x, v, g);
            else
                hipLaunchKernelGGL((allreduce_rowsplit_kernel<4, false>), grid, dim3(256), 0, stream, geo, hp, seg, x, v, g);
        }
        return hipGetLastError();
    }
    // Blocked matrices: shallower batches (pass 1 four rows, not eight).  Blocks of 16 Ki columns, ResNet-50 size,
    // % of the HBM peak with RIF 4 / 2: k = 16 84.2 / 84.9, k = 32 81.7 / 83.0, k = 128 78.0 / 81.0 (k = 8 level; 3 is
    // 4-8 points behind both).
    const bool blocked = geo.block_log2 >= 0;
    if (hp.extended()) {
        if (blocked) GSGD_LAUNCH((allreduce_step_kernel<RIF_BLOCKED, true>), geo, hp, seg, x, v, g, p, grid_for(geo.d));
        else GSGD_LAUNCH((allreduce_step_kernel<RIF, true>), geo, hp, seg, x, v, g, p, grid_for(geo.d));
    } else {
        if (blocked) GSGD_LAUNCH((allreduce_step_kernel<RIF_BLOCKED>), geo, hp, seg, x, v, g, p, grid_for(geo.d));
        else GSGD_LAUNCH((allreduce_step_kernel<RIF>), geo, hp, seg, x, v, g, p, grid_for(geo.d));
    }
    return hipGetLastError();
}

// Elastic averaging keeps an fp64 accumulator next to the rows in flight.  Measured at ResNet-50 size, alternating
// on one allocation, row-major matrices: with many replicas two rows in flight beat four (k = 64: 78.5 % against
// 75.5 % of the HBM peak, k = 128: 79.6 % against 76.7 %), with few it is the other way round (k = 16: 65 % against
// 67 %).  On blocked matrices two rows in flight and one workgroup per compute unit are best at every k (blocks of
// 16 Ki columns, RIF 4 with two workgroups per compute unit against RIF 2 with one: k = 8 85.4 / 88.7, k = 16
// 81.3 / 86.8, k = 32 79.4 / 85.7 %; from k = 48 on the two coincide).
constexpr int EASGD_RIF_MANY_REPLICAS = 2;
constexpr int EASGD_MANY_REPLICAS = 48;

hipError_t launch_step_easgd(const Geom& geo, const Hyper& hp, const SegTable& seg, float alpha_e,
                             float* x, float* v, const float* g, float* center, Persist p, bool row_split,
                             hipStream_t stream)
{
    if (row_split) {
        const dim3 grid(split_grid(geo));
        if (split_waves(geo.k) == 16) {
            if (hp.extended())
                hipLaunchKernelGGL((easgd_rowsplit_kernel<16, true>), grid, dim3(1024), 0, stream, geo, hp, seg, alpha_e, x, v, g, center);
            else
                hipLaunchKernelGGL((easgd_rowsplit_kernel<16, false>), grid, dim3(1024), 0, stream, geo, hp, seg, alpha_e, x, v, g, center);
        } else {
            if (hp.extended())
                hipLaunchKernelGGL((easgd_rowsplit_kernel<4, true>), grid, dim3(256), 0, stream, geo, hp, seg, alpha_e, x, v, g, center);
            else
                hipLaunchKernelGGL((easgd_rowsplit_kernel<4, false>), grid, dim3(256), 0, stream, geo, hp, seg, alpha_e, x, v, g, center);
        }
        return hipGetLastError();
    }
    const bool many = geo.k >= EASGD_MANY_REPLICAS || geo.block_log2 >= 0;
    if (hp.extended()) {
        if (many)
            GSGD_LAUNCH((easgd_step_kernel<EASGD_RIF_MANY_REPLICAS, true>), geo, hp, seg, alpha_e, x, v, g, center, p,
                        grid_for(geo.d));
        else
            GSGD_LAUNCH((easgd_step_kernel<RIF, true>), geo, hp, seg, alpha_e, x, v, g, center, p, grid_for(geo.d));
    } else {
        if (many)
            GSGD_LAUNCH((easgd_step_kernel<EASGD_RIF_MANY_REPLICAS>), geo, hp, seg, alpha_e, x, v, g, center, p,
                        grid_for(geo.d));
        else
            GSGD_LAUNCH((easgd_step_kernel<RIF>), geo, hp, seg, alpha_e, x, v, g, center, p, grid_for(geo.d));
    }
    return hipGetLastError();
}
#undef GSGD_LAUNCH
#endif  // GSGD_NO_LAUNCHERS

}  // namespace gsgd

// The three aggregation-step kernels: gossip (Section 3.1 of the paper),
// all-reduce average (Algorithm 1) and elastic averaging (Algorithm 2).
//
// Every rule couples only the k values of one column, so a thread owns four
// adjacent columns (one 128-bit lane) of all k replica rows and walks the rows.
// A wavefront reads or writes 1 KiB contiguous per access; x, v and g are each
// read once and x, v written once: 20 bytes per replica-element, the minimum.
#include "device_common.hpp"

namespace gsgd {

// Rows fetched together before any of them is processed: 3*U independent
// 16-byte loads per lane are in flight ahead of the first dependent use.
constexpr int ROWS_IN_FLIGHT = 4;

// ---------------------------------------------------------------------------
// Gossip.  x_new[i] needs the post-step parameters of replica i and of its
// peer.  Rows are visited along the cycles of the permutation,
// i -> perm[i] -> perm[perm[i]] ..., so the peer of the row visited last time
// is the row visited now: keeping `first`, `prev` and the current x' in
// registers is enough to finish every row in place, in one pass, without a
// second buffer and without two replicas ever racing on a row.
template <bool FUSED_GEN, int NOISE>
__global__ __launch_bounds__(BLOCK)
void gossip_step_kernel(Geom geo, Hyper hp, SegTable seg, float neg_beta, Walk walk,
                        float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                        const float* __restrict__ h, const float* __restrict__ xstar,
                        float sigma, RngKey key, uint32_t step)
{
    __shared__ SegLds lds;
    stage_segments(seg, lds);
    const Quad qd = my_quad(geo.d);
    if (qd.valid == 0) return;
    const int valid = qd.valid;
    const f32x4 neg_lr = -quad_lr(seg, lds, qd.col, valid, hp.lr);
    float* xq = x + qd.col;
    float* vq = v + qd.col;
    const float* gq = FUSED_GEN ? nullptr : g + qd.col;
    f32x4 h4 = {0.f, 0.f, 0.f, 0.f}, xs4 = {0.f, 0.f, 0.f, 0.f};
    if constexpr (FUSED_GEN) {
        h4 = load_quad_cached(h + qd.col, valid);
        xs4 = load_quad_cached(xstar + qd.col, valid);
    }
    const uint32_t quad_index = static_cast<uint32_t>(qd.col >> 2);

    f32x4 first = {0.f, 0.f, 0.f, 0.f}, prev = {0.f, 0.f, 0.f, 0.f};
    int64_t prev_off = 0;
    const int k = geo.k;
    for (int t0 = 0; t0 < k; t0 += ROWS_IN_FLIGHT) {
        f32x4 X[ROWS_IN_FLIGHT], V[ROWS_IN_FLIGHT], G[ROWS_IN_FLIGHT];
        uint32_t w[ROWS_IN_FLIGHT];
#pragma unroll
        for (int u = 0; u < ROWS_IN_FLIGHT; ++u) {
            if (t0 + u < k) {
                w[u] = walk.seq[t0 + u];
                const int64_t off = static_cast<int64_t>(w[u] & WALK_ROW_MASK) * geo.ld;
                X[u] = load_quad(xq + off, valid);
                V[u] = load_quad(vq + off, valid);
                if constexpr (!FUSED_GEN) G[u] = load_quad(gq + off, valid);
            }
        }
#pragma unroll
        for (int u = 0; u < ROWS_IN_FLIGHT; ++u) {
            if (t0 + u < k) {
                const uint32_t row = w[u] & WALK_ROW_MASK;
                const int64_t off = static_cast<int64_t>(row) * geo.ld;
                if constexpr (FUSED_GEN) {
                    const f32x4 xi = noise4<NOISE>(philox4x32_10(quad_index, row, step, STREAM_GRAD, key.k0, key.k1));
                    const f32x4 t1 = X[u] - xs4;
                    const f32x4 t2 = sigma * xi;
                    G[u] = fma4(h4, t1, t2);
                }
                const f32x4 vn = momentum_update(V[u], G[u], neg_lr, hp.mu);
                const f32x4 xp = X[u] + vn;
                store_quad(vq + off, vn, valid);
                if (w[u] & WALK_FIRST) first = xp;
                else store_quad(xq + prev_off, gossip_mix(prev, xp, neg_beta), valid);
                if (w[u] & WALK_LAST) store_quad(xq + off, gossip_mix(xp, first, neg_beta), valid);
                prev = xp;
                prev_off = off;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// All-reduce average (Algorithm 1).  Pass 1 reads v and g of every row and
// accumulates u_i = mu v_i - lr g_i in fp64 in ascending i; pass 2 adds the
// rounded mean to every row of x and leaves it in every row of v.
__global__ __launch_bounds__(BLOCK)
void allreduce_step_kernel(Geom geo, Hyper hp, SegTable seg,
                           float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g)
{
    __shared__ SegLds lds;
    stage_segments(seg, lds);
    const Quad qd = my_quad(geo.d);
    if (qd.valid == 0) return;
    const int valid = qd.valid;
    const f32x4 neg_lr = -quad_lr(seg, lds, qd.col, valid, hp.lr);
    float* xq = x + qd.col;
    float* vq = v + qd.col;
    const float* gq = g + qd.col;
    const int k = geo.k;

    f64x4 acc = {0.0, 0.0, 0.0, 0.0};
    for (int i0 = 0; i0 < k; i0 += ROWS_IN_FLIGHT) {
        f32x4 V[ROWS_IN_FLIGHT], G[ROWS_IN_FLIGHT];
#pragma unroll
        for (int u = 0; u < ROWS_IN_FLIGHT; ++u) {
            if (i0 + u < k) {
                const int64_t off = static_cast<int64_t>(i0 + u) * geo.ld;
                V[u] = load_quad(vq + off, valid);
                G[u] = load_quad(gq + off, valid);
            }
        }
#pragma unroll
        for (int u = 0; u < ROWS_IN_FLIGHT; ++u) {
            if (i0 + u < k) {
                const f32x4 un = momentum_update(V[u], G[u], neg_lr, hp.mu);
                acc.x += static_cast<double>(un.x);
                acc.y += static_cast<double>(un.y);
                acc.z += static_cast<double>(un.z);
                acc.w += static_cast<double>(un.w);
            }
        }
    }
    const double kd = static_cast<double>(k);
    const f32x4 ubar = {static_cast<float>(acc.x / kd), static_cast<float>(acc.y / kd),
                        static_cast<float>(acc.z / kd), static_cast<float>(acc.w / kd)};
    for (int i0 = 0; i0 < k; i0 += ROWS_IN_FLIGHT) {
        f32x4 X[ROWS_IN_FLIGHT];
#pragma unroll
        for (int u = 0; u < ROWS_IN_FLIGHT; ++u)
            if (i0 + u < k) X[u] = load_quad(xq + static_cast<int64_t>(i0 + u) * geo.ld, valid);
#pragma unroll
        for (int u = 0; u < ROWS_IN_FLIGHT; ++u) {
            if (i0 + u < k) {
                const int64_t off = static_cast<int64_t>(i0 + u) * geo.ld;
                store_quad(vq + off, ubar, valid);
                store_quad(xq + off, X[u] + ubar, valid);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Elastic averaging (Algorithm 2, period 1, one synchronous round):
// every client moves towards the same centre value, the centre moves by the
// sum of what the clients gave up.
__global__ __launch_bounds__(BLOCK)
void easgd_step_kernel(Geom geo, Hyper hp, SegTable seg, float alpha_e,
                       float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                       float* __restrict__ center)
{
    __shared__ SegLds lds;
    stage_segments(seg, lds);
    const Quad qd = my_quad(geo.d);
    if (qd.valid == 0) return;
    const int valid = qd.valid;
    const f32x4 neg_lr = -quad_lr(seg, lds, qd.col, valid, hp.lr);
    float* xq = x + qd.col;
    float* vq = v + qd.col;
    const float* gq = g + qd.col;
    const f32x4 c4 = load_quad_cached(center + qd.col, valid);
    const int k = geo.k;

    f64x4 acc = {0.0, 0.0, 0.0, 0.0};
    for (int i0 = 0; i0 < k; i0 += ROWS_IN_FLIGHT) {
        f32x4 X[ROWS_IN_FLIGHT], V[ROWS_IN_FLIGHT], G[ROWS_IN_FLIGHT];
#pragma unroll
        for (int u = 0; u < ROWS_IN_FLIGHT; ++u) {
            if (i0 + u < k) {
                const int64_t off = static_cast<int64_t>(i0 + u) * geo.ld;
                X[u] = load_quad(xq + off, valid);
                V[u] = load_quad(vq + off, valid);
                G[u] = load_quad(gq + off, valid);
            }
        }
#pragma unroll
        for (int u = 0; u < ROWS_IN_FLIGHT; ++u) {
            if (i0 + u < k) {
                const int64_t off = static_cast<int64_t>(i0 + u) * geo.ld;
                const f32x4 vn = momentum_update(V[u], G[u], neg_lr, hp.mu);
                const f32x4 xp = X[u] + vn;
                const f32x4 e = alpha_e * (xp - c4);
                store_quad(vq + off, vn, valid);
                store_quad(xq + off, xp - e, valid);
                acc.x += static_cast<double>(e.x);
                acc.y += static_cast<double>(e.y);
                acc.z += static_cast<double>(e.z);
                acc.w += static_cast<double>(e.w);
            }
        }
    }
    const f32x4 cn = {static_cast<float>(static_cast<double>(c4.x) + acc.x),
                      static_cast<float>(static_cast<double>(c4.y) + acc.y),
                      static_cast<float>(static_cast<double>(c4.z) + acc.z),
                      static_cast<float>(static_cast<double>(c4.w) + acc.w)};
    store_quad(center + qd.col, cn, valid);
}

// ---------------------------------------------------------------------------
hipError_t launch_step_gossip(const Geom& geo, const Hyper& hp, const SegTable& seg, float beta, const Walk& walk,
                              float* x, float* v, const float* g, hipStream_t stream)
{
    hipLaunchKernelGGL((gossip_step_kernel<false, 0>), dim3(grid_for(geo.d)), dim3(BLOCK), 0, stream,
                       geo, hp, seg, -beta, walk, x, v, g, nullptr, nullptr, 0.0f, RngKey{0u, 0u}, 0u);
    return hipGetLastError();
}

hipError_t launch_step_gossip_fused(const Geom& geo, const Hyper& hp, const SegTable& seg, float beta,
                                    const Walk& walk, float* x, float* v, const float* h, const float* xstar,
                                    float sigma, RngKey key, uint32_t step, int noise_kind, hipStream_t stream)
{
    if (noise_kind == GSGD_NOISE_UNIFORM)
        hipLaunchKernelGGL((gossip_step_kernel<true, GSGD_NOISE_UNIFORM>), dim3(grid_for(geo.d)), dim3(BLOCK), 0,
                           stream, geo, hp, seg, -beta, walk, x, v, nullptr, h, xstar, sigma, key, step);
    else
        hipLaunchKernelGGL((gossip_step_kernel<true, GSGD_NOISE_GAUSSIAN>), dim3(grid_for(geo.d)), dim3(BLOCK), 0,
                           stream, geo, hp, seg, -beta, walk, x, v, nullptr, h, xstar, sigma, key, step);
    return hipGetLastError();
}

hipError_t launch_step_allreduce(const Geom& geo, const Hyper& hp, const SegTable& seg,
                                 float* x, float* v, const float* g, hipStream_t stream)
{
    hipLaunchKernelGGL(allreduce_step_kernel, dim3(grid_for(geo.d)), dim3(BLOCK), 0, stream, geo, hp, seg, x, v, g);
    return hipGetLastError();
}

hipError_t launch_step_easgd(const Geom& geo, const Hyper& hp, const SegTable& seg, float alpha_e,
                             float* x, float* v, const float* g, float* center, hipStream_t stream)
{
    hipLaunchKernelGGL(easgd_step_kernel, dim3(grid_for(geo.d)), dim3(BLOCK), 0, stream,
                       geo, hp, seg, alpha_e, x, v, g, center);
    return hipGetLastError();
}

}  // namespace gsgd

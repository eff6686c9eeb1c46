// Asynchronous pull-gossip, one tick of the master clock (Section 6.1.2 of the
// paper): the node i whose clock ticked takes its local step and mixes with
// node j as node j stands; every other node is untouched,
//   theta_{t+1} = D (theta_t - alpha g_t),   D = I + beta e_i (e_j - e_i)^T.
// One tick streams one replica row (plus the peer's row): a flat kernel, every
// thread owning one quad of the row, one workgroup per 1024-column tile.  (The
// ticket-fed persistent launch of the k-row kernels does not pay here: a tile
// is a single 20 KB visit, and the ticket round trip per visit would dominate.)
#include "device_common.hpp"

namespace gsgd {

template <bool FULL, bool FUSED_GEN, int NOISE, bool EXT>
__device__ __forceinline__
void async_tick_body(const Geom& geo, const Hyper& hp, const SegTable& seg, const SegLds& lds, const Quad& qd,
                     float neg_beta, int32_t i, int32_t j,
                     float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                     const float* __restrict__ h, const float* __restrict__ xstar,
                     float sigma, RngKey key, uint32_t tick)
{
    const int valid = FULL ? 4 : qd.valid;
    const int64_t mine_off = static_cast<int64_t>(i) * geo.rs + qd.mat + qd.lane_col;
    const f32x4 X = load_quad<FULL>(x + mine_off, valid);
    const f32x4 V = load_quad<FULL>(v + mine_off, valid);
    f32x4 G, theirs = {0.f, 0.f, 0.f, 0.f};
    if (j != i) theirs = load_quad<FULL>(x + static_cast<int64_t>(j) * geo.rs + qd.mat + qd.lane_col, valid);   // uniform branch
    if constexpr (FUSED_GEN) {
        const f32x4 h4 = load_quad<FULL>(h + qd.col, valid);
        const f32x4 xs4 = load_quad<FULL>(xstar + qd.col, valid);
        const f32x4 xi = noise4<NOISE>(philox4x32_10(static_cast<uint32_t>(qd.col >> 2), static_cast<uint32_t>(i), tick,
                                                     STREAM_GRAD, key.k0, key.k1));
        const f32x4 t1 = X - xs4;
        const f32x4 t2 = sigma * xi;
        G = fma4(h4, t1, t2);
    } else {
        G = load_quad<FULL>(g + mine_off, valid);
    }
    const f32x4 neg_lr = -quad_lr(seg, lds, qd.col, valid, hp.lr);
    f32x4 vn, post;
    local_step<EXT>(X, V, G, neg_lr, hp, vn, post);
    if (j == i) theirs = post;
    store_quad<FULL>(v + mine_off, vn, valid);
    store_quad<FULL>(x + mine_off, mix_keys(post, post, theirs, neg_beta), valid);
}

template <bool FUSED_GEN, int NOISE, bool EXT>
__global__ __launch_bounds__(BLOCK)
void async_tick_kernel(Geom geo, Hyper hp, SegTable seg, float neg_beta, int32_t i, int32_t j,
                       float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                       const float* __restrict__ h, const float* __restrict__ xstar,
                       float sigma, RngKey key, uint32_t tick)
{
    __shared__ SegLds lds;
    stage_segments(seg, lds);
    const Quad qd = my_quad(geo);
    if (tile_is_full(qd, geo.d))
        async_tick_body<true, FUSED_GEN, NOISE, EXT>(geo, hp, seg, lds, qd, neg_beta, i, j, x, v, g, h, xstar, sigma,
                                                     key, tick);
    else if (qd.valid > 0)
        async_tick_body<false, FUSED_GEN, NOISE, EXT>(geo, hp, seg, lds, qd, neg_beta, i, j, x, v, g, h, xstar, sigma,
                                                      key, tick);
}

// Elastic averaging, one client's exchange with the server (Algorithm 2 in its
// asynchronous client/server form): client i takes its local step, gives up
// e = alpha_e (x'_i - center) and the centre takes it.
template <bool FULL, bool EXT>
__device__ __forceinline__
void easgd_tick_body(const Geom& geo, const Hyper& hp, const SegTable& seg, const SegLds& lds, const Quad& qd,
                     float alpha_e, int32_t i, float* __restrict__ x, float* __restrict__ v,
                     const float* __restrict__ g, float* __restrict__ center)
{
    const int valid = FULL ? 4 : qd.valid;
    const int64_t mine_off = static_cast<int64_t>(i) * geo.rs + qd.mat + qd.lane_col;
    const f32x4 X = load_quad<FULL>(x + mine_off, valid);
    const f32x4 V = load_quad<FULL>(v + mine_off, valid);
    const f32x4 G = load_quad<FULL>(g + mine_off, valid);
    const f32x4 C = load_quad<FULL>(center + qd.col, valid);
    const f32x4 neg_lr = -quad_lr(seg, lds, qd.col, valid, hp.lr);
    f32x4 vn, post;
    local_step<EXT>(X, V, G, neg_lr, hp, vn, post);
    const f32x4 e = alpha_e * (post - C);
    store_quad<FULL>(v + mine_off, vn, valid);
    store_quad<FULL>(x + mine_off, post - e, valid);
    store_quad<FULL>(center + qd.col, C + e, valid);
}

template <bool EXT>
__global__ __launch_bounds__(BLOCK)
void easgd_tick_kernel(Geom geo, Hyper hp, SegTable seg, float alpha_e, int32_t i,
                       float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                       float* __restrict__ center)
{
    __shared__ SegLds lds;
    stage_segments(seg, lds);
    const Quad qd = my_quad(geo);
    if (tile_is_full(qd, geo.d)) easgd_tick_body<true, EXT>(geo, hp, seg, lds, qd, alpha_e, i, x, v, g, center);
    else if (qd.valid > 0) easgd_tick_body<false, EXT>(geo, hp, seg, lds, qd, alpha_e, i, x, v, g, center);
}

hipError_t launch_easgd_tick(const Geom& geo, const Hyper& hp, const SegTable& seg, float alpha_e, int32_t i,
                             float* x, float* v, const float* g, float* center, hipStream_t stream)
{
    if (hp.extended())
        hipLaunchKernelGGL(easgd_tick_kernel<true>, dim3(grid_for(geo.d)), dim3(BLOCK), 0, stream,
                           geo, hp, seg, alpha_e, i, x, v, g, center);
    else
        hipLaunchKernelGGL(easgd_tick_kernel<false>, dim3(grid_for(geo.d)), dim3(BLOCK), 0, stream,
                           geo, hp, seg, alpha_e, i, x, v, g, center);
    return hipGetLastError();
}

template <bool FUSED_GEN, int NOISE>
static void launch_one(const Geom& geo, const Hyper& hp, const SegTable& seg, float beta, int32_t i, int32_t j,
                       float* x, float* v, const float* g, const float* h, const float* xstar,
                       float sigma, RngKey key, uint32_t tick, hipStream_t stream)
{
    const unsigned tiles = grid_for(geo.d);
    if (hp.extended())
        hipLaunchKernelGGL((async_tick_kernel<FUSED_GEN, NOISE, true>), dim3(tiles), dim3(BLOCK), 0, stream,
                           geo, hp, seg, -beta, i, j, x, v, g, h, xstar, sigma, key, tick);
    else
        hipLaunchKernelGGL((async_tick_kernel<FUSED_GEN, NOISE, false>), dim3(tiles), dim3(BLOCK), 0, stream,
                           geo, hp, seg, -beta, i, j, x, v, g, h, xstar, sigma, key, tick);
}

hipError_t launch_async_tick(const Geom& geo, const Hyper& hp, const SegTable& seg, float beta, int32_t i, int32_t j,
                             float* x, float* v, const float* g, hipStream_t stream)
{
    launch_one<false, 0>(geo, hp, seg, beta, i, j, x, v, g, nullptr, nullptr, 0.0f, RngKey{0u, 0u}, 0u, stream);
    return hipGetLastError();
}

hipError_t launch_async_tick_fused(const Geom& geo, const Hyper& hp, const SegTable& seg, float beta, int32_t i,
                                   int32_t j, float* x, float* v, const float* h, const float* xstar,
                                   float sigma, RngKey key, uint32_t tick, int noise_kind, hipStream_t stream)
{
    if (noise_kind == GSGD_NOISE_UNIFORM)
        launch_one<true, GSGD_NOISE_UNIFORM>(geo, hp, seg, beta, i, j, x, v, nullptr, h, xstar, sigma, key, tick,
                                             stream);
    else
        launch_one<true, GSGD_NOISE_GAUSSIAN>(geo, hp, seg, beta, i, j, x, v, nullptr, h, xstar, sigma, key, tick,
                                              stream);
    return hipGetLastError();
}

}  // namespace gsgd

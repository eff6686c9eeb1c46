// Generators: the shared vectors of the noisy quadratic, replica
// initialisation, and the synthetic stochastic gradient
//   g_i = h (.) (x_i - xstar) + sigma xi_i
// that stands in for back-propagation (the gradient-sampling model of the
// paper's Theorem 1).  All randomness is Philox4x32-10 keyed by the seed, with
// counter (column / 4, replica, step, stream): one block of four words feeds
// the four columns of a thread's quad.
#include "device_common.hpp"

namespace gsgd {

// The rows of g are independent, so nothing forces a workgroup to walk them: one workgroup per (tile, replica),
// dispatched band by band -- grid (tiles of a band, k, bands), x fastest -- streams every row in runs of one band
// while h and xstar of the band (2 x 4 bytes per column, read by all k rows) stay in the caches between rows.
// This is the access order of the flat local step, the one the memory system serves best.  Measured against
// persistent workgroups walking the k rows of a tile (% of the HBM peak, same box): k = 32, ResNet-50 size 70.0
// against 68.5; k = 128 68.2 against 62.0; k = 8, ResNet-18 size 72.6 against 60.8.  Bands of 1024 tiles (4 MiB of
// a row; h and xstar of a band 8 MiB) are best or tied with 768 ... 3072 at every shape; from 4096 tiles on h and
// xstar fall out of the caches between rows and the rate drops to 50 %.
constexpr unsigned GEN_BAND_TILES = 1024;
// In the blocked layout bands of 32 tiles (128 KiB of a row, in one block or two) measured best: blocks of 64 Ki
// columns 78 % against 71 % with the whole block as one band, 74 / 72 / 62 % with 16 / 8 / 4 tiles; blocks of 16 Ki
// columns 75 % against 73 % with one block (16 tiles) and 69 / 61 / 67 % with 64 / 128 / 1024.
constexpr unsigned GEN_BLOCKED_BAND_TILES = 32;


template <int NOISE>
__global__ __launch_bounds__(BLOCK)
void gen_grad_kernel(Geom geo, const float* __restrict__ x, const float* __restrict__ h,
                          const float* __restrict__ xstar, float* __restrict__ g,
                          float sigma, RngKey key, uint32_t step, uint32_t band_tiles, uint32_t n_tiles)
{
    const uint32_t tile = blockIdx.z * band_tiles + blockIdx.x;
    if (tile >= n_tiles) return;
    const uint32_t row = blockIdx.y;
    const Quad qd = quad_of_tile(tile, geo);
    if (qd.valid == 0) return;
    const int64_t off = static_cast<int64_t>(row) * geo.rs + qd.mat + qd.lane_col;
    const uint32_t quad_index = static_cast<uint32_t>(qd.col >> 2);
    if (tile_is_full(qd, geo.d)) {
        const f32x4 X = load_quad<true>(x + off, 4);
        const f32x4 h4 = load_quad_cached<true>(h + qd.col, 4);
        const f32x4 xs4 = load_quad_cached<true>(xstar + qd.col, 4);
        const f32x4 xi = noise4<NOISE>(philox4x32_10(quad_index, row, step, STREAM_GRAD, key.k0, key.k1));
        store_quad<true>(g + off, fma4(h4, X - xs4, sigma * xi), 4);
    } else {
        const f32x4 X = load_quad(x + off, qd.valid);
        const f32x4 h4 = load_quad_cached(h + qd.col, qd.valid);
        const f32x4 xs4 = load_quad_cached(xstar + qd.col, qd.valid);
        const f32x4 xi = noise4<NOISE>(philox4x32_10(quad_index, row, step, STREAM_GRAD, key.k0, key.k1));
        store_quad(g + off, fma4(h4, X - xs4, sigma * xi), qd.valid);
    }
}

// The same generator as persistent workgroups that walk the k rows of a tile in ascending order (h and xstar of the
// tile held in registers): the form for blocked matrices, where that order is the address order of a block.
// two rows in flight: 85 % of the HBM peak at k = 16 and 32 against 82 % with four and 80 % with eight (k = 128: 81 / 80 / 77)
constexpr int GEN_WALK_ROWS_IN_FLIGHT = 2;

template <bool FULL, int NOISE>
__device__ __forceinline__
void gen_grad_walk_body(const Geom& geo, const Quad& qd, const float* __restrict__ x, const float* __restrict__ h,
                        const float* __restrict__ xstar, float* __restrict__ g, float sigma, RngKey key, uint32_t step)
{
    constexpr int U = GEN_WALK_ROWS_IN_FLIGHT;
    const int valid = FULL ? 4 : qd.valid;
    const f32x4 h4 = load_quad_cached<FULL>(h + qd.col, valid);
    const f32x4 xs4 = load_quad_cached<FULL>(xstar + qd.col, valid);
    const uint32_t quad_index = static_cast<uint32_t>(qd.col >> 2);
    for_row_batches<U>(geo.k, [&](auto n, int i0) {
        constexpr int N = decltype(n)::value;
        f32x4 X[N];
#pragma unroll
        for (int u = 0; u < N; ++u)
            X[u] = load_quad<FULL>(x + static_cast<int64_t>(i0 + u) * geo.rs + qd.mat + qd.lane_col, valid);
#pragma unroll
        for (int u = 0; u < N; ++u) {
            const uint32_t row = static_cast<uint32_t>(i0 + u);
            const f32x4 xi = noise4<NOISE>(philox4x32_10(quad_index, row, step, STREAM_GRAD, key.k0, key.k1));
            store_quad<FULL>(g + static_cast<int64_t>(row) * geo.rs + qd.mat + qd.lane_col, fma4(h4, X[u] - xs4, sigma * xi),
                             valid);
        }
    });
}

template <int NOISE>
__global__ __launch_bounds__(BLOCK)
void gen_grad_walk_kernel(Geom geo, const float* __restrict__ x, const float* __restrict__ h,
                          const float* __restrict__ xstar, float* __restrict__ g,
                          float sigma, RngKey key, uint32_t step, Persist pst, uint32_t n_tiles)
{
    for_each_tile(pst, n_tiles, [&](uint32_t tile) {
        const Quad qd = quad_of_tile(tile, geo);
        if (tile_is_full(qd, geo.d)) gen_grad_walk_body<true, NOISE>(geo, qd, x, h, xstar, g, sigma, key, step);
        else if (qd.valid > 0) gen_grad_walk_body<false, NOISE>(geo, qd, x, h, xstar, g, sigma, key, step);
    });
}

// xstar ~ N(0,1), x0 ~ N(0,1), h = fma(0.9, u, 0.1) ~ U(0.1, 1); replica and
// step counter words are zero for these shared vectors.
__global__ __launch_bounds__(BLOCK)
void fill_kernel(int64_t d, float* __restrict__ dst, uint32_t which, RngKey key)
{
    const Quad qd = my_quad(d);
    if (qd.valid == 0) return;
    const u32x4 r = philox4x32_10(static_cast<uint32_t>(qd.col >> 2), 0u, 0u, which, key.k0, key.k1);
    f32x4 out;
    if (which == STREAM_H) {
        out = f32x4{__fmaf_rn(0.9f, u01(r.w[0]), 0.1f), __fmaf_rn(0.9f, u01(r.w[1]), 0.1f),
                    __fmaf_rn(0.9f, u01(r.w[2]), 0.1f), __fmaf_rn(0.9f, u01(r.w[3]), 0.1f)};
    } else {
        out = noise4<GSGD_NOISE_GAUSSIAN>(r);
    }
    store_quad(dst + qd.col, out, qd.valid);
}

// Start of Algorithms 1-4: all replicas (and the elastic-averaging centre)
// at one theta_0, momentum buffers at zero.  PER_REPLICA instead draws every
// row from N(0,1) and puts the centre at the rows' mean (fp64 sum, ascending).
template <bool PER_REPLICA>
__global__ __launch_bounds__(BLOCK)
void init_replicas_kernel(Geom geo, float* __restrict__ x, float* __restrict__ v, float* __restrict__ center,
                          const float* __restrict__ x0, RngKey key)
{
    const Quad qd = my_quad(geo);
    if (qd.valid == 0) return;
    const int valid = qd.valid;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    float* xq = x + qd.mat + qd.lane_col;
    float* vq = v + qd.mat + qd.lane_col;
    if constexpr (PER_REPLICA) {
        const uint32_t quad_index = static_cast<uint32_t>(qd.col >> 2);
        f64x4 acc = {0.0, 0.0, 0.0, 0.0};
        for (int i = 0; i < geo.k; ++i) {
            const f32x4 xi = noise4<GSGD_NOISE_GAUSSIAN>(
                philox4x32_10(quad_index, static_cast<uint32_t>(i), 0u, STREAM_INIT, key.k0, key.k1));
            const int64_t off = static_cast<int64_t>(i) * geo.rs;
            store_quad(xq + off, xi, valid);
            store_quad(vq + off, zero, valid);
            acc.x += static_cast<double>(xi.x);
            acc.y += static_cast<double>(xi.y);
            acc.z += static_cast<double>(xi.z);
            acc.w += static_cast<double>(xi.w);
        }
        if (center) {
            const double kd = static_cast<double>(geo.k);
            const f32x4 c = {static_cast<float>(acc.x / kd), static_cast<float>(acc.y / kd),
                             static_cast<float>(acc.z / kd), static_cast<float>(acc.w / kd)};
            store_quad(center + qd.col, c, valid);
        }
    } else {
        const f32x4 x04 = load_quad_cached(x0 + qd.col, valid);
        for (int i = 0; i < geo.k; ++i) {
            const int64_t off = static_cast<int64_t>(i) * geo.rs;
            store_quad(xq + off, x04, valid);
            store_quad(vq + off, zero, valid);
        }
        if (center) store_quad(center + qd.col, x04, valid);
    }
}

__global__ __launch_bounds__(BLOCK)
void philox_raw_kernel(RngKey key, uint32_t c1, uint32_t c2, uint32_t c3, int64_t n_blocks, uint32_t* __restrict__ out)
{
    const int64_t q = static_cast<int64_t>(blockIdx.x) * BLOCK + threadIdx.x;
    if (q >= n_blocks) return;
    const u32x4 r = philox4x32_10(static_cast<uint32_t>(q), c1, c2, c3, key.k0, key.k1);
    for (int m = 0; m < 4; ++m) out[q * 4 + m] = r.w[m];
}

// The generator's arithmetic alone, for the ALU side of the roofline: every thread draws `iters` blocks
// (counter (thread, iteration, 0, gradient stream)), turns each into four noise values and folds them into one
// float that it stores at the end, so the only memory traffic is 4 bytes per thread.  The replica and step words
// are uniform over the wavefront as they are in the real kernels (the compiler keeps their share of the rounds in
// scalar registers in both).
template <int NOISE>
__global__ __launch_bounds__(BLOCK)
void noise_alu_kernel(RngKey key, uint32_t iters, float* __restrict__ out)
{
    const uint32_t q = blockIdx.x * BLOCK + threadIdx.x;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (uint32_t it = 0; it < iters; ++it)
        acc += noise4<NOISE>(philox4x32_10(q, it, 0u, STREAM_GRAD, key.k0, key.k1));
    out[q] = (acc.x + acc.y) + (acc.z + acc.w);
}

hipError_t launch_noise_alu(RngKey key, int noise_kind, uint32_t workgroups, uint32_t iters, float* out,
                            hipStream_t stream)
{
    if (noise_kind == GSGD_NOISE_UNIFORM)
        hipLaunchKernelGGL(noise_alu_kernel<GSGD_NOISE_UNIFORM>, dim3(workgroups), dim3(BLOCK), 0, stream, key, iters, out);
    else
        hipLaunchKernelGGL(noise_alu_kernel<GSGD_NOISE_GAUSSIAN>, dim3(workgroups), dim3(BLOCK), 0, stream, key, iters, out);
    return hipGetLastError();
}

hipError_t launch_philox_raw(RngKey key, uint32_t c1, uint32_t c2, uint32_t c3, int64_t n_blocks, uint32_t* out,
                             hipStream_t stream)
{
    hipLaunchKernelGGL(philox_raw_kernel, dim3(static_cast<unsigned>((n_blocks + BLOCK - 1) / BLOCK)), dim3(BLOCK), 0,
                       stream, key, c1, c2, c3, n_blocks, out);
    return hipGetLastError();
}

hipError_t launch_gen_grad(const Geom& geo, const float* x, const float* h, const float* xstar, float* g,
                           float sigma, RngKey key, uint32_t step, int noise_kind, unsigned band_tiles, Persist p,
                           hipStream_t stream)
{
    const unsigned tiles = grid_for(geo.d);
    if (p.tickets) {                                 // persistent workgroups walking the rows
        const unsigned width = p.workgroups < tiles ? (p.workgroups ? p.workgroups : 1u) : tiles;
        if (noise_kind == GSGD_NOISE_UNIFORM)
            hipLaunchKernelGGL(gen_grad_walk_kernel<GSGD_NOISE_UNIFORM>, dim3(width), dim3(BLOCK), 0, stream,
                               geo, x, h, xstar, g, sigma, key, step, p, tiles);
        else
            hipLaunchKernelGGL(gen_grad_walk_kernel<GSGD_NOISE_GAUSSIAN>, dim3(width), dim3(BLOCK), 0, stream,
                               geo, x, h, xstar, g, sigma, key, step, p, tiles);
        return hipGetLastError();
    }
    const unsigned default_band = geo.block_log2 >= 0 ? GEN_BLOCKED_BAND_TILES : GEN_BAND_TILES;
    const FlatGrid fg = flat_grid(geo, band_tiles == 0 ? default_band : band_tiles);
    const dim3 grid = fg.grid;
    const unsigned band = fg.band;
    if (noise_kind == GSGD_NOISE_UNIFORM)
        hipLaunchKernelGGL(gen_grad_kernel<GSGD_NOISE_UNIFORM>, grid, dim3(BLOCK), 0, stream,
                           geo, x, h, xstar, g, sigma, key, step, band, tiles);
    else
        hipLaunchKernelGGL(gen_grad_kernel<GSGD_NOISE_GAUSSIAN>, grid, dim3(BLOCK), 0, stream,
                           geo, x, h, xstar, g, sigma, key, step, band, tiles);
    return hipGetLastError();
}

// Copy a matrix from one layout into another (row-major with any row stride, or blocked with any block width):
// one workgroup per (tile, row), dispatched in the order of the destination's addresses.
__global__ __launch_bounds__(BLOCK)
void relayout_kernel(Geom from, Geom to, const float* __restrict__ src, float* __restrict__ dst,
                     uint32_t band_tiles, uint32_t n_tiles)
{
    const uint32_t tile = blockIdx.z * band_tiles + blockIdx.x;
    if (tile >= n_tiles) return;
    const int64_t row = blockIdx.y;
    const Quad qa = quad_of_tile(tile, from), qb = quad_of_tile(tile, to);
    if (qa.valid == 0) return;
    const f32x4 val = load_quad(src + row * from.rs + qa.mat + qa.lane_col, qa.valid);
    store_quad(dst + row * to.rs + qb.mat + qb.lane_col, val, qa.valid);
}

hipError_t launch_relayout(const Geom& from, const Geom& to, const float* src, float* dst, hipStream_t stream)
{
    const FlatGrid fg = flat_grid(to, 0);
    hipLaunchKernelGGL(relayout_kernel, fg.grid, dim3(BLOCK), 0, stream, from, to, src, dst, fg.band, grid_for(to.d));
    return hipGetLastError();
}

hipError_t launch_fill(int64_t d, float* dst, int which, RngKey key, hipStream_t stream)
{
    hipLaunchKernelGGL(fill_kernel, dim3(grid_for(d)), dim3(BLOCK), 0, stream, d, dst, static_cast<uint32_t>(which), key);
    return hipGetLastError();
}

hipError_t launch_init_replicas(const Geom& geo, float* x, float* v, float* center, const float* x0, int mode,
                                RngKey key, hipStream_t stream)
{
    if (mode == GSGD_INIT_PER_REPLICA)
        hipLaunchKernelGGL(init_replicas_kernel<true>, dim3(grid_for(geo.d)), dim3(BLOCK), 0, stream,
                           geo, x, v, center, x0, key);
    else
        hipLaunchKernelGGL(init_replicas_kernel<false>, dim3(grid_for(geo.d)), dim3(BLOCK), 0, stream,
                           geo, x, v, center, x0, key);
    return hipGetLastError();
}

}  // namespace gsgd

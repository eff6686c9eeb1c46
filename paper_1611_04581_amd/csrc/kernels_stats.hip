// Diagnostics the paper's analysis is stated in (Section 6.1): the replicas'
// distance to their mean (the agents' consensus), their distance to the optimum,
// and the mean's own distance.  Not part of the timed step.
//
// Per column the replica mean and the squared deviations are taken in fp64 in
// one pass over the rows (x is read once).  Across columns the
// reduction is wavefront-wide by DPP lane exchanges, block-wide through LDS,
// and grid-wide through a partials buffer summed by a second one-block kernel
// in a fixed order, so the result is reproducible run to run.
#include "device_common.hpp"

namespace gsgd {

// Lane exchange through the data-parallel-primitive path (no LDS traffic).
template <int CTRL>
__device__ __forceinline__ double dpp_move(double val)
{
    const long long bits = __double_as_longlong(val);
    const int lo = __builtin_amdgcn_update_dpp(0, static_cast<int>(bits & 0xFFFFFFFFll), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, static_cast<int>(bits >> 32), CTRL, 0xF, 0xF, false);
    return __longlong_as_double((static_cast<long long>(hi) << 32) | static_cast<unsigned int>(lo));
}

// Butterfly sum over the 64 lanes; every lane ends with the total.
__device__ __forceinline__ double wave_sum(double val)
{
    val += dpp_move<0xB1>(val);     // quad_perm [1,0,3,2]: lane ^ 1
    val += dpp_move<0x4E>(val);     // quad_perm [2,3,0,1]: lane ^ 2
    val += dpp_move<0x141>(val);    // row_half_mirror: other quad of the half-row
    val += dpp_move<0x140>(val);    // row_mirror: other half of the 16-lane row
    val += __shfl_xor(val, 16, 64);
    val += __shfl_xor(val, 32, 64);
    return val;
}

// Sum of `val[0..3]` over the block; valid in thread 0.
__device__ __forceinline__ void block_sum4(double val[4], double (*lds)[4])
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int m = 0; m < 4; ++m) val[m] = wave_sum(val[m]);
    if (lane == 0)
        for (int m = 0; m < 4; ++m) lds[wave][m] = val[m];
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int m = 0; m < 4; ++m) {
            double s = lds[0][m];
            for (int wv = 1; wv < BLOCK / 64; ++wv) s += lds[wv][m];
            val[m] = s;
        }
    }
}

// Launch shape of the statistics pass.  A thread keeps up to 32 rows of its quad in flight (its whole column for
// k <= 32), and the grid is sized so that the workgroups together hold STATS_TILE_ROWS_IN_FLIGHT rows of a tile
// (4 KB each) in flight: 512 workgroups from 32 replicas on (one per compute unit resident at a time: 32 rows in
// flight take 255 registers), 1024 at 16, 2048 at 8 and below.  On matrices in
// blocks of columns this read-only pass wants few workgroups that each read a tile's whole column of rows at once
// (adjacent workgroups then cover whole blocks): at k = 32 and ResNet-50 length, 512 workgroups x 32 rows reach
// 82 % of the HBM peak where one workgroup per tile with 4 rows in flight reached 69 %, and 84 % at k = 128;
// row-major matrices reach 85 % (75 % before).  Grids that are no multiple of the 256 compute units lose 10 points.
constexpr unsigned STATS_TILE_ROWS_IN_FLIGHT = 16384;

// One pass over the rows.  Per column the deviations are taken from the first
// row's value r instead of from the mean, which is not known yet:
//   sum_i (x_i - xbar)^2 = sum_i (x_i - r)^2 - (sum_i (x_i - r))^2 / k,   xbar = r + (sum_i (x_i - r)) / k.
// x_i - r is exact in fp64 for fp32 inputs, and since r is one of the k values, (xbar - r)^2 <= the left side, so
// the subtraction loses at most a factor k + 1 of fp64's precision; k equal values give exactly zero.
// Lanes past the vector's end load zeros for x and xstar and so add nothing.
// Every workgroup strides over the tiles and leaves one set of partial sums, so the last bits of the result
// depend on the grid, which depends on k and d only.
template <int STATS_ROWS_IN_FLIGHT>
__global__ __launch_bounds__(BLOCK)
void stats_partial_kernel(Geom geo, int64_t n_tiles, const float* __restrict__ x, const float* __restrict__ xstar,
                          double* __restrict__ partials)
{
    __shared__ double lds[BLOCK / 64][4];
    double acc[4] = {0.0, 0.0, 0.0, 0.0};     // consensus, distance, mean distance, mean norm
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const Quad qd = quad_of_tile(tile, geo);
        if (qd.valid > 0) {
            const int valid = qd.valid;
            const float* xq = x + qd.mat + qd.lane_col;
            const f32x4 xs4 = load_quad_cached(xstar + qd.col, valid);
            const double xs[4] = {static_cast<double>(xs4.x), static_cast<double>(xs4.y),
                                  static_cast<double>(xs4.z), static_cast<double>(xs4.w)};
            double ref[4] = {0.0, 0.0, 0.0, 0.0};
            double s1[4] = {0.0, 0.0, 0.0, 0.0}, s2[4] = {0.0, 0.0, 0.0, 0.0};
            auto visit = [&](const f32x4& xi) {
                const double xv[4] = {static_cast<double>(xi.x), static_cast<double>(xi.y),
                                      static_cast<double>(xi.z), static_cast<double>(xi.w)};
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const double a = xv[m] - ref[m];
                    const double b = xv[m] - xs[m];
                    s1[m] += a;
                    s2[m] += a * a;
                    acc[1] += b * b;
                }
            };
            // row 0 is the reference (its own deviation is zero); it rides in the first batch
            auto take_ref = [&](const f32x4& r) {
                ref[0] = static_cast<double>(r.x); ref[1] = static_cast<double>(r.y);
                ref[2] = static_cast<double>(r.z); ref[3] = static_cast<double>(r.w);
            };
            int i = 0;
            for (; i + STATS_ROWS_IN_FLIGHT <= geo.k; i += STATS_ROWS_IN_FLIGHT) {
                f32x4 xi[STATS_ROWS_IN_FLIGHT];
#pragma unroll
                for (int u = 0; u < STATS_ROWS_IN_FLIGHT; ++u)
                    xi[u] = load_quad(xq + static_cast<int64_t>(i + u) * geo.rs, valid);
                if (i == 0) take_ref(xi[0]);
#pragma unroll
                for (int u = 0; u < STATS_ROWS_IN_FLIGHT; ++u) visit(xi[u]);
            }
            if (i < geo.k) {                                      // the rows left over, together
                f32x4 xi[STATS_ROWS_IN_FLIGHT];
#pragma unroll
                for (int u = 0; u < STATS_ROWS_IN_FLIGHT - 1; ++u)
                    if (i + u < geo.k) xi[u] = load_quad(xq + static_cast<int64_t>(i + u) * geo.rs, valid);
                if (i == 0) take_ref(xi[0]);
#pragma unroll
                for (int u = 0; u < STATS_ROWS_IN_FLIGHT - 1; ++u)
                    if (i + u < geo.k) visit(xi[u]);
            }
            const double kd = static_cast<double>(geo.k);
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const double shift = s1[m] / kd;                  // xbar - ref
                const double dev = s2[m] - s1[m] * shift;
                const double xbar = ref[m] + shift;
                const double c = xbar - xs[m];
                acc[0] += dev > 0.0 ? dev : 0.0;
                acc[2] += c * c;
                acc[3] += xbar * xbar;
            }
        }
    }
    block_sum4(acc, lds);
    if (threadIdx.x == 0)
        for (int m = 0; m < 4; ++m) partials[static_cast<int64_t>(blockIdx.x) * 4 + m] = acc[m];
}

__global__ __launch_bounds__(BLOCK)
void stats_final_kernel(int64_t n_partials, const double* __restrict__ partials, double* __restrict__ result)
{
    __shared__ double lds[BLOCK / 64][4];
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int64_t b = threadIdx.x; b < n_partials; b += BLOCK)
        for (int m = 0; m < 4; ++m) acc[m] += partials[b * 4 + m];
    block_sum4(acc, lds);
    if (threadIdx.x == 0)
        for (int m = 0; m < 4; ++m) result[m] = acc[m];
}

// Squared norm of every replica row (the ingredients of the diffusion
// potential of Section 3.1).  Grid (NORM_CHUNKS, k): a block sums the squares
// of its share of one row's tiles; a second kernel adds the NORM_CHUNKS
// partials of each row in a fixed order.
__global__ __launch_bounds__(BLOCK)
void row_sqnorm_partial_kernel(Geom geo, int64_t n_tiles, const float* __restrict__ x, double* __restrict__ partials)
{
    __shared__ double lds[BLOCK / 64][4];
    const int row = static_cast<int>(blockIdx.y);
    const float* xr = x + static_cast<int64_t>(row) * geo.rs;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const Quad qd = quad_of_tile(tile, geo);
        if (qd.valid == 0) continue;
        const f32x4 xi = load_quad(xr + qd.mat + qd.lane_col, qd.valid);        // lanes beyond `valid` come back as zero
        acc[0] += static_cast<double>(xi.x) * static_cast<double>(xi.x);
        acc[1] += static_cast<double>(xi.y) * static_cast<double>(xi.y);
        acc[2] += static_cast<double>(xi.z) * static_cast<double>(xi.z);
        acc[3] += static_cast<double>(xi.w) * static_cast<double>(xi.w);
    }
    acc[0] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    acc[1] = acc[2] = acc[3] = 0.0;
    block_sum4(acc, lds);
    if (threadIdx.x == 0) partials[static_cast<int64_t>(row) * gridDim.x + blockIdx.x] = acc[0];
}

__global__ __launch_bounds__(64)
void row_sqnorm_final_kernel(int n_chunks, const double* __restrict__ partials, double* __restrict__ result)
{
    const int row = static_cast<int>(blockIdx.x);
    if (threadIdx.x != 0) return;
    double s = 0.0;
    for (int c = 0; c < n_chunks; ++c) s += partials[static_cast<int64_t>(row) * n_chunks + c];
    result[row] = s;
}

hipError_t launch_row_sqnorms(const Geom& geo, const float* x, double* partials, double* result, hipStream_t stream)
{
    hipLaunchKernelGGL(row_sqnorm_partial_kernel, dim3(NORM_CHUNKS, static_cast<unsigned>(geo.k)), dim3(BLOCK), 0,
                       stream, geo, static_cast<int64_t>(grid_for(geo.d)), x, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(row_sqnorm_final_kernel, dim3(static_cast<unsigned>(geo.k)), dim3(64), 0, stream,
                       NORM_CHUNKS, partials, result);
    return hipGetLastError();
}

// Workgroups of the statistics pass = sets of partial sums it leaves.
static unsigned stats_rows_in_flight(int k)
{
    return k >= 32 ? 32u : k >= 16 ? 16u : 8u;
}

static unsigned stats_workgroups(int k, int64_t d)
{
    const unsigned rif = stats_rows_in_flight(k);
    const unsigned per_wg = static_cast<unsigned>(k) < rif ? static_cast<unsigned>(k) : rif;
    unsigned wgs = STATS_TILE_ROWS_IN_FLIGHT / per_wg;
    if (wgs > STATS_MAX_WORKGROUPS) wgs = STATS_MAX_WORKGROUPS;
    const unsigned tiles = grid_for(d);
    return wgs < tiles ? wgs : tiles;
}

hipError_t launch_stats(const Geom& geo, const float* x, const float* xstar, double* partials, double* result,
                        hipStream_t stream)
{
    const int64_t tiles = static_cast<int64_t>(grid_for(geo.d));
    const unsigned wgs = stats_workgroups(geo.k, geo.d);
    switch (stats_rows_in_flight(geo.k)) {
    case 32u:
        hipLaunchKernelGGL(stats_partial_kernel<32>, dim3(wgs), dim3(BLOCK), 0, stream, geo, tiles, x, xstar, partials);
        break;
    case 16u:
        hipLaunchKernelGGL(stats_partial_kernel<16>, dim3(wgs), dim3(BLOCK), 0, stream, geo, tiles, x, xstar, partials);
        break;
    default:
        hipLaunchKernelGGL(stats_partial_kernel<8>, dim3(wgs), dim3(BLOCK), 0, stream, geo, tiles, x, xstar, partials);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(stats_final_kernel, dim3(1), dim3(BLOCK), 0, stream, static_cast<int64_t>(wgs), partials, result);
    return hipGetLastError();
}

}  // namespace gsgd

// Device-side building blocks shared by the kernels: 128-bit streaming
// accesses, the Philox4x32-10 block function, the u32 -> noise transforms and
// the per-layer step-size lookup.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "gsgd_internal.hpp"

namespace gsgd {

typedef float  f32x4 __attribute__((ext_vector_type(4)));
typedef double f64x4 __attribute__((ext_vector_type(4)));

#ifndef GSGD_BLOCK
#define GSGD_BLOCK 256
#endif
constexpr int BLOCK = GSGD_BLOCK;     // threads per workgroup: 4 wavefronts of 64
static_assert(BLOCK_COLUMNS == static_cast<int64_t>(BLOCK) * 4, "a workgroup tile is BLOCK quads wide");

// One thread owns one "quad": four adjacent columns, one 128-bit lane of every
// row.  A wavefront therefore streams 1 KiB contiguous per row access.
// `valid` is 4 for a full quad and 1..3 for the ragged last quad of a row
// whose length is not a multiple of 4.  Row data is touched once per launch:
// non-temporal loads and stores (on blocked matrices the gossip step runs at
// 83.6 % of the HBM peak with both, 76-77 % with either one as an ordinary
// cached access; all-reduce 85 against 77 %, the local step 84 against 77 %).
template <bool FULL = false>
__device__ __forceinline__ f32x4 load_quad(const float* p, int valid)
{
    if (FULL || valid == 4) return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    f32x4 r = {0.f, 0.f, 0.f, 0.f};
    if (valid > 0) r.x = p[0];
    if (valid > 1) r.y = p[1];
    if (valid > 2) r.z = p[2];
    return r;
}

template <bool FULL = false>
__device__ __forceinline__ void store_quad(float* p, f32x4 r, int valid)
{
    if (FULL || valid == 4) { __builtin_nontemporal_store(r, reinterpret_cast<f32x4*>(p)); return; }
    if (valid > 0) p[0] = r.x;
    if (valid > 1) p[1] = r.y;
    if (valid > 2) p[2] = r.z;
}

// Shared vectors (h, xstar, center) are read once per column and reused for
// every replica row: ordinary cached loads.
template <bool FULL = false>
__device__ __forceinline__ f32x4 load_quad_cached(const float* p, int valid)
{
    if (FULL || valid == 4) return *reinterpret_cast<const f32x4*>(p);
    f32x4 r = {0.f, 0.f, 0.f, 0.f};
    if (valid > 0) r.x = p[0];
    if (valid > 1) r.y = p[1];
    if (valid > 2) r.z = p[2];
    return r;
}

// Element-wise helpers with the rounding points spelled out (the library is
// compiled with FP contraction off; the only fused operations are these).
__device__ __forceinline__ f32x4 fma4(float a, f32x4 b, f32x4 c)
{
    return f32x4{__fmaf_rn(a, b.x, c.x), __fmaf_rn(a, b.y, c.y), __fmaf_rn(a, b.z, c.z), __fmaf_rn(a, b.w, c.w)};
}
__device__ __forceinline__ f32x4 fma4(f32x4 a, f32x4 b, f32x4 c)
{
    return f32x4{__fmaf_rn(a.x, b.x, c.x), __fmaf_rn(a.y, b.y, c.y), __fmaf_rn(a.z, b.z, c.z), __fmaf_rn(a.w, b.w, c.w)};
}

// Local momentum step shared by Algorithms 2-4 of the paper:
//   v' = mu v - lr g  (as fma(-lr, g, mu v)),  x' = x + v'
__device__ __forceinline__ f32x4 momentum_update(f32x4 v, f32x4 g, f32x4 neg_lr, float mu)
{
    const f32x4 t3 = mu * v;
    return fma4(neg_lr, g, t3);
}

// The local step of every rule.  EXT = false: the two lines the algorithm
// boxes share.  EXT = true: the form the experiments of Section 4.2 use, with
// weight decay and optionally Nesterov momentum, on the momentum buffer:
//   gt = g + wd x  (gt = g when wd is zero);  v' = mu v - lr gt;
//   heavy ball: x' = x + v'      Nesterov: x' = (x - lr gt) + mu v'
// `gt` is returned because the all-reduce rule needs it again.
template <bool EXT>
__device__ __forceinline__ void local_step(f32x4 x, f32x4 v, f32x4 g, f32x4 neg_lr, const Hyper& hp,
                                           f32x4& v_new, f32x4& x_post, f32x4* gt_out = nullptr)
{
    if constexpr (!EXT) {
        v_new = momentum_update(v, g, neg_lr, hp.mu);
        x_post = x + v_new;
        if (gt_out) *gt_out = g;
    } else {
        // zero weight decay = no decay term: g enters as it stands (so that -0 stays -0, as in the boxed step)
        const f32x4 gt = hp.wd != 0.0f ? fma4(hp.wd, x, g) : g;
        const f32x4 t3 = hp.mu * v;
        v_new = fma4(neg_lr, gt, t3);
        if (hp.nesterov) {
            const f32x4 t4 = fma4(neg_lr, gt, x);
            x_post = fma4(hp.mu, v_new, t4);
        } else {
            x_post = x + v_new;
        }
        if (gt_out) *gt_out = gt;
    }
}

// Gossip mix: post - beta (mine - theirs).  With fresh parameters (Section
// 3.1 / 6.2.2) `mine` is the node's own post-step x' and `theirs` its peer's;
// with stale parameters (Section 6.2.1) they are the two nodes' x from before
// the local step.
__device__ __forceinline__ f32x4 mix_keys(f32x4 post, f32x4 mine, f32x4 theirs, float neg_beta)
{
    const f32x4 diff = mine - theirs;
    return fma4(neg_beta, diff, post);
}

// Push-gossip (Algorithm 4) sums what a node received in fp64.
__device__ __forceinline__ f64x4 widen(f32x4 a)
{
    return f64x4{static_cast<double>(a.x), static_cast<double>(a.y), static_cast<double>(a.z), static_cast<double>(a.w)};
}

// average of `count` received values whose fp64 sum is `sum`, rounded once
__device__ __forceinline__ f32x4 average(f64x4 sum, uint32_t count)
{
    const double c = static_cast<double>(count);
    if ((count & (count - 1u)) == 0u) {
        // a power of two (uniform test: `count` is the same for the whole workgroup): scaling by its reciprocal is
        // the same quotient exactly, without four fp64 divisions; with uniformly drawn targets half of the rows
        // that received anything received from one sender
        const double r = 1.0 / c;
        return f32x4{static_cast<float>(sum.x * r), static_cast<float>(sum.y * r),
                     static_cast<float>(sum.z * r), static_cast<float>(sum.w * r)};
    }
    return f32x4{static_cast<float>(sum.x / c), static_cast<float>(sum.y / c),
                 static_cast<float>(sum.z / c), static_cast<float>(sum.w / c)};
}

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11).  Stream ids select what
// the numbers are used for; they are the fourth counter word.
enum : uint32_t { STREAM_GRAD = 0, STREAM_INIT = 1, STREAM_XSTAR = 2, STREAM_H = 3, STREAM_X0 = 4, STREAM_PERM = 5 };

struct u32x4 { uint32_t w[4]; };

// The two 32 x 32 -> 64-bit products of a round are written as 64-bit multiplies: one v_mad_u64_u32 each
// gives the high and the low word together (measured: 211 instead of 263 SIMD cycles per wavefront block).
__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1)
{
    constexpr uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = M0 * c0;
        const uint64_t p1 = M1 * c2;
        c0 = static_cast<uint32_t>(p1 >> 32) ^ c1 ^ k0;
        c1 = static_cast<uint32_t>(p1);
        c2 = static_cast<uint32_t>(p0 >> 32) ^ c3 ^ k1;
        c3 = static_cast<uint32_t>(p0);
        k0 += W0;
        k1 += W1;
    }
    return u32x4{{c0, c1, c2, c3}};
}

// Top 23 bits b -> (2b+1) / 2^24: exact in fp32, strictly inside (0,1).
__device__ __forceinline__ float u01(uint32_t r)
{
    return __fmaf_rn(static_cast<float>(r >> 9), 0x1.0p-23f, 0x1.0p-24f);   // exact: no rounding occurs
}

// sin(pi t) and cos(pi t) for the angles Box-Muller draws: t = 2u in (0, 2), a multiple of 2^-23.  The quadrant
// reduction r = t - n/2, n = round(2t), is exact for such t and leaves |r| <= 1/4; on that interval the odd / even
// power series of sin(pi r) / cos(pi r), cut after r^9 / r^10, are below 0.3 units in the last place.  Maximum
// absolute error against fp64 over all 2^23 angles: 8.8e-8 (the general-purpose library routine: 5.1e-8, at
// about 40 more instructions per pair, which this kernel cannot hide behind its memory traffic).
__device__ __forceinline__ void sincospi_box_muller(float t, float* s, float* c)
{
    const float n = rintf(2.0f * t);                                  // 0 .. 4
    const float r = __fmaf_rn(-0.5f, n, t);
    const float r2 = r * r;
    float ps = 0.08214588661112823f;                                  //  pi^9 / 9!
    ps = __fmaf_rn(ps, r2, -0.5992645293207921f);                     // -pi^7 / 7!
    ps = __fmaf_rn(ps, r2, 2.550164039877345f);                       //  pi^5 / 5!
    ps = __fmaf_rn(ps, r2, -5.16771278004997f);                       // -pi^3 / 3!
    const float sr = __fmaf_rn(ps * r2, r, 3.141592653589793f * r);
    float pc = -0.02580689139001406f;                                 // -pi^10 / 10!
    pc = __fmaf_rn(pc, r2, 0.23533063035889320f);                     //  pi^8 / 8!
    pc = __fmaf_rn(pc, r2, -1.3352627688545893f);                     // -pi^6 / 6!
    pc = __fmaf_rn(pc, r2, 4.058712126416768f);                       //  pi^4 / 4!
    pc = __fmaf_rn(pc, r2, -4.934802200544679f);                      // -pi^2 / 2!
    const float cr = __fmaf_rn(pc, r2, 1.0f);
    const uint32_t q = static_cast<uint32_t>(static_cast<int>(n));    // quadrant: angle = pi (q/2 + r)
    const bool odd = (q & 1u) != 0u;
    const float ss = odd ? cr : sr;
    const float cc = odd ? sr : cr;
    // sine changes sign in quadrants 2, 3, cosine in 1, 2: flip the sign bit rather than select
    *s = __uint_as_float(__float_as_uint(ss) ^ ((q & 2u) << 30));
    *c = __uint_as_float(__float_as_uint(cc) ^ (((q + 1u) & 2u) << 30));
}

// ln u for u = (2b+1) / 2^24 (a normal number in [2^-24, 1)): the hardware base-2 logarithm times ln 2, with
// ln 2 held as the sum of two floats and the product's rounding error recovered by a fused multiply-add, so the
// result is as accurate as the instruction itself (about one unit in the last place).  The library's logf does the
// same after scaling and special-case tests that these arguments never need.
__device__ __forceinline__ float ln_u01(float u)
{
    constexpr float LN2_HI = 0x1.62e430p-1f;       // nearest float to ln 2
    constexpr float LN2_LO = -0x1.05c610p-29f;     // ln 2 - LN2_HI
    const float y = __builtin_amdgcn_logf(u);
    const float hi = y * LN2_HI;
    const float err = __fmaf_rn(y, LN2_HI, -hi);
    return hi + __fmaf_rn(y, LN2_LO, err);
}

// Four zero-mean unit-variance values (the noise model of Theorem 1).
//   uniform : sqrt(3) (2u - 1), bit-reproducible on any IEEE machine
//   gaussian: Box-Muller, words (0,1) -> lanes (0,1), words (2,3) -> lanes (2,3);
//             even lane carries the cosine
template <int NOISE>
__device__ __forceinline__ f32x4 noise4(const u32x4& r)
{
    if constexpr (NOISE == GSGD_NOISE_UNIFORM) {
        constexpr float sqrt3 = 1.7320508075688772f;
        f32x4 z;
        z.x = sqrt3 * __fmaf_rn(2.0f, u01(r.w[0]), -1.0f);
        z.y = sqrt3 * __fmaf_rn(2.0f, u01(r.w[1]), -1.0f);
        z.z = sqrt3 * __fmaf_rn(2.0f, u01(r.w[2]), -1.0f);
        z.w = sqrt3 * __fmaf_rn(2.0f, u01(r.w[3]), -1.0f);
        return z;
    } else {
        // -2 ln u lies in [1.2e-7, 33.3]: always a normal number, so the hardware square root (one unit in the
        // last place) needs none of the scaling and fix-up steps of the library's correctly rounded one
        const float rho0 = __builtin_amdgcn_sqrtf(-2.0f * ln_u01(u01(r.w[0])));
        const float rho1 = __builtin_amdgcn_sqrtf(-2.0f * ln_u01(u01(r.w[2])));
        float s0, c0, s1, c1;
        sincospi_box_muller(2.0f * u01(r.w[1]), &s0, &c0);
        sincospi_box_muller(2.0f * u01(r.w[3]), &s1, &c1);
        return f32x4{rho0 * c0, rho0 * s0, rho1 * c1, rho1 * s1};
    }
}

// ---------------------------------------------------------------------------
// Per-layer step size.  Column j belongs to segment s when
// offsets[s] <= j < offsets[s+1]; its step size is lr * scales[s].
// The block stages the table in LDS when it fits and binary-searches there;
// larger tables are searched in global memory.
constexpr int SEG_LDS_MAX = 1024;     // segments held in LDS (12 KiB)

struct SegLds {
    int64_t offsets[SEG_LDS_MAX + 1];
    float   scales[SEG_LDS_MAX];
};

// All threads of the block must call this (it contains a barrier).
__device__ __forceinline__ void stage_segments(const SegTable& seg, SegLds& lds)
{
    if (seg.n_seg > 0 && seg.n_seg <= SEG_LDS_MAX) {
        for (int t = threadIdx.x; t <= seg.n_seg; t += blockDim.x) lds.offsets[t] = seg.offsets[t];
        for (int t = threadIdx.x; t < seg.n_seg; t += blockDim.x) lds.scales[t] = seg.scales[t];
        __syncthreads();
    }
}

template <typename OffT, typename ScT>
__device__ __forceinline__ f32x4 seg_lookup(const OffT* off, const ScT* sc, int n_seg, int64_t col, int valid, float lr)
{
    // largest s with off[s] <= col
    int lo = 0, hi = n_seg - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (off[mid] <= col) lo = mid; else hi = mid - 1;
    }
    f32x4 out;
    int s = lo;
    out.x = lr * sc[s];
    if (valid > 1) { while (col + 1 >= off[s + 1]) ++s; } out.y = lr * sc[s];
    if (valid > 2) { while (col + 2 >= off[s + 1]) ++s; } out.z = lr * sc[s];
    if (valid > 3) { while (col + 3 >= off[s + 1]) ++s; } out.w = lr * sc[s];
    return out;
}

// Step sizes of the four columns of a quad starting at column `col`.
__device__ __forceinline__ f32x4 quad_lr(const SegTable& seg, const SegLds& lds, int64_t col, int valid, float lr)
{
    if (seg.n_seg == 0) return f32x4{lr, lr, lr, lr};
    if (seg.n_seg <= SEG_LDS_MAX) return seg_lookup(lds.offsets, lds.scales, seg.n_seg, col, valid, lr);
    return seg_lookup(seg.offsets, seg.scales, seg.n_seg, col, valid, lr);
}

// Where column `col` of row 0 sits in a matrix (uniform arithmetic when `col` is).
__device__ __forceinline__ int64_t column_origin(const Geom& geo, int64_t col)
{
    if (geo.block_log2 < 0) return col;
    const int b = geo.block_log2;
    return (((col >> b) * geo.k) << b) + (col & ((static_cast<int64_t>(1) << b) - 1));
}

// Quad geometry of a thread.  Matrix addresses are formed as
//   (array + row * rs + mat)  +  lane_col
// with the first part uniform over the workgroup (scalar registers, scalar
// arithmetic) and only the small lane offset per thread, so that row accesses
// compile to scalar-base + 32-bit-offset global loads and stores.  The shared
// vectors (h, xstar, center) are plain arrays indexed by `col`.
struct Quad {
    int64_t  tile_col;   // first column of the workgroup's tile (uniform)
    int64_t  mat;        // where that column of row 0 sits in a matrix (uniform)
    uint32_t lane_col;   // this thread's first column inside the tile
    int64_t  col;        // tile_col + lane_col
    int      valid;      // 0 (no work), 1..3 (ragged tail) or 4
};

// Vectors only (no matrix in sight): `mat` is the column itself.
__device__ __forceinline__ Quad quad_of_tile(int64_t tile, int64_t d)
{
    Quad out;
    out.tile_col = tile * (BLOCK * 4);
    out.mat = out.tile_col;
    out.lane_col = threadIdx.x * 4u;
    out.col = out.tile_col + out.lane_col;
    const int64_t left = d - out.col;
    out.valid = left >= 4 ? 4 : (left > 0 ? static_cast<int>(left) : 0);
    return out;
}

__device__ __forceinline__ Quad quad_of_tile(int64_t tile, const Geom& geo)
{
    Quad out = quad_of_tile(tile, geo.d);
    out.mat = column_origin(geo, out.tile_col);
    return out;
}

// One tile per workgroup, tile = workgroup index (the cold kernels).
__device__ __forceinline__ Quad my_quad(int64_t d) { return quad_of_tile(static_cast<int64_t>(blockIdx.x), d); }
__device__ __forceinline__ Quad my_quad(const Geom& geo) { return quad_of_tile(static_cast<int64_t>(blockIdx.x), geo); }

// Persistent workgroups for the streaming kernels.  A launch has far fewer
// workgroups than tiles (about one per compute unit); each pulls the next
// 1024-column tile from a device-wide ticket counter until none are left.
// Two reasons, both measured: (i) tiles are handed out in address order to
// whichever compute unit is free, so the chip finishes together (a static
// tile-to-workgroup map left half the XCDs idle for the last 8 % of the
// kernel); (ii) with k rows per tile, few concurrent tiles keep the set of
// DRAM pages in use small, which the HBM controller rewards.
//   tickets[0] = next tile, tickets[1] = workgroups that have finished.
// One tile per ticket, whatever k: handing out 2, 4 or 8 consecutive tiles per ticket (to spread the ticket's
// round trip over more work when k is small) was 3-12 % slower at every k from 4 to 32, and so was splitting the
// tiles into one contiguous band per XCD with a counter each: the narrower the front of tiles in flight, the
// better the memory system does.
// The last workgroup out zeroes both, so a launch leaves them as it found them.
// Every workgroup leaves the loop after exactly one failed fetch, so the grid
// always drains.  `body(tile)` must not return early for part of a workgroup.
template <typename Body>
__device__ __forceinline__ void for_each_tile(const Persist& p, uint32_t n_tiles, Body&& body)
{
    __shared__ uint32_t s_tile;
    uint32_t* __restrict__ tickets = p.tickets;
    for (;;) {
        if (threadIdx.x == 0) s_tile = atomicAdd(&tickets[0], 1u);
        __syncthreads();
        const uint32_t tile = s_tile;
        __syncthreads();
        if (tile >= n_tiles) break;
        body(tile);
    }
    if (threadIdx.x == 0) {
        const uint32_t finished = atomicAdd(&tickets[1], 1u);
        if (finished == gridDim.x - 1) {
            atomicExch(&tickets[0], 0u);
            atomicExch(&tickets[1], 0u);
        }
    }
}

// Row batches.  Rows are fetched U at a time: all loads of a batch are issued before the first dependent
// instruction, and the k % U leftover rows run through a batch of one, so the batch loop has no conditionals.
// Runs body(Count<U>, t) for full batches and body(Count<1>, t) for the rest.
template <int N> using Count = std::integral_constant<int, N>;

template <int U, typename Body>
__device__ __forceinline__ void for_row_batches(int k, Body&& body)
{
    int t = 0;
    for (; t + U <= k; t += U) body(Count<U>{}, t);
    for (; t < k; ++t) body(Count<1>{}, t);
}

// True when every thread of the workgroup owns a full quad (uniform test), so
// the body can be compiled without any per-lane tail handling.
__device__ __forceinline__ bool tile_is_full(const Quad& qd, int64_t d)
{
    return qd.tile_col + static_cast<int64_t>(BLOCK) * 4 <= d;
}

inline int64_t num_quads(int64_t d) { return (d + 3) / 4; }
inline unsigned grid_for(int64_t d) { return static_cast<unsigned>((num_quads(d) + BLOCK - 1) / BLOCK); }

// Grid of the plain (one tile of one row per workgroup) kernels: x = tile inside a band of `band` consecutive
// tiles, y = row, z = band; a kernel's tile is blockIdx.z * band + blockIdx.x.  Workgroups are dispatched x
// first, then y: a band's k row pieces follow one another, so what the rows share (h, xstar of the band's
// columns) is still cached, and in the blocked layout, where a band is a block, the sweep is in address order.
// `row_major_band` is the band for row-major matrices (0: the whole row); blocked matrices use it only if it
// divides a block or is a whole number of blocks.
struct FlatGrid {
    dim3     grid;
    unsigned band;
};
inline FlatGrid flat_grid(const Geom& geo, unsigned row_major_band)
{
    const unsigned tiles = grid_for(geo.d);
    unsigned band = row_major_band == 0 ? tiles : row_major_band;
    if (geo.block_log2 >= 0) {
        // a block, or the requested band if it is a whole part or a whole multiple of one
        const unsigned per_block = static_cast<unsigned>(geo.rs / (BLOCK * 4));
        const bool fits = row_major_band != 0 && (per_block % row_major_band == 0 || row_major_band % per_block == 0);
        band = fits ? row_major_band : per_block;
    }
    if (band > tiles) band = tiles;
    unsigned bands = (tiles + band - 1) / band;
    if (bands > 65535u) {                                  // the grid's z extent is 16 bits: whole multiples of a band
        const unsigned per = (bands + 65534u) / 65535u;
        band *= per;
        bands = (tiles + band - 1) / band;
    }
    return FlatGrid{dim3(band, static_cast<unsigned>(geo.k), bands), band};
}

}  // namespace gsgd

// Gossip in two ascending sweeps over the rows of a tile: the form of the pull,
// push and stale-parameter rules (Section 3.1, Algorithms 3-4, Section 6.2 of
// the paper) on blocked matrices, and on short vectors in either layout.  The
// walks along the peer map, all-reduce, elastic averaging and the local step
// are in kernels_step.hip.
#include "device_common.hpp"

namespace gsgd {

// ---------------------------------------------------------------------------
// Gossip as two sweeps (the form for blocked matrices).  The cycle walk above
// visits the rows in the order of the peer map, i.e. in a random order; in the
// blocked layout the k row pieces of a tile are neighbours in memory, and the
// memory system serves them markedly faster when they are visited in address
// order (one sequential stream per block instead of jumps inside it).  So the
// rows are visited in ascending order twice:
//   sweep 1: load x, v, g of a row, take the local step, store v, park the
//            row's x' in LDS;
//   sweep 2: finish every row from its own and its peer's parked values and
//            store x.
// The stale-parameter rule mixes the x from before the local step, so there
// sweep 1 only loads and parks x, and sweep 2 loads v and g, takes the local
// step from the parked x, mixes with the peer's parked x and stores v and x:
// one parked value per row in either rule.
// Each of x, v, g is still read once and x, v written once (20 bytes per
// replica-element); the parked values cost 16 bytes of LDS per thread and row.
// Any peer map works (no cycles or trees to follow).
//
// SPLIT = false: a workgroup owns a 1024-column tile, a thread parks its own
// quads of all k rows (rows <= ROWS, ROWS * 4 KiB of LDS, no barrier at all).
// SPLIT = true: a workgroup owns a tile of CG x 256 columns; CG wavefronts
// side by side cover its columns, and the rows are shared out equally among
// the rows of wavefronts (ROWS x CG KiB of LDS, one barrier between the
// sweeps).  CG = 1, four wavefronts or more (see sweep_block): the form for
// many replicas.  CG = 4, eight wavefronts: a whole 1024-column tile for the
// kernels whose arithmetic one wavefront per SIMD does not hide.
constexpr int SWEEP_SPLIT_COLUMNS = 256;
// Threads per workgroup.  Of the split form for the most rows only one workgroup fits a compute unit's LDS, and four
// wavefronts (one per SIMD) leave the arithmetic of a sweep uncovered; the rows are split over however many
// wavefronts there are, so these kernels run with 8 (12 with the generator fused, where 8 and 4 are level).  Blocks
// of 16 Ki columns, ResNet-50 length, % of the HBM peak with 4 -> 8 wavefronts: push-gossip k = 80 73 -> 81.5,
// k = 128 73 -> 80; stale rule k = 128 80.5 -> 83; plain gossip k = 128 80.5 -> 81.5 (k = 80 level); 4 -> 12 with the
// generator fused: k = 80 74 -> 79, k = 128 76 -> 78.5 (12 lose 2-3 points in the others; 16 spill registers).
constexpr int SWEEP_ROWS_ONE_PER_CU = 65;          // parking space from which only one workgroup fits
// Whole 1024-column tiles for the kernels with arithmetic to hide, beyond the 16 rows of which two workgroups fit:
// SWEEP_WIDE_GROUPS wavefronts side by side cover the tile's columns, and two such rows of wavefronts take half of
// the tile's rows each (eight wavefronts, one barrier between the sweeps, the same LDS as a thread per quad).
// % of the HBM peak, a thread per quad -> this form: generator-fused gossip k = 24 82 -> 84.6, k = 32 83.5 -> 84.4;
// push-gossip k = 18 78.8 -> 81.4.  The kernels that read g and do little else lose 1.5-2.5 points and keep a
// thread per quad.
constexpr int SWEEP_WIDE_GROUPS = 4;
constexpr int sweep_block(bool split, int rows, bool fused_gossip, int column_groups)
{
    if (column_groups > 1) return 2 * column_groups * 64;
    return split && rows >= SWEEP_ROWS_ONE_PER_CU ? (fused_gossip ? 12 : 8) * 64 : BLOCK;
}

template <bool SPLIT, bool FULL, int ROWS, int U, bool FUSED_GEN, int NOISE, bool EXT, bool STALE, bool PUSH = false,
          int CG = 1>
__device__ __forceinline__
void gossip_sweep_body(const Geom& geo, const Hyper& hp, const SegTable& seg, const SegLds& lds,
                       int64_t tile_col, int64_t mat, float neg_beta, const Walk& peers, const Walk& senders,
                       f32x4* __restrict__ park_key,
                       float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                       const float* __restrict__ h, const float* __restrict__ xstar,
                       float sigma, RngKey key, uint32_t step)
{
    constexpr int SLOTS = SPLIT ? 64 * CG : BLOCK;              // parked quads per row
    const int slot = SPLIT ? static_cast<int>(((threadIdx.x >> 6) % CG) * 64u + (threadIdx.x & 63u))
                           : static_cast<int>(threadIdx.x);
    const uint32_t lane_col = static_cast<uint32_t>(slot) * 4u;
    const int64_t col = tile_col + lane_col;
    const int64_t left = geo.d - col;
    const int valid = FULL ? 4 : (left >= 4 ? 4 : (left > 0 ? static_cast<int>(left) : 0));
    // rows of this thread: all of them, or its wavefront's share
    int r0 = 0, r1 = geo.k;
    if constexpr (SPLIT) {
        const int wave = static_cast<int>(threadIdx.x >> 6) / CG;          // CG wavefronts side by side share rows
        const int waves = static_cast<int>(blockDim.x >> 6) / CG;
        const int per = (geo.k + waves - 1) / waves;
        r0 = wave * per < geo.k ? wave * per : geo.k;
        r1 = r0 + per < geo.k ? r0 + per : geo.k;
    }
    if (FULL || valid > 0) {
        const f32x4 neg_lr = -quad_lr(seg, lds, col, valid, hp.lr);
        f32x4 h4 = {0.f, 0.f, 0.f, 0.f}, xs4 = {0.f, 0.f, 0.f, 0.f};
        if constexpr (FUSED_GEN) {
            h4 = load_quad_cached<FULL>(h + col, valid);
            xs4 = load_quad_cached<FULL>(xstar + col, valid);
        }
        const uint32_t quad_index = static_cast<uint32_t>(col >> 2);
        int i0 = r0;
        // rows i0 .. i0 + N - 1: X (and V, G unless STALE) in, local step, v out, x' parked; STALE: X in and parked
        auto batch = [&](auto n) {
            constexpr int N = decltype(n)::value;
            f32x4 X[N], V[N], G[N];
#pragma unroll
            for (int u = 0; u < N; ++u) {
                const int64_t off = static_cast<int64_t>(i0 + u) * geo.rs + mat;
                X[u] = load_quad<FULL>(x + off + lane_col, valid);
                if constexpr (!STALE) V[u] = load_quad<FULL>(v + off + lane_col, valid);
                if constexpr (!STALE && !FUSED_GEN) G[u] = load_quad<FULL>(g + off + lane_col, valid);
            }
#pragma unroll
            for (int u = 0; u < N; ++u) {
                const int row = i0 + u;
                if constexpr (STALE) {
                    park_key[row * SLOTS + slot] = X[u];
                } else {
                    const int64_t off = static_cast<int64_t>(row) * geo.rs + mat;
                    if constexpr (FUSED_GEN) {
                        const f32x4 xi = noise4<NOISE>(philox4x32_10(quad_index, static_cast<uint32_t>(row), step,
                                                                     STREAM_GRAD, key.k0, key.k1));
                        const f32x4 t1 = X[u] - xs4;
                        const f32x4 t2 = sigma * xi;
                        G[u] = fma4(h4, t1, t2);
                    }
                    f32x4 vn, post;
                    local_step<EXT>(X[u], V[u], G[u], neg_lr, hp, vn, post);
                    store_quad<FULL>(v + off + lane_col, vn, valid);
                    park_key[row * SLOTS + slot] = post;
                }
            }
            i0 += N;
        };
        constexpr int U1 = STALE ? 2 * U : U;         // the stale rule's first sweep loads x alone: twice the rows
        while (i0 + U1 <= r1) batch(Count<U1>{});
        // the rows left over go out in batches of 8, 4, 2 and 1 rather than one at a time
        if constexpr (U1 > 8) { if (i0 + 8 <= r1) batch(Count<8>{}); }
        if constexpr (U1 > 4) { if (i0 + 4 <= r1) batch(Count<4>{}); }
        if constexpr (U1 > 2) { if (i0 + 2 <= r1) batch(Count<2>{}); }
        if (i0 < r1) batch(Count<1>{});
    }
    if constexpr (SPLIT) __syncthreads();             // a row's peer may be parked by another wavefront
    if constexpr (STALE) {
        if (FULL || valid > 0) {
            const f32x4 neg_lr = -quad_lr(seg, lds, col, valid, hp.lr);
            f32x4 h4 = {0.f, 0.f, 0.f, 0.f}, xs4 = {0.f, 0.f, 0.f, 0.f};
            if constexpr (FUSED_GEN) {
                h4 = load_quad_cached<FULL>(h + col, valid);
                xs4 = load_quad_cached<FULL>(xstar + col, valid);
            }
            const uint32_t quad_index = static_cast<uint32_t>(col >> 2);
            int i0 = r0;
            // second sweep of the stale rule: V (and G) in, local step from the parked x, mix with the peer's parked x, v and x out
            auto stale_batch = [&](auto n) {
                constexpr int N = decltype(n)::value;
                f32x4 V[N], G[N];
#pragma unroll
                for (int u = 0; u < N; ++u) {
                    const int64_t off = static_cast<int64_t>(i0 + u) * geo.rs + mat;
                    V[u] = load_quad<FULL>(v + off + lane_col, valid);
                    if constexpr (!FUSED_GEN) G[u] = load_quad<FULL>(g + off + lane_col, valid);
                }
#pragma unroll
                for (int u = 0; u < N; ++u) {
                    const int row = i0 + u;
                    const int64_t off = static_cast<int64_t>(row) * geo.rs + mat;
                    const f32x4 mine = park_key[row * SLOTS + slot];
                    const f32x4 theirs = park_key[static_cast<int>(peers.seq[row]) * SLOTS + slot];
                    if constexpr (FUSED_GEN) {
                        const f32x4 xi = noise4<NOISE>(philox4x32_10(quad_index, static_cast<uint32_t>(row), step, STREAM_GRAD,
                                                                     key.k0, key.k1));
                        const f32x4 t1 = mine - xs4;
                        const f32x4 t2 = sigma * xi;
                        G[u] = fma4(h4, t1, t2);
                    }
                    f32x4 vn, post;
                    local_step<EXT>(mine, V[u], G[u], neg_lr, hp, vn, post);
                    store_quad<FULL>(v + off + lane_col, vn, valid);
                    store_quad<FULL>(x + off + lane_col, mix_keys(post, mine, theirs, neg_beta), valid);
                }
                i0 += N;
            };
            while (i0 + U <= r1) stale_batch(Count<U>{});
            if constexpr (U > 4) { if (i0 + 4 <= r1) stale_batch(Count<4>{}); }
            if constexpr (U > 2) { if (i0 + 2 <= r1) stale_batch(Count<2>{}); }
            if (i0 < r1) stale_batch(Count<1>{});
        }
        return;
    }
    if (FULL || valid > 0) {
        for (int row = r0; row < r1; ++row) {
            const f32x4 mine = park_key[row * SLOTS + slot];
            f32x4 out;
            if constexpr (PUSH) {
                // Algorithm 4: the average of the row's own x' and of every x' sent to it, summed in fp64, own
                // value first, then the senders in ascending index.  peers.seq[row] = the first sender (bits 0-9: most
                // rows that receive anything have one, and need no second lookup), the place of the row's group
                // in `senders` (bits 10-19) and how many senders there are (bits 20-29).
                const uint32_t word = peers.seq[row];
                const uint32_t first = word & 0x3FFu, start = (word >> 10) & 0x3FFu, count = word >> 20;
                f64x4 sum = widen(mine);
                if (count > 0) sum = sum + widen(park_key[static_cast<int>(first) * SLOTS + slot]);
                for (uint32_t t = 1; t < count; ++t)
                    sum = sum + widen(park_key[static_cast<int>(senders.seq[start + t]) * SLOTS + slot]);
                out = count == 0 ? mine : average(sum, count + 1u);
            } else {
                const f32x4 theirs = park_key[static_cast<int>(peers.seq[row]) * SLOTS + slot];
                out = mix_keys(mine, mine, theirs, neg_beta);
            }
            store_quad<FULL>(x + static_cast<int64_t>(row) * geo.rs + mat + lane_col, out, valid);
        }
    }
}

// `peers.seq[i]` is the plain index of the row that row i mixes with.  n_tiles counts tiles of the kernel's own
// width (1024 columns, or 256 when SPLIT).  Needs k <= ROWS (checked by the launcher).
template <bool SPLIT, int ROWS, int U, bool FUSED_GEN, int NOISE, bool EXT, bool STALE, int CG = 1>
__global__ __launch_bounds__(sweep_block(SPLIT, ROWS, FUSED_GEN, CG))
void gossip_sweep_kernel(Geom geo, Hyper hp, SegTable seg, float neg_beta, Walk peers,
                         float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                         const float* __restrict__ h, const float* __restrict__ xstar,
                         float sigma, RngKey key, uint32_t step, Persist pst, uint32_t n_tiles)
{
    constexpr int SLOTS = SPLIT ? 64 * CG : BLOCK;
    constexpr int TILE_COLUMNS = SPLIT ? SWEEP_SPLIT_COLUMNS * CG : BLOCK * 4;
    __shared__ SegLds lds;
    __shared__ f32x4 park_key[ROWS * SLOTS];
    stage_segments(seg, lds);
    for_each_tile(pst, n_tiles, [&](uint32_t tile) {
        const int64_t tile_col = static_cast<int64_t>(tile) * TILE_COLUMNS;
        const int64_t mat = column_origin(geo, tile_col);
        // every thread takes the same branch (the barrier inside the body is reached by all or by none)
        if (tile_col + TILE_COLUMNS <= geo.d)
            gossip_sweep_body<SPLIT, true, ROWS, U, FUSED_GEN, NOISE, EXT, STALE, false, CG>(
                geo, hp, seg, lds, tile_col, mat, neg_beta, peers, peers, park_key, x, v, g, h, xstar, sigma, key,
                step);
        else
            gossip_sweep_body<SPLIT, false, ROWS, U, FUSED_GEN, NOISE, EXT, STALE, false, CG>(
                geo, hp, seg, lds, tile_col, mat, neg_beta, peers, peers, park_key, x, v, g, h, xstar, sigma, key,
                step);
    });
}

// Push-gossip (Algorithm 4) in the same two sweeps: sweep 2 averages what a row received.  `index.seq[r]` = row r's
// first sender (bits 0-9), the place of its group in `senders` (bits 10-19) and the number of its senders (bits
// 20-29); `senders.seq` lists the senders of row 0, then of row 1, ..., each group in ascending order, self-sends
// left out.
template <bool SPLIT, int ROWS, int U, bool FUSED_GEN, int NOISE, bool EXT, int CG = 1>
__global__ __launch_bounds__(sweep_block(SPLIT, ROWS, false, CG))
void push_sweep_kernel(Geom geo, Hyper hp, SegTable seg, Walk index, Walk senders,
                       float* __restrict__ x, float* __restrict__ v, const float* __restrict__ g,
                       const float* __restrict__ h, const float* __restrict__ xstar,
                       float sigma, RngKey key, uint32_t step, Persist pst, uint32_t n_tiles)
{
    constexpr int SLOTS = SPLIT ? 64 * CG : BLOCK;
    constexpr int TILE_COLUMNS = SPLIT ? SWEEP_SPLIT_COLUMNS * CG : BLOCK * 4;
    __shared__ SegLds lds;
    __shared__ f32x4 park_key[ROWS * SLOTS];
    stage_segments(seg, lds);
    for_each_tile(pst, n_tiles, [&](uint32_t tile) {
        const int64_t tile_col = static_cast<int64_t>(tile) * TILE_COLUMNS;
        const int64_t mat = column_origin(geo, tile_col);
        if (tile_col + TILE_COLUMNS <= geo.d)
            gossip_sweep_body<SPLIT, true, ROWS, U, FUSED_GEN, NOISE, EXT, false, true, CG>(
                geo, hp, seg, lds, tile_col, mat, 0.0f, index, senders, park_key, x, v, g, h, xstar, sigma, key,
                step);
        else
            gossip_sweep_body<SPLIT, false, ROWS, U, FUSED_GEN, NOISE, EXT, false, true, CG>(
                geo, hp, seg, lds, tile_col, mat, 0.0f, index, senders, park_key, x, v, g, h, xstar, sigma, key,
                step);
    });
}

// Rows in flight per thread in the first sweep.
#ifndef GSGD_SWEEP_ROWS_IN_FLIGHT
#define GSGD_SWEEP_ROWS_IN_FLIGHT 4
#endif
constexpr int SWEEP_RIF = GSGD_SWEEP_ROWS_IN_FLIGHT;
// With the generator fused and the rows split over the wavefronts a deeper batch hides the generator's arithmetic
// behind the loads (k = 128: 76.7 % of the HBM peak with 8 rows against 73.7 % with 4; k = 32 and the kernels that
// read g: 4 is best or tied, 3 / 5 / 6 / 8 rows 81.8 / 81.2 / 81.9 / 80.1 % against 83.0 % at the benchmark shape).
// Issuing the next batch's loads before the generator works on the current one (two register sets in turn) does not
// help: level at k = 16 and 32, 5-10 points worse at k = 64 and 128.
constexpr int SWEEP_RIF_FUSED_SPLIT = 8;
// Whole tiles with g read from memory: two rows in flight are half a point to a point ahead of four at k = 8, 16, 32
// (84.0 against 83.4 % at the benchmark shape); with the generator fused two lose 7 points.
constexpr int SWEEP_RIF_WHOLE = 2;
// Push-gossip with g read from memory: two rows in flight a point ahead of four at k = 32, level at k = 16.  One row
// in flight loses 8-10 points in every kernel.
constexpr int SWEEP_RIF_PUSH = 2;
// The stale rule: rows of v and g in flight in its second sweep; its first sweep, which loads x alone, takes twice
// as many.  Whole tiles: 2 and 4 level, 1 loses 13 points; split tiles: 8 a point ahead of 4 at k = 40 and 64, level
// at k = 128, 2 loses 4-6 points.
constexpr int SWEEP_RIF_STALE_WHOLE = 2, SWEEP_RIF_STALE_SPLIT = 8;
constexpr int SWEEP_RIF_WIDE = 2;                 // whole tiles under eight wavefronts: 2 a point ahead of 4
constexpr int sweep_rif(bool split, bool fused, bool stale, int column_groups)
{
    if (column_groups > 1) return SWEEP_RIF_WIDE;
    if (stale && !fused) return split ? SWEEP_RIF_STALE_SPLIT : SWEEP_RIF_STALE_WHOLE;
    if (split && fused) return SWEEP_RIF_FUSED_SPLIT;
    if (!split && !fused) return SWEEP_RIF_WHOLE;
    return SWEEP_RIF;
}
// Parking space compiled in (rows): what fits the 160 KiB of LDS beside the segment table.
constexpr int SWEEP_ROWS_WHOLE = 36, SWEEP_ROWS_WHOLE_FEW = 16;             // 1024-column tiles: 4 KiB per row
constexpr int SWEEP_ROWS_SPLIT_FEW = 48, SWEEP_ROWS_SPLIT = 144;            // 256-column tiles: 1 KiB
// The largest forms that leave room for two workgroups per compute unit (64 KiB + the 12 KiB segment table, twice,
// in 160 KiB), which the kernels with arithmetic to hide want: push-gossip's averaging, the fused generator.
// SWEEP_ROWS_WHOLE_FEW is the same for whole tiles.
constexpr int SWEEP_ROWS_SPLIT_MID = 64;

// Most rows for which two workgroups of the split push kernel fit one compute unit's LDS.
int sweep_rows_two_per_cu(bool split) { return split ? SWEEP_ROWS_SPLIT_MID : SWEEP_ROWS_WHOLE_FEW; }

int sweep_capacity(bool split) { return split ? SWEEP_ROWS_SPLIT : SWEEP_ROWS_WHOLE; }

// The gossip step in its two-sweep form; `fused` takes g from the generator (h, xstar, sigma, key, step) instead
// of reading it.  The caller has checked geo.k <= sweep_capacity(split).
hipError_t launch_step_gossip_sweep(const Geom& geo, const Hyper& hp, const SegTable& seg, float beta, const Walk& peers,
                                    bool stale, bool split, bool fused, float* x, float* v, const float* g,
                                    const float* h, const float* xstar, float sigma, RngKey key, uint32_t step,
                                    int noise_kind, Persist p, hipStream_t stream)
{
    const uint32_t tiles = split ? static_cast<uint32_t>((geo.d + SWEEP_SPLIT_COLUMNS - 1) / SWEEP_SPLIT_COLUMNS)
                                 : grid_for(geo.d);
    const unsigned width = p.workgroups < tiles ? (p.workgroups ? p.workgroups : 1u) : tiles;
#define GSGD_SWEEP(SPLIT, ROWS, CG, FUSED, NOISE, EXT, STALE) \
    hipLaunchKernelGGL((gossip_sweep_kernel<SPLIT, ROWS, sweep_rif(SPLIT, FUSED, STALE, CG), FUSED, NOISE, EXT, STALE, CG>), \
                       dim3(width), dim3(sweep_block(SPLIT, ROWS, FUSED, CG)), 0, \
                       stream, geo, hp, seg, -beta, peers, x, v, g, h, xstar, sigma, key, step, p, tiles)
    // the extended local step covers the plain one (no weight decay, heavy ball) wherever only one is compiled
#define GSGD_SWEEP_GIVEN_G(SPLIT, ROWS) \
    do { \
        if (stale) GSGD_SWEEP(SPLIT, ROWS, 1, false, 0, true, true); \
        else if (hp.extended()) GSGD_SWEEP(SPLIT, ROWS, 1, false, 0, true, false); \
        else GSGD_SWEEP(SPLIT, ROWS, 1, false, 0, false, false); \
    } while (0)
#define GSGD_SWEEP_FUSED(SPLIT, ROWS, CG) \
    do { \
        if (noise_kind == GSGD_NOISE_UNIFORM) { \
            if (stale) GSGD_SWEEP(SPLIT, ROWS, CG, true, GSGD_NOISE_UNIFORM, true, true); \
            else GSGD_SWEEP(SPLIT, ROWS, CG, true, GSGD_NOISE_UNIFORM, true, false); \
        } else { \
            if (stale) GSGD_SWEEP(SPLIT, ROWS, CG, true, GSGD_NOISE_GAUSSIAN, true, true); \
            else GSGD_SWEEP(SPLIT, ROWS, CG, true, GSGD_NOISE_GAUSSIAN, true, false); \
        } \
    } while (0)
#define GSGD_SWEEP_EITHER(SPLIT, ROWS) \
    do { if (fused) GSGD_SWEEP_FUSED(SPLIT, ROWS, 1); else GSGD_SWEEP_GIVEN_G(SPLIT, ROWS); } while (0)
    if (!split && geo.k <= SWEEP_ROWS_WHOLE_FEW) GSGD_SWEEP_EITHER(false, SWEEP_ROWS_WHOLE_FEW);
    else if (!split && fused) GSGD_SWEEP_FUSED(true, SWEEP_ROWS_WHOLE, SWEEP_WIDE_GROUPS);     // whole tiles, eight wavefronts
    else if (!split) GSGD_SWEEP_GIVEN_G(false, SWEEP_ROWS_WHOLE);
    else if (geo.k <= SWEEP_ROWS_SPLIT_FEW) GSGD_SWEEP_EITHER(true, SWEEP_ROWS_SPLIT_FEW);
    else if (geo.k <= SWEEP_ROWS_SPLIT_MID) GSGD_SWEEP_EITHER(true, SWEEP_ROWS_SPLIT_MID);
    else GSGD_SWEEP_EITHER(true, SWEEP_ROWS_SPLIT);
#undef GSGD_SWEEP_EITHER
#undef GSGD_SWEEP_FUSED
#undef GSGD_SWEEP_GIVEN_G
#undef GSGD_SWEEP
    return hipGetLastError();
}

// Push-gossip in the two-sweep form; `index` / `senders` as push_sweep_kernel takes them.  The caller has checked
// geo.k <= sweep_capacity(split).
hipError_t launch_step_gossip_push_sweep(const Geom& geo, const Hyper& hp, const SegTable& seg, const Walk& index,
                                         const Walk& senders, bool split, bool fused, float* x, float* v, const float* g,
                                         const float* h, const float* xstar, float sigma, RngKey key, uint32_t step,
                                         int noise_kind, Persist p, hipStream_t stream)
{
    const uint32_t tiles = split ? static_cast<uint32_t>((geo.d + SWEEP_SPLIT_COLUMNS - 1) / SWEEP_SPLIT_COLUMNS)
                                 : grid_for(geo.d);
    const unsigned width = p.workgroups < tiles ? (p.workgroups ? p.workgroups : 1u) : tiles;
#define GSGD_PUSH_SWEEP(SPLIT, ROWS, CG, FUSED, NOISE, EXT) \
    hipLaunchKernelGGL((push_sweep_kernel<SPLIT, ROWS, (FUSED && CG == 1) ? SWEEP_RIF : SWEEP_RIF_PUSH, FUSED, NOISE, EXT, CG>), \
                       dim3(width), dim3(sweep_block(SPLIT, ROWS, false, CG)), 0, stream, \
                       geo, hp, seg, index, senders, x, v, g, h, xstar, sigma, key, step, p, tiles)
#define GSGD_PUSH_SWEEP_FLAGS(SPLIT, ROWS, CG) \
    do { \
        if (fused && noise_kind == GSGD_NOISE_UNIFORM) GSGD_PUSH_SWEEP(SPLIT, ROWS, CG, true, GSGD_NOISE_UNIFORM, true); \
        else if (fused) GSGD_PUSH_SWEEP(SPLIT, ROWS, CG, true, GSGD_NOISE_GAUSSIAN, true); \
        else if (hp.extended()) GSGD_PUSH_SWEEP(SPLIT, ROWS, CG, false, 0, true); \
        else GSGD_PUSH_SWEEP(SPLIT, ROWS, CG, false, 0, false); \
    } while (0)
    if (!split && geo.k <= SWEEP_ROWS_WHOLE_FEW) GSGD_PUSH_SWEEP_FLAGS(false, SWEEP_ROWS_WHOLE_FEW, 1);
    else if (!split) GSGD_PUSH_SWEEP_FLAGS(true, SWEEP_ROWS_WHOLE, SWEEP_WIDE_GROUPS);          // whole tiles, eight wavefronts
    else if (geo.k <= SWEEP_ROWS_SPLIT_FEW) GSGD_PUSH_SWEEP_FLAGS(true, SWEEP_ROWS_SPLIT_FEW, 1);
    else if (geo.k <= SWEEP_ROWS_SPLIT_MID) GSGD_PUSH_SWEEP_FLAGS(true, SWEEP_ROWS_SPLIT_MID, 1);
    else GSGD_PUSH_SWEEP_FLAGS(true, SWEEP_ROWS_SPLIT, 1);
#undef GSGD_PUSH_SWEEP_FLAGS
#undef GSGD_PUSH_SWEEP
    return hipGetLastError();
}

}  // namespace gsgd

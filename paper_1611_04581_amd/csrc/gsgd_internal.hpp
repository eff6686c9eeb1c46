// Host-side declarations shared by the translation units of libgsgd.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gsgd.h"

namespace gsgd {

// Replica visiting order of the gossip kernel, carried in the kernel-argument
// block (uniform for the whole grid, so it lives in scalar registers).
// Entries are whole dwords so that the kernel fetches them with scalar loads
// (a sub-dword element would be fetched per lane through the vector memory
// path and its wait would drain every row load still in flight).
constexpr uint32_t WALK_ROW_MASK = 0x0FFF;
constexpr uint32_t WALK_FIRST    = 0x4000;   // first member of a cycle
constexpr uint32_t WALK_LAST     = 0x8000;   // last member of a cycle
// General pull maps (several replicas may pull from the same one) add tree
// nodes hanging off the cycles.  A tree node's peer is its parent, which was
// visited earlier; the kernel keeps the parent's value in a register `par`
// and is told per entry how to maintain it:
//   restore (before use): par <- the last cycle node's value, or <- stack slot
//   descend (after use) : par <- this node's value (its children follow)
//   save    (with descend): stack slot <- par first (a sibling subtree follows)
// The stack lives in LDS, one 16-byte lane per thread and slot.
constexpr uint32_t WALK_TREE          = 0x2000;    // not on a cycle: finished as soon as it is loaded
constexpr uint32_t WALK_DESCEND       = 0x1000;
constexpr uint32_t WALK_RESTORE_SHIFT = 16;        // bits 16..17: 0 keep par, 1 from the cycle register, 2 from a slot
constexpr uint32_t WALK_RESTORE_PREV  = 1u << WALK_RESTORE_SHIFT;
constexpr uint32_t WALK_RESTORE_SLOT  = 2u << WALK_RESTORE_SHIFT;
constexpr uint32_t WALK_RESTORE_MASK  = 3u << WALK_RESTORE_SHIFT;
constexpr uint32_t WALK_SAVE          = 0x40000;   // bit 18
constexpr uint32_t WALK_SLOT_SHIFT    = 20;        // bits 20..23: the slot restored from or saved to
constexpr uint32_t WALK_SLOT_MASK     = 0xFu << WALK_SLOT_SHIFT;
// Children are visited so that the subtree needing most slots comes last and
// reuses its parent's slot; a subtree that needs s slots then has at least
// 3 * 2^s - 1 nodes, so 8 slots cover every map on up to GSGD_MAX_K replicas.
constexpr int      WALK_SLOTS         = 8;
// Push-gossip (Algorithm 4) visits children before parents: a node's new value
// is the average of its own x' and the x' of every node that sent to it.  The
// kernel keeps the running sum of the node being assembled in `acc`; an entry
// says how the visited node's x' joins its receiver's sum:
//   START        acc <- x'                 (first sender visited)
//   ADD          acc <- acc + x'
//   RESTORE_ADD  acc <- stack slot + x'    (a subtree in between used acc)
// and whether acc is then saved to the slot because such a subtree comes next.
constexpr uint32_t PUSH_HAS_SENDERS  = 0x1000;    // acc holds the sum of this node's (tree) senders
constexpr uint32_t PUSH_MODE_SHIFT   = 16;
constexpr uint32_t PUSH_START        = 1u << PUSH_MODE_SHIFT;
constexpr uint32_t PUSH_ADD          = 2u << PUSH_MODE_SHIFT;
constexpr uint32_t PUSH_RESTORE_ADD  = 3u << PUSH_MODE_SHIFT;
constexpr uint32_t PUSH_MODE_MASK    = 3u << PUSH_MODE_SHIFT;
constexpr uint32_t PUSH_SAVE_AFTER   = 0x40000;   // bit 18
constexpr uint32_t PUSH_SLOT_SHIFT   = 19;        // bits 19..21
constexpr uint32_t PUSH_SLOT_MASK    = 7u << PUSH_SLOT_SHIFT;
constexpr uint32_t PUSH_COUNT_SHIFT  = 22;        // bits 22..31: number of values averaged (1 + senders)
struct Walk {
    uint32_t seq[GSGD_MAX_K];
};

// Per-layer tensor table on the device (n_seg == 0: flat, pointers unused).
struct SegTable {
    const int64_t* offsets;   // n_seg + 1
    const float*   scales;    // n_seg
    int32_t        n_seg;
};

// Problem geometry common to every kernel.  A matrix holds k rows of ld
// columns in k * ld elements; element (i, j) sits at  origin(j) + i * rs.
//   row-major:  origin(j) = j,  rs = ld;
//   blocked (blocks of B = 2^block_log2 columns, a block holding its k row
//   pieces back to back):  origin(j) = (j / B) * k * B + j % B,  rs = B.
// B is a multiple of every tile width, so a tile never straddles a block.
struct Geom {
    int32_t k;
    int32_t block_log2;   // -1: row-major
    int64_t d;
    int64_t ld;
    int64_t rs;           // distance between rows i and i + 1 of a column
};

// block_columns == 0: row-major; otherwise a power of two (checked by the caller).
inline Geom make_geom(int32_t k, int64_t d, int64_t ld, int64_t block_columns)
{
    if (block_columns <= 0) return Geom{k, -1, d, ld, ld};
    int32_t lg = 0;
    while ((static_cast<int64_t>(1) << lg) < block_columns) ++lg;
    return Geom{k, lg, d, ld, block_columns};
}

// Step size, momentum, and the two extras of the experiments' local step
// (Section 4.2): weight decay and the Nesterov flag.  Kernels compiled without
// the extras ignore wd and nesterov.
struct Hyper {
    float   lr, mu, wd;
    int32_t nesterov;
    bool    extended() const { return wd != 0.0f || nesterov != 0; }
};

// Philox key and the per-call counter words.
struct RngKey {
    uint32_t k0, k1;
};

// How a streaming kernel is launched: `workgroups` persistent workgroups that
// pull tiles through the two ticket words at `tickets` (device memory, both
// zero between launches).
struct Persist {
    uint32_t* tickets;
    unsigned  workgroups;
};

// ---- launchers (defined next to their kernels) ---------------------------
hipError_t launch_step_gossip(const Geom&, const Hyper&, const SegTable&, float beta, const Walk&, bool stale,
                              bool has_trees, float* x, float* v, const float* g, Persist, hipStream_t);
hipError_t launch_step_gossip_push(const Geom&, const Hyper&, const SegTable&, const Walk&,
                                   float* x, float* v, const float* g, Persist, hipStream_t);
hipError_t launch_async_tick(const Geom&, const Hyper&, const SegTable&, float beta, int32_t i, int32_t j,
                             float* x, float* v, const float* g, hipStream_t);
hipError_t launch_async_tick_fused(const Geom&, const Hyper&, const SegTable&, float beta, int32_t i, int32_t j,
                                   float* x, float* v, const float* h, const float* xstar,
                                   float sigma, RngKey key, uint32_t tick, int noise_kind, hipStream_t);
hipError_t launch_easgd_tick(const Geom&, const Hyper&, const SegTable&, float alpha_e, int32_t i,
                             float* x, float* v, const float* g, float* center, hipStream_t);
// Persist with tickets: persistent workgroups walking the rows; without (tickets == nullptr): the plain banded grid
hipError_t launch_step_local(const Geom&, const Hyper&, const SegTable&, float* x, float* v, const float* g,
                             unsigned band_tiles, Persist, hipStream_t);
int        sweep_capacity(bool split);                   // most replicas the two-sweep gossip kernels can park
int        sweep_rows_two_per_cu(bool split);   // most replicas for which two workgroups fit a compute unit's LDS
hipError_t launch_step_gossip_push_sweep(const Geom&, const Hyper&, const SegTable&, const Walk& index,
                                         const Walk& senders, bool split, bool fused, float* x, float* v, const float* g,
                                         const float* h, const float* xstar, float sigma, RngKey key, uint32_t step,
                                         int noise_kind, Persist, hipStream_t);
hipError_t launch_step_gossip_sweep(const Geom&, const Hyper&, const SegTable&, float beta, const Walk& peers,
                                    bool stale, bool split, bool fused, float* x, float* v, const float* g,
                                    const float* h, const float* xstar, float sigma, RngKey key, uint32_t step,
                                    int noise_kind, Persist, hipStream_t);
hipError_t launch_step_gossip_fused(const Geom&, const Hyper&, const SegTable&, float beta, const Walk&, bool stale,
                                    bool has_trees, float* x, float* v, const float* h, const float* xstar,
                                    float sigma, RngKey key, uint32_t step, int noise_kind, Persist, hipStream_t);
hipError_t launch_step_gossip_push_fused(const Geom&, const Hyper&, const SegTable&, const Walk&,
                                         float* x, float* v, const float* h, const float* xstar,
                                         float sigma, RngKey key, uint32_t step, int noise_kind, Persist, hipStream_t);
hipError_t launch_step_allreduce(const Geom&, const Hyper&, const SegTable&, float* x, float* v, const float* g,
                                 Persist, bool row_split, hipStream_t);
hipError_t launch_step_easgd(const Geom&, const Hyper&, const SegTable&, float alpha_e,
                             float* x, float* v, const float* g, float* center, Persist, bool row_split, hipStream_t);
// band_tiles: 1024-column tiles per band of the plain grid, 0 = the default
// Persist with tickets: persistent workgroups walking the rows; without (tickets == nullptr): the plain banded grid
hipError_t launch_gen_grad(const Geom&, const float* x, const float* h, const float* xstar, float* g,
                           float sigma, RngKey key, uint32_t step, int noise_kind, unsigned band_tiles, Persist,
                           hipStream_t);
hipError_t launch_fill(int64_t d, float* dst, int which, RngKey key, hipStream_t);
hipError_t launch_relayout(const Geom& from, const Geom& to, const float* src, float* dst, hipStream_t);
hipError_t launch_init_replicas(const Geom&, float* x, float* v, float* center, const float* x0, int mode,
                                RngKey key, hipStream_t);
hipError_t launch_noise_alu(RngKey key, int noise_kind, uint32_t workgroups, uint32_t iters, float* out, hipStream_t);
hipError_t launch_philox_raw(RngKey key, uint32_t c1, uint32_t c2, uint32_t c3, int64_t n_blocks, uint32_t* out,
                             hipStream_t);
// columns per workgroup tile (256 threads x 4 columns)
#ifndef GSGD_BLOCK
#define GSGD_BLOCK 256
#endif
constexpr int64_t BLOCK_COLUMNS = static_cast<int64_t>(GSGD_BLOCK) * 4;
// stats: partials holds STATS_MAX_WORKGROUPS * 4 doubles (one set per workgroup of the pass); result 4 doubles (device)
constexpr unsigned STATS_MAX_WORKGROUPS = 2048;
hipError_t launch_stats(const Geom&, const float* x, const float* xstar, double* partials, double* result,
                        hipStream_t);

// row norms: partials holds k * NORM_CHUNKS doubles, result k doubles (device)
constexpr int NORM_CHUNKS = 256;
hipError_t launch_row_sqnorms(const Geom&, const float* x, double* partials, double* result, hipStream_t);

// ---- host-only helpers -----------------------------------------------------
void host_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
int  build_walk(const int32_t* perm, int32_t k, Walk* out);   // GSGD_OK or GSGD_ERR_BAD_PERM
// any map into 0..k-1; *has_trees = 0 when the map is a permutation
int  build_pull_walk(const int32_t* peer, int32_t k, Walk* out, int* has_trees, int* slots_used);
int  build_push_walk(const int32_t* target, int32_t k, Walk* out, int* slots_used);

}  // namespace gsgd

// C ABI of libgsgd: argument checking, context ownership, and dispatch to the
// kernel launchers.  No computation of the method happens here.
#include <mutex>
#include <new>
#include <string.h>

#include "gsgd_internal.hpp"

using namespace gsgd;

// Launches on one stream run one after the other and can share a ticket pair;
// launches on different streams may overlap and must not.  Every stream that
// has launched through the context owns one pair, each on a cache line of its own.
constexpr int    TICKET_PAIRS = 32;
constexpr size_t TICKET_STRIDE_WORDS = 32;     // 128 bytes
constexpr size_t TICKET_BYTES = TICKET_PAIRS * TICKET_STRIDE_WORDS * sizeof(uint32_t);

struct gsgd_ctx {
    gsgd_config cfg;          // host pointers inside are cleared after copying
    int         device;
    int64_t*    d_offsets;    // device copy of the segment table
    float*      d_scales;
    double*     d_partials;   // stats scratch: STATS_MAX_WORKGROUPS * 4 doubles
    double*     d_result;     // max(4, k) doubles
    double*     h_result;     // pinned host, max(4, k) doubles, then one more that receives a ticket pair
    double*     d_norm_partials;   // row-norm scratch: k * NORM_CHUNKS doubles
    uint32_t*   d_tickets;    // tile tickets of the persistent kernels: TICKET_PAIRS pairs, zero between launches
    hipStream_t pair_stream[TICKET_PAIRS];   // which stream launches through which pair
    int         n_pairs;
    int         cu_count;     // compute units of the device
    unsigned    width[GSGD_KERNEL_COUNT];   // persistent workgroups per streaming kernel
    bool        width_set[GSGD_KERNEL_COUNT];   // the width came from gsgd_set_launch_width, not from the defaults
    float       weight_decay;               // extras of the local step (Section 4.2); 0 / 0 = the boxed algorithms
    int         nesterov;
    int         row_split;                  // GSGD_ROW_SPLIT_*: how the k-way sums of short vectors are laid out
    int         gossip_form;                // GSGD_GOSSIP_*: cycle walk or two ascending sweeps
    int         last_hip;
};

namespace {

// Persistent workgroups per compute unit for each streaming kernel
// (GSGD_KERNEL_* order).  Measured on MI355X at the benchmark shapes.
// (the generator and the local step are plain grids: their width is the tiles per band of the grid, 0 = default)
constexpr unsigned DEFAULT_WORKGROUPS_PER_CU[GSGD_KERNEL_COUNT] = {1u, 1u, 1u, 0u, 2u, 0u};

// Elastic averaging with few replicas is not limited by the memory system but by what one workgroup per compute
// unit keeps in flight over its short tiles (almost no DRAM-credit stalls at k = 16): two per compute unit gain
// 1.5-2 points at k = 16 and 32; from k = 48 on (two rows in flight) one is better by as much.  On blocked matrices
// (two rows in flight at every k) one workgroup per compute unit is best throughout.
constexpr int EASGD_FEW_REPLICAS = 48;

// From this many replicas on, short vectors split the rows of a tile over the wavefronts of a workgroup.
constexpr int ROW_SPLIT_MIN_K = 16;

// Up to this many replicas the two-sweep gossip kernel keeps whole 1024-column tiles per workgroup; beyond, 256-column
// tiles with the rows split over the wavefronts.
constexpr int SWEEP_WHOLE_UP_TO = 36;

inline unsigned default_width(const gsgd_ctx* c, int kernel)
{
    unsigned per_cu = DEFAULT_WORKGROUPS_PER_CU[kernel];
    if (kernel == GSGD_KERNEL_EASGD && c->cfg.k < EASGD_FEW_REPLICAS && c->cfg.block_columns == 0) per_cu = 2u;
    return static_cast<unsigned>(c->cu_count) * per_cu;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// 0 (row-major), or the blocked layout's block: a power of two that every tile width divides, and whole blocks only
inline bool ok_block_columns(int64_t b, int64_t ld)
{
    return b == 0 || (b >= BLOCK_COLUMNS && (b & (b - 1)) == 0 && ld % b == 0);
}

inline int hip_fail(gsgd_ctx* ctx, hipError_t e)
{
    if (ctx) ctx->last_hip = static_cast<int>(e);
    return GSGD_ERR_HIP;
}

inline Geom geom_of(const gsgd_ctx* c) { return make_geom(c->cfg.k, c->cfg.d, c->cfg.ld, c->cfg.block_columns); }
inline Hyper hyper_of(const gsgd_ctx* c) { return Hyper{c->cfg.lr, c->cfg.momentum, c->weight_decay, c->nesterov}; }
inline SegTable seg_of(const gsgd_ctx* c) { return SegTable{c->d_offsets, c->d_scales, c->cfg.n_seg}; }
// Index of the ticket pair of `stream`, claiming a free one on first use; -1 when all are taken.
inline int pair_of(gsgd_ctx* c, hipStream_t stream)
{
    for (int p = 0; p < c->n_pairs; ++p)
        if (c->pair_stream[p] == stream) return p;
    if (c->n_pairs == TICKET_PAIRS) return -1;
    c->pair_stream[c->n_pairs] = stream;
    return c->n_pairs++;
}
inline uint32_t* pair_words(const gsgd_ctx* c, int pair) { return c->d_tickets + static_cast<size_t>(pair) * TICKET_STRIDE_WORDS; }

// Launch shape of one streaming kernel on one stream; tickets == nullptr when the context has run on
// TICKET_PAIRS other streams already.
inline Persist persist_of(gsgd_ctx* c, int kernel, void* stream)
{
    const int pair = pair_of(c, static_cast<hipStream_t>(stream));
    return Persist{pair < 0 ? nullptr : pair_words(c, pair), c->width[kernel]};
}
// The two kernels that do not couple the rows (local step, gradient generator) run as persistent workgroups walking
// the rows of a tile in ascending order on blocked matrices, where that is the address order of a block, and as plain
// banded grids (tickets == nullptr) on row-major ones.  Measured on MI355X, blocks of 16 Ki columns, ResNet-50 size
// (% of the HBM peak, grid -> walk): local step k = 16 / 32 / 128: 70 / 76 / 73 -> 84 / 84 / 82 with one workgroup per
// compute unit (79 / 79 / 78 with two); generator k = 12 / 32 / 128: 76 / 73 / 71 -> 85 / 85 / 81 with two per compute
// unit (64 / 63 with one); with few replicas the generator's tiles are too short for a walk and its grid stays
// ahead (k = 8: 77 against 68, k = 4: 80 against 41), hence the threshold.
constexpr unsigned LOCAL_WALK_WGS_PER_CU = 1, GEN_WALK_WGS_PER_CU = 2;
constexpr int GEN_WALK_FROM_K = 12;
// `set_width`: what gsgd_set_launch_width left for the kernel (0 = default); as a walk it counts workgroups.
inline Persist row_walk_of(gsgd_ctx* c, int kernel, void* stream)
{
    if (c->cfg.block_columns == 0) return Persist{nullptr, 0u};
    if (kernel == GSGD_KERNEL_GEN_GRAD && c->cfg.k < GEN_WALK_FROM_K) return Persist{nullptr, 0u};
    const unsigned per_cu = kernel == GSGD_KERNEL_GEN_GRAD ? GEN_WALK_WGS_PER_CU : LOCAL_WALK_WGS_PER_CU;
    const unsigned width = c->width[kernel] ? c->width[kernel] : static_cast<unsigned>(c->cu_count) * per_cu;
    const int pair = pair_of(c, static_cast<hipStream_t>(stream));
    return Persist{pair < 0 ? nullptr : pair_words(c, pair), width};
}
inline bool row_walk_wanted(const gsgd_ctx* c, int kernel)
{
    return c->cfg.block_columns > 0 && !(kernel == GSGD_KERNEL_GEN_GRAD && c->cfg.k < GEN_WALK_FROM_K);
}
// Rows split over the wavefronts of a workgroup when one thread per four columns cannot fill the chip: fewer
// 1024-column tiles than compute units, and enough rows for the split to shorten the walk.  Measured on MI355X
// (serial / split, microseconds per all-reduce step): d = 16,384: k = 8 8.8 / 8.8, k = 32 14.9 / 8.9, k = 128
// 45.6 / 10.9, k = 512 170 / 40; d = 65,536: 8.3 / 8.8, 17.1 / 8.8, 56 / 33, 217 / 116; d = 262,144 (as many tiles
// as compute units): 13.1 / 8.4, 31 / 28, 118 / 126, 479 / 543; from d = 1,048,576 on the serial walk wins.
inline bool row_split_of(const gsgd_ctx* c)
{
    if (c->row_split == GSGD_ROW_SPLIT_ON) return true;
    if (c->row_split == GSGD_ROW_SPLIT_OFF) return false;
    const int64_t tiles = (c->cfg.d + BLOCK_COLUMNS - 1) / BLOCK_COLUMNS;
    return tiles < c->cu_count && c->cfg.k >= ROW_SPLIT_MIN_K;
}

inline RngKey key_of(const gsgd_ctx* c)
{
    return RngKey{static_cast<uint32_t>(c->cfg.seed), static_cast<uint32_t>(c->cfg.seed >> 32)};
}

// Row matrices must be non-null and 16-byte aligned (rows then are, since ld % 4 == 0).
inline bool ok_matrix(const void* p) { return p && aligned16(p); }

// Bytes from the first element of a k x ld row matrix to one past the last column any kernel touches,
// and the same for a shared d-vector.
inline size_t span_of(int32_t k, int64_t d, int64_t ld, int64_t block_columns)
{
    const size_t kk = static_cast<size_t>(k), dd = static_cast<size_t>(d);
    if (block_columns > 0) {
        // every block before the one holding column d - 1 in full, then that block up to the last row's piece
        const size_t b = static_cast<size_t>(block_columns), last = (dd - 1) / b;
        return sizeof(float) * (last * kk * b + (kk - 1) * b + (dd - last * b));
    }
    return sizeof(float) * ((kk - 1) * static_cast<size_t>(ld) + dd);
}
inline size_t matrix_span(const gsgd_ctx* c) { return span_of(c->cfg.k, c->cfg.d, c->cfg.ld, c->cfg.block_columns); }
inline size_t vector_span(const gsgd_ctx* c) { return sizeof(float) * static_cast<size_t>(c->cfg.d); }

inline bool overlap(const void* a, size_t na, const void* b, size_t nb)
{
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + nb && b0 < a0 + na;
}

// x, v, g: distinct, non-overlapping k x ld matrices.
int check_state(const gsgd_ctx* ctx, const float* x, const float* v, const float* g)
{
    if (!ctx) return GSGD_ERR_INVALID_ARG;
    if (!ok_matrix(x) || !ok_matrix(v) || !ok_matrix(g)) return GSGD_ERR_INVALID_ARG;
    const size_t m = matrix_span(ctx);
    if (overlap(x, m, v, m) || overlap(x, m, g, m) || overlap(v, m, g, m)) return GSGD_ERR_INVALID_ARG;
    return GSGD_OK;
}

// a shared d-vector (centre, h, xstar) against the matrices a call writes
bool vector_clear_of(const gsgd_ctx* ctx, const float* vec, const float* a, const float* b, const float* c = nullptr)
{
    const size_t m = matrix_span(ctx), n = vector_span(ctx);
    return !overlap(vec, n, a, m) && !overlap(vec, n, b, m) && !(c && overlap(vec, n, c, m));
}

void release(gsgd_ctx* c)
{
    if (c->d_offsets) (void)hipFree(c->d_offsets);
    if (c->d_scales) (void)hipFree(c->d_scales);
    if (c->d_partials) (void)hipFree(c->d_partials);
    if (c->d_result) (void)hipFree(c->d_result);
    if (c->h_result) (void)hipHostFree(c->h_result);
    if (c->d_tickets) (void)hipFree(c->d_tickets);
    if (c->d_norm_partials) (void)hipFree(c->d_norm_partials);
    delete c;
}

}  // namespace

// ---- the statistics for callers that cannot allocate --------------------------------------------------------
// The partial sums of the two statistics kernels (one set per workgroup of the pass, 64 KiB at most) live in a
// fixed array in device memory instead of a hipMalloc'ed buffer.  Every GPU the library runs on holds its own copy until the process ends.  The array's
// name is only a handle on the host: its device address is looked up once per device and kept.
static __device__ __align__(256) double scratch[STATS_MAX_WORKGROUPS * 4];

namespace {
constexpr int MAX_DEVICES = 64;
double*    g_scratch_ptr[MAX_DEVICES];      // device address of `scratch` on each device, nullptr until resolved
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (resolved on first use).
hipError_t scratch_on_current_device(double** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        double* ptr = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}
}  // namespace

extern "C" int gsgd_create(const gsgd_config* cfg, gsgd_ctx** out)
{
    if (!cfg || !out) return GSGD_ERR_INVALID_ARG;
    *out = nullptr;
    if (cfg->k < 1 || cfg->k > GSGD_MAX_K || cfg->d < 1 || cfg->ld < cfg->d || (cfg->ld & 3) != 0)
        return GSGD_ERR_INVALID_ARG;
    if (cfg->d > (static_cast<int64_t>(1) << 34)) return GSGD_ERR_INVALID_ARG;   // quad index is a 32-bit counter word
    if (!ok_block_columns(cfg->block_columns, cfg->ld)) return GSGD_ERR_INVALID_ARG;
    if (cfg->noise_kind != GSGD_NOISE_GAUSSIAN && cfg->noise_kind != GSGD_NOISE_UNIFORM) return GSGD_ERR_INVALID_ARG;
    if (!(cfg->sigma >= 0.0f) || !(cfg->lr == cfg->lr) || !(cfg->momentum == cfg->momentum)) return GSGD_ERR_INVALID_ARG;
    if (cfg->n_seg < 0) return GSGD_ERR_INVALID_ARG;
    if (cfg->n_seg > 0) {
        if (!cfg->seg_offsets || !cfg->seg_lr_scale) return GSGD_ERR_INVALID_ARG;
        if (cfg->seg_offsets[0] != 0 || cfg->seg_offsets[cfg->n_seg] != cfg->d) return GSGD_ERR_BAD_SEGMENTS;
        for (int32_t s = 0; s < cfg->n_seg; ++s)
            if (cfg->seg_offsets[s + 1] <= cfg->seg_offsets[s]) return GSGD_ERR_BAD_SEGMENTS;
    }

    gsgd_ctx* c = new (std::nothrow) gsgd_ctx;
    if (!c) return GSGD_ERR_NO_MEMORY;
    memset(c, 0, sizeof(*c));
    c->cfg = *cfg;
    c->cfg.seg_offsets = nullptr;
    c->cfg.seg_lr_scale = nullptr;

    hipError_t e = hipGetDevice(&c->device);
    if (e == hipSuccess && cfg->n_seg > 0) {
        const size_t nb_off = sizeof(int64_t) * static_cast<size_t>(cfg->n_seg + 1);
        const size_t nb_sc = sizeof(float) * static_cast<size_t>(cfg->n_seg);
        e = hipMalloc(reinterpret_cast<void**>(&c->d_offsets), nb_off);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->d_scales), nb_sc);
        if (e == hipSuccess) e = hipMemcpy(c->d_offsets, cfg->seg_offsets, nb_off, hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemcpy(c->d_scales, cfg->seg_lr_scale, nb_sc, hipMemcpyHostToDevice);
    }
    if (e == hipSuccess)
        e = hipMalloc(reinterpret_cast<void**>(&c->d_partials), sizeof(double) * 4 * STATS_MAX_WORKGROUPS);
    const size_t n_result = static_cast<size_t>(cfg->k > 4 ? cfg->k : 4);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->d_result), sizeof(double) * n_result);
    if (e == hipSuccess)
        e = hipHostMalloc(reinterpret_cast<void**>(&c->h_result), sizeof(double) * (n_result + 1), hipHostMallocDefault);
    if (e == hipSuccess)
        e = hipMalloc(reinterpret_cast<void**>(&c->d_norm_partials),
                      sizeof(double) * static_cast<size_t>(cfg->k) * NORM_CHUNKS);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->d_tickets), TICKET_BYTES);
    if (e == hipSuccess) e = hipMemset(c->d_tickets, 0, TICKET_BYTES);
    // the clear runs on the null stream, which a non-blocking stream does not wait for
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e == hipSuccess) {                       // so that gsgd_stats_static's first call on this device looks nothing up
        double* unused = nullptr;
        e = scratch_on_current_device(&unused);
    }
    if (e == hipSuccess) e = hipDeviceGetAttribute(&c->cu_count, hipDeviceAttributeMultiprocessorCount, c->device);
    if (e == hipSuccess) {
        if (c->cu_count < 1) c->cu_count = 1;
        for (int kn = 0; kn < GSGD_KERNEL_COUNT; ++kn) { c->width[kn] = default_width(c, kn); c->width_set[kn] = false; }
    }
    if (e != hipSuccess) {
        release(c);
        return e == hipErrorOutOfMemory ? GSGD_ERR_NO_MEMORY : GSGD_ERR_HIP;
    }
    *out = c;
    return GSGD_OK;
}

extern "C" int gsgd_destroy(gsgd_ctx* ctx)
{
    if (!ctx) return GSGD_ERR_INVALID_ARG;
    release(ctx);
    return GSGD_OK;
}

extern "C" int gsgd_set_lr(gsgd_ctx* ctx, float lr)
{
    if (!ctx || !(lr == lr)) return GSGD_ERR_INVALID_ARG;
    ctx->cfg.lr = lr;
    return GSGD_OK;
}

extern "C" int gsgd_set_local_step(gsgd_ctx* ctx, float weight_decay, int nesterov)
{
    if (!ctx || !(weight_decay >= 0.0f) || (nesterov != 0 && nesterov != 1)) return GSGD_ERR_INVALID_ARG;
    ctx->weight_decay = weight_decay;
    ctx->nesterov = nesterov;
    return GSGD_OK;
}

extern "C" int gsgd_set_gossip_form(gsgd_ctx* ctx, int form)
{
    if (!ctx || form < GSGD_GOSSIP_AUTO || form > GSGD_GOSSIP_SWEEP_SPLIT) return GSGD_ERR_INVALID_ARG;
    ctx->gossip_form = form;
    return GSGD_OK;
}

extern "C" int gsgd_set_row_split(gsgd_ctx* ctx, int mode)
{
    if (!ctx || (mode != GSGD_ROW_SPLIT_AUTO && mode != GSGD_ROW_SPLIT_OFF && mode != GSGD_ROW_SPLIT_ON))
        return GSGD_ERR_INVALID_ARG;
    ctx->row_split = mode;
    return GSGD_OK;
}

extern "C" int gsgd_comm_due(uint64_t step, uint32_t tau)
{
    if (tau == 0) return GSGD_ERR_INVALID_ARG;
    return (step + 1) % tau == 0 ? 1 : 0;
}

extern "C" int gsgd_set_launch_width(gsgd_ctx* ctx, int kernel, int workgroups)
{
    if (!ctx || kernel < 0 || kernel >= GSGD_KERNEL_COUNT || workgroups < 0 || workgroups > (1 << 20))
        return GSGD_ERR_INVALID_ARG;
    ctx->width[kernel] = workgroups > 0 ? static_cast<unsigned>(workgroups) : default_width(ctx, kernel);
    ctx->width_set[kernel] = workgroups > 0;
    return GSGD_OK;
}

extern "C" int gsgd_init_replicas(gsgd_ctx* ctx, float* x, float* v, float* center, const float* x0, int mode,
                                  void* stream)
{
    if (!ctx || !ok_matrix(x) || !ok_matrix(v) || overlap(x, matrix_span(ctx), v, matrix_span(ctx)))
        return GSGD_ERR_INVALID_ARG;
    if (mode != GSGD_INIT_BROADCAST && mode != GSGD_INIT_PER_REPLICA) return GSGD_ERR_INVALID_ARG;
    if (mode == GSGD_INIT_BROADCAST && !ok_matrix(x0)) return GSGD_ERR_INVALID_ARG;
    if (center && (!aligned16(center) || !vector_clear_of(ctx, center, x, v))) return GSGD_ERR_INVALID_ARG;
    if (mode == GSGD_INIT_BROADCAST && !vector_clear_of(ctx, x0, x, v)) return GSGD_ERR_INVALID_ARG;
    const hipError_t e = launch_init_replicas(geom_of(ctx), x, v, center, x0, mode, key_of(ctx),
                                              static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_fill(gsgd_ctx* ctx, float* dst, int which, void* stream)
{
    if (!ctx || !ok_matrix(dst)) return GSGD_ERR_INVALID_ARG;
    if (which != GSGD_FILL_XSTAR && which != GSGD_FILL_H && which != GSGD_FILL_X0) return GSGD_ERR_INVALID_ARG;
    const hipError_t e = launch_fill(ctx->cfg.d, dst, which, key_of(ctx), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_relayout(int32_t k, int64_t d, int64_t src_ld, int64_t src_block_columns, const float* src,
                             int64_t dst_ld, int64_t dst_block_columns, float* dst, void* stream)
{
    if (k < 1 || k > GSGD_MAX_K || d < 1 || d > (static_cast<int64_t>(1) << 34)) return GSGD_ERR_INVALID_ARG;
    if (src_ld < d || (src_ld & 3) != 0 || dst_ld < d || (dst_ld & 3) != 0) return GSGD_ERR_INVALID_ARG;
    if (!ok_block_columns(src_block_columns, src_ld) || !ok_block_columns(dst_block_columns, dst_ld))
        return GSGD_ERR_INVALID_ARG;
    if (!ok_matrix(src) || !ok_matrix(dst)) return GSGD_ERR_INVALID_ARG;
    if (overlap(src, span_of(k, d, src_ld, src_block_columns), dst, span_of(k, d, dst_ld, dst_block_columns)))
        return GSGD_ERR_INVALID_ARG;
    const hipError_t e = launch_relayout(make_geom(k, d, src_ld, src_block_columns), make_geom(k, d, dst_ld, dst_block_columns),
                                         src, dst, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : GSGD_ERR_HIP;
}

extern "C" int gsgd_gen_grad(gsgd_ctx* ctx, const float* x, const float* h, const float* xstar, float* g,
                             uint64_t step, void* stream)
{
    if (!ctx || !ok_matrix(x) || !ok_matrix(g) || !ok_matrix(h) || !ok_matrix(xstar)) return GSGD_ERR_INVALID_ARG;
    if (overlap(x, matrix_span(ctx), g, matrix_span(ctx)) || !vector_clear_of(ctx, h, g, g) ||
        !vector_clear_of(ctx, xstar, g, g))
        return GSGD_ERR_INVALID_ARG;
    if (step > 0xFFFFFFFFull) return GSGD_ERR_INVALID_ARG;
    const Persist ps = row_walk_of(ctx, GSGD_KERNEL_GEN_GRAD, stream);
    if (row_walk_wanted(ctx, GSGD_KERNEL_GEN_GRAD) && !ps.tickets) return GSGD_ERR_UNSUPPORTED;
    const hipError_t e = launch_gen_grad(geom_of(ctx), x, h, xstar, g, ctx->cfg.sigma, key_of(ctx),
                                         static_cast<uint32_t>(step), ctx->cfg.noise_kind,
                                         ctx->width[GSGD_KERNEL_GEN_GRAD], ps, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_philox_raw(gsgd_ctx* ctx, uint32_t c1, uint32_t c2, uint32_t c3, int64_t n_blocks, uint32_t* out,
                               void* stream)
{
    if (!ctx || !out || n_blocks < 1 || n_blocks > (static_cast<int64_t>(1) << 32)) return GSGD_ERR_INVALID_ARG;
    const hipError_t e = launch_philox_raw(key_of(ctx), c1, c2, c3, n_blocks, out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_noise_alu_probe(gsgd_ctx* ctx, int32_t workgroups, uint32_t iters, float* out, void* stream)
{
    if (!ctx || !out || workgroups < 1 || workgroups > (1 << 20) || iters < 1) return GSGD_ERR_INVALID_ARG;
    const hipError_t e = launch_noise_alu(key_of(ctx), ctx->cfg.noise_kind, static_cast<uint32_t>(workgroups), iters, out,
                                          static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_step_allreduce(gsgd_ctx* ctx, float* x, float* v, const float* g, void* stream)
{
    const int rc = check_state(ctx, x, v, g);
    if (rc != GSGD_OK) return rc;
    const bool split = row_split_of(ctx);
    Persist ps{nullptr, 0u};                              // the row-split kernels are plain grids
    if (!split) {
        ps = persist_of(ctx, GSGD_KERNEL_ALLREDUCE, stream);
        if (!ps.tickets) return GSGD_ERR_UNSUPPORTED;
    }
    const hipError_t e = launch_step_allreduce(geom_of(ctx), hyper_of(ctx), seg_of(ctx), x, v, g, ps, split,
                                               static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

namespace {
// Which kernel form a gossip call takes: GSGD_GOSSIP_WALK, _SWEEP or _SWEEP_SPLIT (never AUTO).  Measured on MI355X:
// on row-major matrices the walk along the peer map is the faster form (71 against 65-69 % of the HBM peak at the
// benchmark shape), on blocked ones the two ascending sweeps are (80-84 against 72-75 %; 81 against 67 % at k = 128).
// Short vectors (fewer 1024-column tiles than compute units) with 16 replicas or more take the split sweeps in either
// layout: four times the workgroups and a quarter of the rows per wavefront (microseconds per step, walk -> split,
// row-major: d = 16,384: k = 32 17.1 -> 10.6, k = 128 58 -> 20; d = 65,536: 19.9 -> 14.3, 66 -> 37; at d = 262,144 the
// walk is level or ahead).  A form that cannot park k rows falls back to the next one.
int gossip_form_of(const gsgd_ctx* c)
{
    int form = c->gossip_form;
    if (form == GSGD_GOSSIP_AUTO) {
        const int64_t tiles = (c->cfg.d + BLOCK_COLUMNS - 1) / BLOCK_COLUMNS;
        if (tiles < c->cu_count && c->cfg.k >= ROW_SPLIT_MIN_K) form = GSGD_GOSSIP_SWEEP_SPLIT;
        else if (c->cfg.block_columns == 0) form = GSGD_GOSSIP_WALK;
        else form = c->cfg.k <= SWEEP_WHOLE_UP_TO ? GSGD_GOSSIP_SWEEP : GSGD_GOSSIP_SWEEP_SPLIT;
    }
    if (form == GSGD_GOSSIP_SWEEP && c->cfg.k > sweep_capacity(false)) form = GSGD_GOSSIP_SWEEP_SPLIT;
    if (form == GSGD_GOSSIP_SWEEP_SPLIT && c->cfg.k > sweep_capacity(true)) form = GSGD_GOSSIP_WALK;
    return form;
}

// The peer map as the sweep kernels take it: entry i = the row that row i mixes with (validated by the caller).
Walk peers_of(const int32_t* peer, int32_t k)
{
    Walk w;
    for (int32_t i = 0; i < k; ++i) w.seq[i] = static_cast<uint32_t>(peer[i]);
    return w;
}

// One gossip step on a validated peer map: `walk` is its cycle (or cycle-and-tree) order, `peer` the map itself.
hipError_t launch_gossip(gsgd_ctx* ctx, const Walk& walk, const int32_t* peer, bool stale, bool has_trees, bool fused,
                         float beta, float* x, float* v, const float* g, const float* h, const float* xstar,
                         uint64_t step, const Persist& ps, void* stream)
{
    const hipStream_t st = static_cast<hipStream_t>(stream);
    const int form = gossip_form_of(ctx);
    if (form != GSGD_GOSSIP_WALK)
        return launch_step_gossip_sweep(geom_of(ctx), hyper_of(ctx), seg_of(ctx), beta, peers_of(peer, ctx->cfg.k), stale,
                                        form == GSGD_GOSSIP_SWEEP_SPLIT, fused, x, v, g, h, xstar, ctx->cfg.sigma,
                                        key_of(ctx), static_cast<uint32_t>(step), ctx->cfg.noise_kind, ps, st);
    if (fused)
        return launch_step_gossip_fused(geom_of(ctx), hyper_of(ctx), seg_of(ctx), beta, walk, stale, has_trees, x, v, h,
                                        xstar, ctx->cfg.sigma, key_of(ctx), static_cast<uint32_t>(step),
                                        ctx->cfg.noise_kind, ps, st);
    return launch_step_gossip(geom_of(ctx), hyper_of(ctx), seg_of(ctx), beta, walk, stale, has_trees, x, v, g, ps, st);
}

// One push-gossip step on a validated target map: `walk` is its senders-first order for the walk kernel; the sweep
// kernels take the senders of every row instead (ascending, self-sends left out: a node always keeps its own copy).
hipError_t launch_push(gsgd_ctx* ctx, const Walk& walk, const int32_t* target, bool fused, float* x, float* v,
                       const float* g, const float* h, const float* xstar, uint64_t step, const Persist& ps, void* stream)
{
    const hipStream_t st = static_cast<hipStream_t>(stream);
    const int form = gossip_form_of(ctx);
    if (form != GSGD_GOSSIP_WALK) {
        const int32_t k = ctx->cfg.k;
        Persist wide = ps;
        // Push-gossip does more arithmetic per row in the second sweep (fp64 sums and a division) than one workgroup
        // per compute unit hides: two where they fit, unless the caller has chosen the width
        if (k <= sweep_rows_two_per_cu(form == GSGD_GOSSIP_SWEEP_SPLIT) &&
            !ctx->width_set[fused ? GSGD_KERNEL_GOSSIP_FUSED : GSGD_KERNEL_GOSSIP])
            wide.workgroups = 2u * static_cast<unsigned>(ctx->cu_count);
        Walk index{}, senders{};
        static_assert(GSGD_MAX_K <= 0x3FF, "the index word holds ten bits per field");
        uint32_t count[GSGD_MAX_K];
        for (int32_t r = 0; r < k; ++r) count[r] = 0;
        for (int32_t i = 0; i < k; ++i)
            if (target[i] != i) ++count[target[i]];
        uint32_t at = 0;
        for (int32_t r = 0; r < k; ++r) {
            index.seq[r] = (at << 10) | (count[r] << 20);   // bits 0-9, the group's first sender, are filled in below
            at += count[r];
            count[r] = 0;                                   // reused below as the fill position inside the group
        }
        for (int32_t i = 0; i < k; ++i) {                   // ascending i: every group ends up in ascending order
            const int32_t r = target[i];
            if (r == i) continue;
            if (count[r] == 0) index.seq[r] |= static_cast<uint32_t>(i);
            senders.seq[((index.seq[r] >> 10) & 0x3FFu) + count[r]++] = static_cast<uint32_t>(i);
        }
        return launch_step_gossip_push_sweep(geom_of(ctx), hyper_of(ctx), seg_of(ctx), index, senders,
                                             form == GSGD_GOSSIP_SWEEP_SPLIT, fused, x, v, g, h, xstar, ctx->cfg.sigma,
                                             key_of(ctx), static_cast<uint32_t>(step), ctx->cfg.noise_kind, wide, st);
    }
    if (fused)
        return launch_step_gossip_push_fused(geom_of(ctx), hyper_of(ctx), seg_of(ctx), walk, x, v, h, xstar, ctx->cfg.sigma,
                                             key_of(ctx), static_cast<uint32_t>(step), ctx->cfg.noise_kind, ps, st);
    return launch_step_gossip_push(geom_of(ctx), hyper_of(ctx), seg_of(ctx), walk, x, v, g, ps, st);
}

int gossip_on_permutation(gsgd_ctx* ctx, float* x, float* v, const float* g, const int32_t* peer_perm, float beta,
                          bool stale, void* stream)
{
    int rc = check_state(ctx, x, v, g);
    if (rc != GSGD_OK) return rc;
    if (!peer_perm || !(beta == beta)) return GSGD_ERR_INVALID_ARG;
    Walk walk;
    rc = build_walk(peer_perm, ctx->cfg.k, &walk);
    if (rc != GSGD_OK) return rc;
    const Persist ps = persist_of(ctx, GSGD_KERNEL_GOSSIP, stream);
    if (!ps.tickets) return GSGD_ERR_UNSUPPORTED;
    const hipError_t e = launch_gossip(ctx, walk, peer_perm, stale, false, false, beta, x, v, g, nullptr, nullptr, 0, ps,
                                       stream);
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}
}  // namespace

extern "C" int gsgd_step_gossip_pull(gsgd_ctx* ctx, float* x, float* v, const float* g,
                                     const int32_t* peer, float beta, int stale, void* stream)
{
    int rc = check_state(ctx, x, v, g);
    if (rc != GSGD_OK) return rc;
    if (!peer || !(beta == beta) || (stale != 0 && stale != 1)) return GSGD_ERR_INVALID_ARG;
    Walk walk;
    int has_trees = 0, slots = 0;
    rc = build_pull_walk(peer, ctx->cfg.k, &walk, &has_trees, &slots);
    if (rc != GSGD_OK) return rc;
    const Persist ps = persist_of(ctx, GSGD_KERNEL_GOSSIP, stream);
    if (!ps.tickets) return GSGD_ERR_UNSUPPORTED;
    const hipError_t e = launch_gossip(ctx, walk, peer, stale != 0, has_trees != 0, false, beta, x, v, g, nullptr, nullptr,
                                       0, ps, stream);
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_step_gossip(gsgd_ctx* ctx, float* x, float* v, const float* g,
                                const int32_t* peer_perm, float beta, void* stream)
{
    return gossip_on_permutation(ctx, x, v, g, peer_perm, beta, false, stream);
}

extern "C" int gsgd_step_gossip_stale(gsgd_ctx* ctx, float* x, float* v, const float* g,
                                      const int32_t* peer_perm, float beta, void* stream)
{
    return gossip_on_permutation(ctx, x, v, g, peer_perm, beta, true, stream);
}

extern "C" int gsgd_step_gossip_push(gsgd_ctx* ctx, float* x, float* v, const float* g,
                                     const int32_t* target, void* stream)
{
    int rc = check_state(ctx, x, v, g);
    if (rc != GSGD_OK) return rc;
    if (!target) return GSGD_ERR_INVALID_ARG;
    Walk walk;
    int slots = 0;
    rc = build_push_walk(target, ctx->cfg.k, &walk, &slots);
    if (rc != GSGD_OK) return rc;
    const Persist ps = persist_of(ctx, GSGD_KERNEL_GOSSIP, stream);
    if (!ps.tickets) return GSGD_ERR_UNSUPPORTED;
    const hipError_t e = launch_push(ctx, walk, target, false, x, v, g, nullptr, nullptr, 0, ps, stream);
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_step_async_tick(gsgd_ctx* ctx, float* x, float* v, const float* g, int32_t i, int32_t j,
                                    float beta, void* stream)
{
    const int rc = check_state(ctx, x, v, g);
    if (rc != GSGD_OK) return rc;
    if (i < 0 || i >= ctx->cfg.k || j < 0 || j >= ctx->cfg.k || !(beta == beta)) return GSGD_ERR_INVALID_ARG;
    const hipError_t e = launch_async_tick(geom_of(ctx), hyper_of(ctx), seg_of(ctx), beta, i, j, x, v, g,
                                           static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_step_easgd_tick(gsgd_ctx* ctx, float* x, float* v, const float* g, float* center, int32_t i,
                                    float alpha_e, void* stream)
{
    const int rc = check_state(ctx, x, v, g);
    if (rc != GSGD_OK) return rc;
    if (!ok_matrix(center) || !vector_clear_of(ctx, center, x, v, g) || !(alpha_e == alpha_e))
        return GSGD_ERR_INVALID_ARG;
    if (i < 0 || i >= ctx->cfg.k) return GSGD_ERR_INVALID_ARG;
    const hipError_t e = launch_easgd_tick(geom_of(ctx), hyper_of(ctx), seg_of(ctx), alpha_e, i, x, v, g, center,
                                           static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_step_async_tick_fused(gsgd_ctx* ctx, float* x, float* v, const float* h, const float* xstar,
                                          int32_t i, int32_t j, float beta, uint64_t tick, void* stream)
{
    if (!ctx || !ok_matrix(x) || !ok_matrix(v) || !ok_matrix(h) || !ok_matrix(xstar)) return GSGD_ERR_INVALID_ARG;
    if (overlap(x, matrix_span(ctx), v, matrix_span(ctx)) || !vector_clear_of(ctx, h, x, v) ||
        !vector_clear_of(ctx, xstar, x, v))
        return GSGD_ERR_INVALID_ARG;
    if (i < 0 || i >= ctx->cfg.k || j < 0 || j >= ctx->cfg.k || !(beta == beta) || tick > 0xFFFFFFFFull)
        return GSGD_ERR_INVALID_ARG;
    const hipError_t e = launch_async_tick_fused(geom_of(ctx), hyper_of(ctx), seg_of(ctx), beta, i, j, x, v, h, xstar,
                                                 ctx->cfg.sigma, key_of(ctx), static_cast<uint32_t>(tick),
                                                 ctx->cfg.noise_kind, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_run_async_ticks(gsgd_ctx* ctx, float* x, float* v, const float* h, const float* xstar,
                                    float beta, uint64_t first_tick, uint64_t n_ticks, void* stream)
{
    if (!ctx || first_tick > 0xFFFFFFFFull || n_ticks > 0xFFFFFFFFull || first_tick + n_ticks > 0x100000000ull)
        return GSGD_ERR_INVALID_ARG;
    for (uint64_t t = first_tick; t < first_tick + n_ticks; ++t) {
        int32_t i = 0, j = 0;
        int rc = gsgd_make_tick(ctx->cfg.seed, t, ctx->cfg.k, &i, &j);
        if (rc == GSGD_OK) rc = gsgd_step_async_tick_fused(ctx, x, v, h, xstar, i, j, beta, t, stream);
        if (rc != GSGD_OK) return rc;
    }
    return GSGD_OK;
}

extern "C" int gsgd_step_local(gsgd_ctx* ctx, float* x, float* v, const float* g, void* stream)
{
    const int rc = check_state(ctx, x, v, g);
    if (rc != GSGD_OK) return rc;
    const Persist ps = row_walk_of(ctx, GSGD_KERNEL_LOCAL, stream);
    if (row_walk_wanted(ctx, GSGD_KERNEL_LOCAL) && !ps.tickets) return GSGD_ERR_UNSUPPORTED;
    const hipError_t e = launch_step_local(geom_of(ctx), hyper_of(ctx), seg_of(ctx), x, v, g,
                                           ctx->width[GSGD_KERNEL_LOCAL], ps, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

namespace {
int check_fused(const gsgd_ctx* ctx, const float* x, const float* v, const float* h, const float* xstar,
                const int32_t* map, uint64_t step)
{
    if (!ctx || !ok_matrix(x) || !ok_matrix(v) || !ok_matrix(h) || !ok_matrix(xstar)) return GSGD_ERR_INVALID_ARG;
    if (overlap(x, matrix_span(ctx), v, matrix_span(ctx)) || !vector_clear_of(ctx, h, x, v) ||
        !vector_clear_of(ctx, xstar, x, v))
        return GSGD_ERR_INVALID_ARG;
    if (!map || step > 0xFFFFFFFFull) return GSGD_ERR_INVALID_ARG;
    return GSGD_OK;
}
}  // namespace

extern "C" int gsgd_step_gossip_fused(gsgd_ctx* ctx, float* x, float* v, const float* h, const float* xstar,
                                      const int32_t* peer_perm, float beta, uint64_t step, void* stream)
{
    int rc = check_fused(ctx, x, v, h, xstar, peer_perm, step);
    if (rc != GSGD_OK) return rc;
    if (!(beta == beta)) return GSGD_ERR_INVALID_ARG;
    Walk walk;
    rc = build_walk(peer_perm, ctx->cfg.k, &walk);
    if (rc != GSGD_OK) return rc;
    const Persist ps = persist_of(ctx, GSGD_KERNEL_GOSSIP_FUSED, stream);
    if (!ps.tickets) return GSGD_ERR_UNSUPPORTED;
    const hipError_t e = launch_gossip(ctx, walk, peer_perm, false, false, true, beta, x, v, nullptr, h, xstar, step, ps,
                                       stream);
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_step_gossip_pull_fused(gsgd_ctx* ctx, float* x, float* v, const float* h, const float* xstar,
                                           const int32_t* peer, float beta, int stale, uint64_t step, void* stream)
{
    int rc = check_fused(ctx, x, v, h, xstar, peer, step);
    if (rc != GSGD_OK) return rc;
    if (!(beta == beta) || (stale != 0 && stale != 1)) return GSGD_ERR_INVALID_ARG;
    Walk walk;
    int has_trees = 0, slots = 0;
    rc = build_pull_walk(peer, ctx->cfg.k, &walk, &has_trees, &slots);
    if (rc != GSGD_OK) return rc;
    const Persist ps = persist_of(ctx, GSGD_KERNEL_GOSSIP_FUSED, stream);
    if (!ps.tickets) return GSGD_ERR_UNSUPPORTED;
    const hipError_t e = launch_gossip(ctx, walk, peer, stale != 0, has_trees != 0, true, beta, x, v, nullptr, h, xstar,
                                       step, ps, stream);
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_step_gossip_push_fused(gsgd_ctx* ctx, float* x, float* v, const float* h, const float* xstar,
                                           const int32_t* target, uint64_t step, void* stream)
{
    int rc = check_fused(ctx, x, v, h, xstar, target, step);
    if (rc != GSGD_OK) return rc;
    Walk walk;
    int slots = 0;
    rc = build_push_walk(target, ctx->cfg.k, &walk, &slots);
    if (rc != GSGD_OK) return rc;
    const Persist ps = persist_of(ctx, GSGD_KERNEL_GOSSIP_FUSED, stream);
    if (!ps.tickets) return GSGD_ERR_UNSUPPORTED;
    const hipError_t e = launch_push(ctx, walk, target, true, x, v, nullptr, h, xstar, step, ps, stream);
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_step_easgd(gsgd_ctx* ctx, float* x, float* v, const float* g,
                               float* center, float alpha_e, void* stream)
{
    const int rc = check_state(ctx, x, v, g);
    if (rc != GSGD_OK) return rc;
    if (!ok_matrix(center) || !vector_clear_of(ctx, center, x, v, g) || !(alpha_e == alpha_e))
        return GSGD_ERR_INVALID_ARG;
    const bool split = row_split_of(ctx);
    Persist ps{nullptr, 0u};
    if (!split) {
        ps = persist_of(ctx, GSGD_KERNEL_EASGD, stream);
        if (!ps.tickets) return GSGD_ERR_UNSUPPORTED;
    }
    const hipError_t e = launch_step_easgd(geom_of(ctx), hyper_of(ctx), seg_of(ctx), alpha_e, x, v, g, center, ps,
                                           split, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

namespace {
// The calls that wait for a stream also look at that stream's ticket pair: with the stream drained both
// words must read zero.  If they do not, a launch did not run to its end (or two launches shared the pair);
// the pair is cleared so that later launches hand out every tile again, and the caller is told.
// Enqueues the copy of the pair behind whatever is on the stream; `slot` is the index into h_result.
hipError_t fetch_ticket_pair(gsgd_ctx* ctx, hipStream_t s, size_t slot, int* pair_out)
{
    *pair_out = -1;
    for (int p = 0; p < ctx->n_pairs; ++p)
        if (ctx->pair_stream[p] == s) *pair_out = p;
    if (*pair_out < 0) return hipSuccess;
    return hipMemcpyAsync(ctx->h_result + slot, pair_words(ctx, *pair_out), 2 * sizeof(uint32_t),
                          hipMemcpyDeviceToHost, s);
}

int verify_ticket_pair(gsgd_ctx* ctx, hipStream_t s, size_t slot, int pair)
{
    if (pair < 0) return GSGD_OK;
    uint32_t words[2];
    memcpy(words, ctx->h_result + slot, sizeof(words));
    if (words[0] == 0u && words[1] == 0u) return GSGD_OK;
    hipError_t e = hipMemsetAsync(pair_words(ctx, pair), 0, 2 * sizeof(uint32_t), s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(ctx, e);
    return GSGD_ERR_BAD_STATE;
}
}  // namespace

extern "C" int gsgd_stats(gsgd_ctx* ctx, const float* x, const float* xstar, double out[4], void* stream)
{
    if (!ctx || !ok_matrix(x) || !ok_matrix(xstar) || !out) return GSGD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t slot = static_cast<size_t>(ctx->cfg.k > 4 ? ctx->cfg.k : 4);
    int pair = -1;
    hipError_t e = launch_stats(geom_of(ctx), x, xstar, ctx->d_partials, ctx->d_result, s);
    if (e == hipSuccess) e = hipMemcpyAsync(ctx->h_result, ctx->d_result, sizeof(double) * 4, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = fetch_ticket_pair(ctx, s, slot, &pair);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(ctx, e);
    for (int m = 0; m < 4; ++m) out[m] = ctx->h_result[m];
    return verify_ticket_pair(ctx, s, slot, pair);
}

extern "C" int gsgd_row_sqnorms(gsgd_ctx* ctx, const float* x, double* out, void* stream)
{
    if (!ctx || !ok_matrix(x) || !out) return GSGD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t slot = static_cast<size_t>(ctx->cfg.k > 4 ? ctx->cfg.k : 4);
    int pair = -1;
    hipError_t e = launch_row_sqnorms(geom_of(ctx), x, ctx->d_norm_partials, ctx->d_result, s);
    if (e == hipSuccess)
        e = hipMemcpyAsync(ctx->h_result, ctx->d_result, sizeof(double) * static_cast<size_t>(ctx->cfg.k),
                           hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = fetch_ticket_pair(ctx, s, slot, &pair);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(ctx, e);
    for (int32_t i = 0; i < ctx->cfg.k; ++i) out[i] = ctx->h_result[i];
    return verify_ticket_pair(ctx, s, slot, pair);
}

extern "C" int gsgd_stats_static(int32_t k, int64_t d, int64_t ld, int64_t block_columns, const float* x,
                                 const float* xstar, double* out_device, void* stream)
{
    if (k < 1 || k > GSGD_MAX_K || d < 1 || ld < d || (ld & 3) != 0) return GSGD_ERR_INVALID_ARG;
    if (!ok_block_columns(block_columns, ld)) return GSGD_ERR_INVALID_ARG;
    if (d > GSGD_STATS_STATIC_MAX_D) return GSGD_ERR_TOO_LARGE;
    if (!ok_matrix(x) || !ok_matrix(xstar) || !out_device || (reinterpret_cast<uintptr_t>(out_device) & 7u) != 0)
        return GSGD_ERR_INVALID_ARG;
    double* partials = nullptr;
    hipError_t e = scratch_on_current_device(&partials);
    if (e == hipSuccess)
        e = launch_stats(make_geom(k, d, ld, block_columns), x, xstar, partials, out_device,
                         static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : GSGD_ERR_HIP;
}

// Test hook: overwrite the ticket pair of `stream` (claiming one if the stream has none yet) behind the work
// already on the stream, and wait.
extern "C" int gsgd_poke_tickets(gsgd_ctx* ctx, uint32_t next_tile, uint32_t finished, void* stream)
{
    if (!ctx) return GSGD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int pair = pair_of(ctx, s);
    if (pair < 0) return GSGD_ERR_UNSUPPORTED;
    const uint32_t words[2] = {next_tile, finished};
    hipError_t e = hipStreamSynchronize(s);
    if (e == hipSuccess) e = hipMemcpy(pair_words(ctx, pair), words, sizeof(words), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

// ---- the weights v_ij of Section 3.1 and the diffusion potential: host arithmetic on k x k matrices -----------

extern "C" int gsgd_weights_pull(double* V, int32_t k, const int32_t* peer, double beta)
{
    if (!V || !peer || k < 1 || k > GSGD_MAX_K || !(beta == beta)) return GSGD_ERR_INVALID_ARG;
    for (int32_t i = 0; i < k; ++i)
        if (peer[i] < 0 || peer[i] >= k) return GSGD_ERR_BAD_PERM;
    double* old = new (std::nothrow) double[static_cast<size_t>(k) * k];
    if (!old) return GSGD_ERR_NO_MEMORY;
    memcpy(old, V, sizeof(double) * static_cast<size_t>(k) * k);
    for (int32_t i = 0; i < k; ++i)
        for (int32_t j = 0; j < k; ++j) {
            const double mine = old[static_cast<size_t>(i) * k + j], theirs = old[static_cast<size_t>(peer[i]) * k + j];
            V[static_cast<size_t>(i) * k + j] = mine - beta * (mine - theirs);
        }
    delete[] old;
    return GSGD_OK;
}

extern "C" int gsgd_weights_push(double* V, int32_t k, const int32_t* target)
{
    if (!V || !target || k < 1 || k > GSGD_MAX_K) return GSGD_ERR_INVALID_ARG;
    for (int32_t i = 0; i < k; ++i)
        if (target[i] < 0 || target[i] >= k) return GSGD_ERR_BAD_PERM;
    double* old = new (std::nothrow) double[static_cast<size_t>(k) * k];
    if (!old) return GSGD_ERR_NO_MEMORY;
    memcpy(old, V, sizeof(double) * static_cast<size_t>(k) * k);
    for (int32_t r = 0; r < k; ++r) {
        int32_t received = 1;
        for (int32_t i = 0; i < k; ++i)
            if (i != r && target[i] == r) {
                ++received;
                for (int32_t j = 0; j < k; ++j) V[static_cast<size_t>(r) * k + j] += old[static_cast<size_t>(i) * k + j];
            }
        for (int32_t j = 0; j < k; ++j) V[static_cast<size_t>(r) * k + j] /= static_cast<double>(received);
    }
    delete[] old;
    return GSGD_OK;
}

extern "C" int gsgd_diffusion_potential(const double* V, int32_t k, const double* sqnorm_start,
                                        const double* sqnorm_now, double* out)
{
    if (!V || !sqnorm_start || !sqnorm_now || !out || k < 1 || k > GSGD_MAX_K) return GSGD_ERR_INVALID_ARG;
    double total = 0.0;
    for (int32_t i = 0; i < k; ++i) {
        double own = 0.0;
        for (int32_t j = 0; j < k; ++j) own += V[static_cast<size_t>(i) * k + j] * V[static_cast<size_t>(i) * k + j] * sqnorm_start[j];
        total += own - sqnorm_now[i] / static_cast<double>(k);
    }
    *out = total;
    return GSGD_OK;
}

extern "C" const char* gsgd_strerror(int code)
{
    switch (code) {
        case GSGD_OK: return "ok";
        case GSGD_ERR_INVALID_ARG: return "invalid argument";
        case GSGD_ERR_BAD_PERM: return "peer map has an entry outside 0..k-1 or is not the permutation the call requires";
        case GSGD_ERR_BAD_SEGMENTS: return "segment table must ascend strictly from 0 to d";
        case GSGD_ERR_HIP: return "HIP runtime error";
        case GSGD_ERR_UNSUPPORTED: return "unsupported (a context serves at most 32 streams)";
        case GSGD_ERR_NO_MEMORY: return "out of memory";
        case GSGD_ERR_TOO_LARGE: return "d is larger than GSGD_STATS_STATIC_MAX_D, the most gsgd_stats_static takes";
        case GSGD_ERR_BAD_STATE: return "a tile counter of the context was not zero on a drained stream (cleared now)";
        default: return "unknown error";
    }
}

extern "C" int gsgd_last_hip_error(const gsgd_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

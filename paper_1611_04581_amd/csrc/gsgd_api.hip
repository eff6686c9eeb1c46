// C ABI of libgsgd: argument checking, context ownership, and dispatch to the
// kernel launchers.  No computation of the method happens here.
#include <new>
#include <string.h>

#include "gsgd_internal.hpp"

using namespace gsgd;

struct gsgd_ctx {
    gsgd_config cfg;          // host pointers inside are cleared after copying
    int         device;
    int64_t*    d_offsets;    // device copy of the segment table
    float*      d_scales;
    double*     d_partials;   // stats scratch: stats_num_blocks(d) * 4 doubles
    double*     d_result;     // max(4, k) doubles
    double*     h_result;     // pinned host, max(4, k) doubles
    double*     d_norm_partials;   // row-norm scratch: k * NORM_CHUNKS doubles
    uint32_t*   d_tickets;    // tile tickets of the persistent kernels (2 words, zero between launches)
    int         cu_count;     // compute units of the device
    unsigned    width[GSGD_KERNEL_COUNT];   // persistent workgroups per streaming kernel
    float       weight_decay;               // extras of the local step (Section 4.2); 0 / 0 = the boxed algorithms
    int         nesterov;
    int         last_hip;
};

namespace {

// Persistent workgroups per compute unit for each streaming kernel
// (GSGD_KERNEL_* order).  Measured on MI355X at the benchmark shapes.
constexpr unsigned DEFAULT_WORKGROUPS_PER_CU[GSGD_KERNEL_COUNT] = {1u, 1u, 1u, 4u, 2u, 1u};

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int hip_fail(gsgd_ctx* ctx, hipError_t e)
{
    if (ctx) ctx->last_hip = static_cast<int>(e);
    return GSGD_ERR_HIP;
}

inline Geom geom_of(const gsgd_ctx* c) { return Geom{c->cfg.k, c->cfg.d, c->cfg.ld}; }
inline Hyper hyper_of(const gsgd_ctx* c) { return Hyper{c->cfg.lr, c->cfg.momentum, c->weight_decay, c->nesterov}; }
inline SegTable seg_of(const gsgd_ctx* c) { return SegTable{c->d_offsets, c->d_scales, c->cfg.n_seg}; }
inline Persist persist_of(const gsgd_ctx* c, int kernel) { return Persist{c->d_tickets, c->width[kernel]}; }
inline RngKey key_of(const gsgd_ctx* c)
{
    return RngKey{static_cast<uint32_t>(c->cfg.seed), static_cast<uint32_t>(c->cfg.seed >> 32)};
}

// Row matrices must be non-null and 16-byte aligned (rows then are, since ld % 4 == 0).
inline bool ok_matrix(const void* p) { return p && aligned16(p); }

int check_state(const gsgd_ctx* ctx, const float* x, const float* v, const float* g)
{
    if (!ctx) return GSGD_ERR_INVALID_ARG;
    if (!ok_matrix(x) || !ok_matrix(v) || !ok_matrix(g)) return GSGD_ERR_INVALID_ARG;
    if (x == v || x == g || v == g) return GSGD_ERR_INVALID_ARG;
    return GSGD_OK;
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

extern "C" int gsgd_create(const gsgd_config* cfg, gsgd_ctx** out)
{
    if (!cfg || !out) return GSGD_ERR_INVALID_ARG;
    *out = nullptr;
    if (cfg->k < 1 || cfg->k > GSGD_MAX_K || cfg->d < 1 || cfg->ld < cfg->d || (cfg->ld & 3) != 0)
        return GSGD_ERR_INVALID_ARG;
    if (cfg->d > (static_cast<int64_t>(1) << 34)) return GSGD_ERR_INVALID_ARG;   // quad index is a 32-bit counter word
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
        e = hipMalloc(reinterpret_cast<void**>(&c->d_partials), sizeof(double) * 4 * static_cast<size_t>(stats_num_blocks(cfg->d)));
    const size_t n_result = static_cast<size_t>(cfg->k > 4 ? cfg->k : 4);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->d_result), sizeof(double) * n_result);
    if (e == hipSuccess)
        e = hipHostMalloc(reinterpret_cast<void**>(&c->h_result), sizeof(double) * n_result, hipHostMallocDefault);
    if (e == hipSuccess)
        e = hipMalloc(reinterpret_cast<void**>(&c->d_norm_partials),
                      sizeof(double) * static_cast<size_t>(cfg->k) * NORM_CHUNKS);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->d_tickets), 256);
    if (e == hipSuccess) e = hipMemset(c->d_tickets, 0, 256);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&c->cu_count, hipDeviceAttributeMultiprocessorCount, c->device);
    if (e == hipSuccess) {
        if (c->cu_count < 1) c->cu_count = 1;
        for (int kn = 0; kn < GSGD_KERNEL_COUNT; ++kn)
            c->width[kn] = static_cast<unsigned>(c->cu_count) * DEFAULT_WORKGROUPS_PER_CU[kn];
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

extern "C" int gsgd_comm_due(uint64_t step, uint32_t tau)
{
    if (tau == 0) return GSGD_ERR_INVALID_ARG;
    return (step + 1) % tau == 0 ? 1 : 0;
}

extern "C" int gsgd_set_launch_width(gsgd_ctx* ctx, int kernel, int workgroups)
{
    if (!ctx || kernel < 0 || kernel >= GSGD_KERNEL_COUNT || workgroups < 0 || workgroups > (1 << 20))
        return GSGD_ERR_INVALID_ARG;
    ctx->width[kernel] = workgroups > 0 ? static_cast<unsigned>(workgroups)
                                        : static_cast<unsigned>(ctx->cu_count) * DEFAULT_WORKGROUPS_PER_CU[kernel];
    return GSGD_OK;
}

extern "C" int gsgd_init_replicas(gsgd_ctx* ctx, float* x, float* v, float* center, const float* x0, int mode,
                                  void* stream)
{
    if (!ctx || !ok_matrix(x) || !ok_matrix(v) || x == v) return GSGD_ERR_INVALID_ARG;
    if (mode != GSGD_INIT_BROADCAST && mode != GSGD_INIT_PER_REPLICA) return GSGD_ERR_INVALID_ARG;
    if (mode == GSGD_INIT_BROADCAST && !ok_matrix(x0)) return GSGD_ERR_INVALID_ARG;
    if (center && !aligned16(center)) return GSGD_ERR_INVALID_ARG;
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

extern "C" int gsgd_gen_grad(gsgd_ctx* ctx, const float* x, const float* h, const float* xstar, float* g,
                             uint64_t step, void* stream)
{
    if (!ctx || !ok_matrix(x) || !ok_matrix(g) || !ok_matrix(h) || !ok_matrix(xstar) || x == g)
        return GSGD_ERR_INVALID_ARG;
    if (step > 0xFFFFFFFFull) return GSGD_ERR_INVALID_ARG;
    const hipError_t e = launch_gen_grad(geom_of(ctx), x, h, xstar, g, ctx->cfg.sigma, key_of(ctx),
                                         static_cast<uint32_t>(step), ctx->cfg.noise_kind,
                                         persist_of(ctx, GSGD_KERNEL_GEN_GRAD), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_philox_raw(gsgd_ctx* ctx, uint32_t c1, uint32_t c2, uint32_t c3, int64_t n_blocks, uint32_t* out,
                               void* stream)
{
    if (!ctx || !out || n_blocks < 1 || n_blocks > (static_cast<int64_t>(1) << 32)) return GSGD_ERR_INVALID_ARG;
    const hipError_t e = launch_philox_raw(key_of(ctx), c1, c2, c3, n_blocks, out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_step_allreduce(gsgd_ctx* ctx, float* x, float* v, const float* g, void* stream)
{
    const int rc = check_state(ctx, x, v, g);
    if (rc != GSGD_OK) return rc;
    const hipError_t e = launch_step_allreduce(geom_of(ctx), hyper_of(ctx), seg_of(ctx), x, v, g,
                                               persist_of(ctx, GSGD_KERNEL_ALLREDUCE), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

namespace {
int gossip_on_permutation(gsgd_ctx* ctx, float* x, float* v, const float* g, const int32_t* peer_perm, float beta,
                          bool stale, void* stream)
{
    int rc = check_state(ctx, x, v, g);
    if (rc != GSGD_OK) return rc;
    if (!peer_perm || !(beta == beta)) return GSGD_ERR_INVALID_ARG;
    Walk walk;
    rc = build_walk(peer_perm, ctx->cfg.k, &walk);
    if (rc != GSGD_OK) return rc;
    const hipError_t e = launch_step_gossip(geom_of(ctx), hyper_of(ctx), seg_of(ctx), beta, walk, stale, false, x, v, g,
                                            persist_of(ctx, GSGD_KERNEL_GOSSIP), static_cast<hipStream_t>(stream));
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
    const hipError_t e = launch_step_gossip(geom_of(ctx), hyper_of(ctx), seg_of(ctx), beta, walk, stale != 0,
                                            has_trees != 0, x, v, g, persist_of(ctx, GSGD_KERNEL_GOSSIP),
                                            static_cast<hipStream_t>(stream));
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
    const hipError_t e = launch_step_gossip_push(geom_of(ctx), hyper_of(ctx), seg_of(ctx), walk, x, v, g,
                                                 persist_of(ctx, GSGD_KERNEL_GOSSIP), static_cast<hipStream_t>(stream));
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
    if (!ok_matrix(center) || center == x || center == v || center == g || !(alpha_e == alpha_e))
        return GSGD_ERR_INVALID_ARG;
    if (i < 0 || i >= ctx->cfg.k) return GSGD_ERR_INVALID_ARG;
    const hipError_t e = launch_easgd_tick(geom_of(ctx), hyper_of(ctx), seg_of(ctx), alpha_e, i, x, v, g, center,
                                           static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_step_async_tick_fused(gsgd_ctx* ctx, float* x, float* v, const float* h, const float* xstar,
                                          int32_t i, int32_t j, float beta, uint64_t tick, void* stream)
{
    if (!ctx || !ok_matrix(x) || !ok_matrix(v) || !ok_matrix(h) || !ok_matrix(xstar) || x == v)
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
    const hipError_t e = launch_step_local(geom_of(ctx), hyper_of(ctx), seg_of(ctx), x, v, g,
                                           persist_of(ctx, GSGD_KERNEL_LOCAL), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

namespace {
int check_fused(const gsgd_ctx* ctx, const float* x, const float* v, const float* h, const float* xstar,
                const int32_t* map, uint64_t step)
{
    if (!ctx || !ok_matrix(x) || !ok_matrix(v) || !ok_matrix(h) || !ok_matrix(xstar) || x == v)
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
    const hipError_t e = launch_step_gossip_fused(geom_of(ctx), hyper_of(ctx), seg_of(ctx), beta, walk, false, false,
                                                  x, v, h, xstar, ctx->cfg.sigma, key_of(ctx),
                                                  static_cast<uint32_t>(step), ctx->cfg.noise_kind,
                                                  persist_of(ctx, GSGD_KERNEL_GOSSIP_FUSED),
                                                  static_cast<hipStream_t>(stream));
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
    const hipError_t e = launch_step_gossip_fused(geom_of(ctx), hyper_of(ctx), seg_of(ctx), beta, walk, stale != 0,
                                                  has_trees != 0, x, v, h, xstar, ctx->cfg.sigma, key_of(ctx),
                                                  static_cast<uint32_t>(step), ctx->cfg.noise_kind,
                                                  persist_of(ctx, GSGD_KERNEL_GOSSIP_FUSED),
                                                  static_cast<hipStream_t>(stream));
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
    const hipError_t e = launch_step_gossip_push_fused(geom_of(ctx), hyper_of(ctx), seg_of(ctx), walk, x, v, h, xstar,
                                                       ctx->cfg.sigma, key_of(ctx), static_cast<uint32_t>(step),
                                                       ctx->cfg.noise_kind, persist_of(ctx, GSGD_KERNEL_GOSSIP_FUSED),
                                                       static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_step_easgd(gsgd_ctx* ctx, float* x, float* v, const float* g,
                               float* center, float alpha_e, void* stream)
{
    const int rc = check_state(ctx, x, v, g);
    if (rc != GSGD_OK) return rc;
    if (!ok_matrix(center) || center == x || center == v || center == g || !(alpha_e == alpha_e))
        return GSGD_ERR_INVALID_ARG;
    const hipError_t e = launch_step_easgd(geom_of(ctx), hyper_of(ctx), seg_of(ctx), alpha_e, x, v, g, center,
                                           persist_of(ctx, GSGD_KERNEL_EASGD), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSGD_OK : hip_fail(ctx, e);
}

extern "C" int gsgd_stats(gsgd_ctx* ctx, const float* x, const float* xstar, double out[4], void* stream)
{
    if (!ctx || !ok_matrix(x) || !ok_matrix(xstar) || !out) return GSGD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = launch_stats(geom_of(ctx), x, xstar, ctx->d_partials, ctx->d_result, s);
    if (e == hipSuccess) e = hipMemcpyAsync(ctx->h_result, ctx->d_result, sizeof(double) * 4, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(ctx, e);
    for (int m = 0; m < 4; ++m) out[m] = ctx->h_result[m];
    return GSGD_OK;
}

extern "C" int gsgd_row_sqnorms(gsgd_ctx* ctx, const float* x, double* out, void* stream)
{
    if (!ctx || !ok_matrix(x) || !out) return GSGD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = launch_row_sqnorms(geom_of(ctx), x, ctx->d_norm_partials, ctx->d_result, s);
    if (e == hipSuccess)
        e = hipMemcpyAsync(ctx->h_result, ctx->d_result, sizeof(double) * static_cast<size_t>(ctx->cfg.k),
                           hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(ctx, e);
    for (int32_t i = 0; i < ctx->cfg.k; ++i) out[i] = ctx->h_result[i];
    return GSGD_OK;
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
        case GSGD_ERR_UNSUPPORTED: return "unsupported";
        case GSGD_ERR_NO_MEMORY: return "out of memory";
        default: return "unknown error";
    }
}

extern "C" int gsgd_last_hip_error(const gsgd_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

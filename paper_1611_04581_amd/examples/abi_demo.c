/*
 * abi_demo.c -- libgsgd through its C ABI alone: plain C, device memory from
 * hipMalloc, no Python and no PyTorch anywhere.
 *
 * Runs pull-gossip SGD (a fresh random peer permutation per step, then iid
 * targets) on the synthetic noisy quadratic for k replicas that start apart,
 * and checks what the method promises: the replicas are pulled together
 * (consensus distance falls by orders of magnitude), they approach the
 * optimum, and a step whose mix is a permutation leaves the replica mean
 * where the local step put it.  Exit status 0 and a line "abi_demo ok" on
 * success.  Optional argument: columns per block of the matrix layout (default
 * 16384; 0 = row-major).
 *
 * Build (done by the package's build step):
 *   gcc -std=c99 abi_demo.c -I <repo>/include -I /opt/rocm/include -L <dir of libgsgd.so> -L /opt/rocm/lib \
 *       -lgsgd -lamdhip64 -lm -Wl,-rpath,'$ORIGIN'
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>

#include "gsgd.h"

#define CHECK_HIP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { \
    fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_GSGD(call) do { int rc_ = (call); if (rc_ != GSGD_OK) { \
    fprintf(stderr, "%s failed: %s (%d)\n", #call, gsgd_strerror(rc_), rc_); return 3; } } while (0)

int main(int argc, char** argv)
{
    enum { K = 8 };
    /* matrices in blocks of 16,384 columns (the layout the kernels stream fastest), or what the first argument says
     * (0 = row-major with the row stride rounded up to 1024) */
    const int64_t block = argc > 1 ? atoll(argv[1]) : 16384;
    const int64_t unit = block > 0 ? block : 1024;
    const int64_t d = 300 * 1000 + 3, ld = (d + unit - 1) / unit * unit;
    const uint64_t seed = 0x161104581ull;
    gsgd_config cfg = { K, d, ld, 0.05f, 0.9f, 0.05f, seed, GSGD_NOISE_GAUSSIAN, 0, NULL, NULL, block };
    gsgd_ctx* ctx = NULL;
    CHECK_GSGD(gsgd_create(&cfg, &ctx));

    float *x, *v, *g, *h, *xstar, *xl, *vl;
    const size_t rows = sizeof(float) * (size_t)K * (size_t)ld, vec = sizeof(float) * (size_t)ld;
    CHECK_HIP(hipMalloc((void**)&x, rows));
    CHECK_HIP(hipMalloc((void**)&v, rows));
    CHECK_HIP(hipMalloc((void**)&g, rows));
    CHECK_HIP(hipMalloc((void**)&xl, rows));
    CHECK_HIP(hipMalloc((void**)&vl, rows));
    CHECK_HIP(hipMalloc((void**)&h, vec));
    CHECK_HIP(hipMalloc((void**)&xstar, vec));
    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));

    CHECK_GSGD(gsgd_fill(ctx, h, GSGD_FILL_H, stream));
    CHECK_GSGD(gsgd_fill(ctx, xstar, GSGD_FILL_XSTAR, stream));
    CHECK_GSGD(gsgd_init_replicas(ctx, x, v, NULL, NULL, GSGD_INIT_PER_REPLICA, stream));

    double before[4], after[4];
    CHECK_GSGD(gsgd_stats(ctx, x, xstar, before, stream));

    int32_t peer[K];
    for (uint64_t t = 0; t < 120; ++t) {
        CHECK_GSGD(gsgd_gen_grad(ctx, x, h, xstar, g, t, stream));
        if (t % 2 == 0) {
            CHECK_GSGD(gsgd_make_perm(seed, t, K, peer));
            CHECK_GSGD(gsgd_step_gossip(ctx, x, v, g, peer, 0.5f, stream));
        } else {
            CHECK_GSGD(gsgd_make_targets(seed, t, K, 0, peer));
            CHECK_GSGD(gsgd_step_gossip_pull(ctx, x, v, g, peer, 0.5f, 0, stream));
        }
    }
    CHECK_GSGD(gsgd_stats(ctx, x, xstar, after, stream));
    printf("consensus distance %.4g -> %.4g, distance to the optimum %.4g -> %.4g\n",
           before[0], after[0], before[1], after[1]);
    int ok = after[0] < 1e-3 * before[0] && after[1] < 1e-2 * before[1];

    /* a permutation mix moves no mass: same call with beta = 0 (local step only) on a copy, compare the means */
    CHECK_GSGD(gsgd_gen_grad(ctx, x, h, xstar, g, 1000, stream));
    CHECK_HIP(hipMemcpyAsync(xl, x, rows, hipMemcpyDeviceToDevice, stream));
    CHECK_HIP(hipMemcpyAsync(vl, v, rows, hipMemcpyDeviceToDevice, stream));
    CHECK_GSGD(gsgd_make_perm(seed, 1000, K, peer));
    CHECK_GSGD(gsgd_step_gossip(ctx, xl, vl, g, peer, 0.0f, stream));
    CHECK_GSGD(gsgd_step_gossip(ctx, x, v, g, peer, 0.5f, stream));
    double mixed[4], local[4];
    CHECK_GSGD(gsgd_stats(ctx, x, xstar, mixed, stream));
    CHECK_GSGD(gsgd_stats(ctx, xl, xstar, local, stream));
    /* out[3] = ||mean||^2, out[2] = ||mean - xstar||^2: equal means give equal values */
    const double rel = fabs(mixed[3] - local[3]) / local[3] + fabs(mixed[2] - local[2]) / (local[2] + 1e-30);
    printf("replica mean after the mix vs after the local step alone: relative difference %.3g\n", rel);
    ok = ok && rel < 1e-5 && mixed[0] < local[0];

    /* error paths come back as codes */
    peer[0] = peer[1];
    ok = ok && gsgd_step_gossip(ctx, x, v, g, peer, 0.5f, stream) == GSGD_ERR_BAD_PERM;
    ok = ok && gsgd_step_gossip(ctx, x, x, g, peer, 0.5f, stream) == GSGD_ERR_INVALID_ARG;

    CHECK_HIP(hipStreamSynchronize(stream));
    CHECK_GSGD(gsgd_destroy(ctx));
    CHECK_HIP(hipStreamDestroy(stream));
    hipFree(x); hipFree(v); hipFree(g); hipFree(xl); hipFree(vl); hipFree(h); hipFree(xstar);
    if (!ok) { fprintf(stderr, "abi_demo FAILED\n"); return 1; }
    printf("abi_demo ok\n");
    return 0;
}

"""Throughput of the gossip step on one MI355X.

Metric: replica-steps/s (= k x gossip steps per second) of gsgd_step_gossip at
ResNet-50-sized vectors (d = 25,557,032 fp32) with k = 32 replicas, a fresh
seeded peer permutation per step, x / v / g resident in HBM.  One JSON line on
stdout; progress on stderr.

Also reported in the same line: the roofline of the dominant kernel (the fused
SGD+momentum+mix kernel, HBM-bound, 20 algorithmic bytes per replica-element),
the cost of the synthetic-gradient generator and of the full simulated
iteration, and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published peak HBM3E bandwidth
BYTES_PER_REPLICA_ELEMENT = {   # algorithmic traffic of each kernel, fp32
    "gossip": 20.0,             # read x, v, g; write x, v
    "allreduce": 20.0,
    "easgd": 20.0,              # + 8/k for the centre, added below
}
# HBM bytes per launch of the gossip kernel at the benchmark shape, from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs scaled by a copy kernel of known
# size (see profiles/); None until measured.
MEASURED_TRAFFIC_BYTES = {
    # profiles/gossip_step_kernel_gossip_r50.md: FETCH_SIZE 4,792,017.0 x 2.000 KiB + WRITE_SIZE 6,390,054.1 KiB
    "gossip_r50": (4792017.0 * 2.0 + 6390054.1) * 1024.0,
}


KERNEL_OF_RULE = {"gossip": "gossip_step_kernel", "gossip_stale": "gossip_step_kernel (stale)",
                  "gossip_pull": "gossip_step_kernel (tree walk)", "gossip_push": "push_step_kernel",
                  "allreduce": "allreduce_step_kernel", "easgd": "easgd_step_kernel",
                  "async_tick": "async_tick_kernel (generator fused, one launch per tick)"}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", default="gossip_r50")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget for the oracle baseline (0 = skip)")
    ap.add_argument("--no-extras", action="store_true", help="time only the metric kernel")
    ap.add_argument("--no-fused", action="store_true", help="skip the fused-generator extra")
    ap.add_argument("--launch-width", type=int, default=0,
                    help="persistent workgroups per streaming kernel (0 = the library's default)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain elementwise copy of a k x ld fp32 matrix (known size), so that a "
                         "rocprofv3 --pmc run has a reference dispatch to scale FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU (k replicas live in one GPU's HBM); run with --gpus 1")

    import numpy as np
    import torch
    from paper_1611_04581_amd import gsgd, workloads as W

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the library has no CPU fallback")
    torch.cuda.set_device(0)
    cfg = W.CONFIGS[args.config]
    k, d = cfg.k, cfg.d
    ld = W.round_up(d, 1024)
    seg = {}
    if cfg.layout:
        off, sc, _ = W.resnet_layout(cfg.layout)
        seg = dict(seg_offsets=off, seg_lr_scale=sc)
    K, Wm = args.steps, args.warmup
    log("config %s: rule=%s k=%d d=%d ld=%d steps=%d warmup=%d" % (cfg.name, cfg.rule, k, d, ld, K, Wm))

    ctx = gsgd.Context(k, d, ld, lr=cfg.lr, momentum=cfg.momentum, sigma=cfg.sigma, seed=cfg.seed,
                       noise_kind=gsgd.NOISE_GAUSSIAN, **seg)
    if args.launch_width:
        for kern in range(gsgd.KERNEL_COUNT):
            ctx.set_launch_width(kern, args.launch_width)
    x = torch.empty((k, ld), dtype=torch.float32, device="cuda")
    v = torch.empty_like(x)
    g = torch.empty_like(x)
    h = torch.empty(ld, dtype=torch.float32, device="cuda")
    xstar = torch.empty_like(h)
    x0 = torch.empty_like(h)
    center = torch.empty_like(h)
    ctx.fill(h, gsgd.FILL_H)
    ctx.fill(xstar, gsgd.FILL_XSTAR)
    ctx.fill(x0, gsgd.FILL_X0)
    ctx.init_replicas(x, v, center, x0, gsgd.INIT_BROADCAST)
    ctx.gen_grad(x, h, xstar, g, 0)
    torch.cuda.synchronize()
    if args.calibrate_copy:
        # reads k*ld*4 bytes and writes k*ld*4 bytes; g is regenerated right after
        torch.mul(x, 1.0, out=g)
        torch.cuda.synchronize()
        log("calibration copy: %d bytes read, %d bytes written" % (k * ld * 4, k * ld * 4))
        ctx.gen_grad(x, h, xstar, g, 0)
        torch.cuda.synchronize()

    ctx.set_local_step(cfg.weight_decay, cfg.nesterov)

    def one_step(t):
        rule = cfg.rule if gsgd.comm_due(t, cfg.tau) else "local"
        if rule == "gossip":
            ctx.step_gossip(x, v, g, gsgd.make_perm(cfg.seed, t, k), cfg.beta)
        elif rule == "gossip_stale":
            ctx.step_gossip_stale(x, v, g, gsgd.make_perm(cfg.seed, t, k), cfg.beta)
        elif rule == "gossip_pull":
            ctx.step_gossip_pull(x, v, g, gsgd.make_targets(cfg.seed, t, k), cfg.beta)
        elif rule == "gossip_push":
            ctx.step_gossip_push(x, v, g, gsgd.make_targets(cfg.seed, t, k, True))
        elif rule == "local":
            ctx.step_local(x, v, g)
        elif rule == "async_tick":                      # k ticks of the one-node-per-tick model = k replica-steps
            ctx.run_async_ticks(x, v, h, xstar, t * k, k, cfg.beta)
        elif rule == "allreduce":
            ctx.step_allreduce(x, v, g)
        else:
            ctx.step_easgd(x, v, g, center, cfg.alpha_e)

    def timed(fn, n, t_start):
        """n calls of fn(t) bracketed by synchronize; returns (wall seconds, HIP-event seconds)."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        w0 = time.perf_counter()
        e0.record()
        for t in range(t_start, t_start + n):
            fn(t)
        e1.record()
        torch.cuda.synchronize()
        w1 = time.perf_counter()
        return w1 - w0, e0.elapsed_time(e1) * 1e-3

    # ---- the metric: K step calls on resident x, v, g -----------------------------------
    for t in range(Wm):
        one_step(t)
    wall, ev = timed(one_step, K, Wm)
    ms_per_step = wall / K * 1e3
    value = k * K / wall
    bpe = BYTES_PER_REPLICA_ELEMENT.get(cfg.rule, 20.0) + (8.0 / k if cfg.rule == "easgd" else 0.0)
    alg_bytes = bpe * k * d
    kern_s = ev / K                                  # one kernel per step in the timed region
    if cfg.rule == "async_tick":
        # per tick and element of the ticking row: x_i, v_i, h, xstar and the peer's x read (the peer's only when
        # j != i, probability 1 - 1/k), x_i and v_i written; k launches per step
        alg_bytes = (28.0 - 4.0 / k) * d
        kern_s = ev / (K * k)
    achieved = alg_bytes / kern_s / 1e9
    traffic = MEASURED_TRAFFIC_BYTES.get(cfg.name)
    log("step: %.3f ms wall, %.3f ms by HIP events -> %.0f replica-steps/s, %.0f GB/s algorithmic (%.1f%% of peak)"
        % (ms_per_step, kern_s * 1e3, value, achieved, 100 * achieved / HBM_PEAK_GBS))

    out = {
        "metric": "replica-steps/sec + achieved HBM GB/s, gossip step, ResNet-50-size d, k=32" if cfg.name == "gossip_r50"
                  else "replica-steps/sec, %s step" % cfg.rule,
        "value": value, "unit": "replica-steps/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: k=%d replicas, d=%d fp32 (row stride %d), rule=%s, fresh Philox peer permutation "
                               "per step, x/v/g resident in HBM" % (cfg.name, k, d, ld, cfg.rule),
                   "k": k, "d": d, "ld": ld, "rule": cfg.rule, "lr": cfg.lr, "momentum": cfg.momentum,
                   "beta": cfg.beta, "sigma": cfg.sigma, "layout": cfg.layout or "flat"},
        "roofline": {"bound": "hbm", "kernel": KERNEL_OF_RULE[cfg.rule], "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": kern_s * 1e3},
    }

    # ---- context: generator and full simulated iteration --------------------------------
    if not args.no_extras:
        n2 = min(100, max(10, K // 4))
        t_next = Wm + K
        w_gen, e_gen = timed(lambda t: ctx.gen_grad(x, h, xstar, g, t), n2, t_next)

        def full(t):
            ctx.gen_grad(x, h, xstar, g, t)
            one_step(t)
        w_full, e_full = timed(full, n2, t_next + n2)
        extras = {
            "gen_grad_ms": e_gen / n2 * 1e3,
            "gen_grad_GBps_algorithmic": (8.0 + 8.0 / k) * k * d / (e_gen / n2) / 1e9,
            "full_iteration_ms": w_full / n2 * 1e3,
            "full_iteration_replica_steps_per_s": k * n2 / w_full,
        }
        if cfg.rule == "gossip" and not args.no_fused:
            def fused(t):
                ctx.step_gossip_fused(x, v, h, xstar, gsgd.make_perm(cfg.seed, t, k), t, cfg.beta)
            for t in range(3):
                fused(t_next + 2 * n2 + t)
            w_fu, e_fu = timed(fused, n2, t_next + 2 * n2 + 3)
            extras["fused_iteration_ms"] = w_fu / n2 * 1e3
            extras["fused_iteration_replica_steps_per_s"] = k * n2 / w_fu
            extras["fused_iteration_GBps_algorithmic"] = (16.0 + 8.0 / k) * k * d / (e_fu / n2) / 1e9
        # what this machine's memory delivers to a plain device-to-device copy of the same matrices (read 4 B, write 4 B per
        # element), as context for the fractions above; g is regenerated by the next gen_grad
        scratch = torch.empty_like(g)
        w_cp, e_cp = timed(lambda t: scratch.copy_(g), 20, 0)
        extras["plain_copy_GBps"] = 8.0 * k * ld / (e_cp / 20) / 1e9
        del scratch
        if cfg.name == "gossip_r50":
            # the other gossip forms on the same resident state (same 20 B per replica-element)
            forms = {
                "pull_gossip_iid_targets": lambda t: ctx.step_gossip_pull(x, v, g, gsgd.make_targets(cfg.seed, t, k), cfg.beta),
                "push_gossip": lambda t: ctx.step_gossip_push(x, v, g, gsgd.make_targets(cfg.seed, t, k, True)),
                "stale_parameter_gossip": lambda t: ctx.step_gossip_stale(x, v, g, gsgd.make_perm(cfg.seed, t, k), cfg.beta),
                "local_step_only": lambda t: ctx.step_local(x, v, g),
            }
            for name, fn in forms.items():
                for t in range(3):
                    fn(t)
                w_f, e_f = timed(fn, n2, 1000)
                extras[name + "_ms"] = e_f / n2 * 1e3
                extras[name + "_frac_of_hbm_peak"] = 20.0 * k * d / (e_f / n2) / 1e9 / HBM_PEAK_GBS
        out["extras"] = extras
        log("extras:", json.dumps(extras))

    # ---- CPU baseline: the oracle, as it stands, on a bounded sample ---------------------
    if args.cpu_seconds > 0:
        from oracle import oracle
        ds = min(d, 1 << 20)                       # first 2^20 columns of every replica row
        inp = W.make_inputs(k, ds, seed=5)
        perm0 = oracle.make_perm(cfg.seed, 0, k)
        lrc = np.full(ds, np.float32(cfg.lr), np.float32)

        def ostep(t):
            if cfg.rule == "gossip":
                oracle.step_gossip(inp.x, inp.v, inp.g, lrc, cfg.momentum, cfg.beta, oracle.make_perm(cfg.seed, t, k))
            elif cfg.rule in ("gossip_stale", "gossip_pull"):
                peer = oracle.make_perm(cfg.seed, t, k) if cfg.rule == "gossip_stale" else oracle.make_targets(cfg.seed, t, k)
                oracle.step_gossip_ext(inp.x, inp.v, inp.g, lrc, cfg.momentum, cfg.beta, peer, wd=cfg.weight_decay,
                                       nesterov=cfg.nesterov, stale=cfg.rule == "gossip_stale")
            elif cfg.rule == "gossip_push":
                oracle.step_gossip_push(inp.x, inp.v, inp.g, lrc, cfg.momentum, oracle.make_targets(cfg.seed, t, k, True),
                                        wd=cfg.weight_decay, nesterov=cfg.nesterov)
            elif cfg.rule == "async_tick":
                for tick in range(t * k, (t + 1) * k):
                    i, j = oracle.make_tick(cfg.seed, tick, k)
                    oracle.gen_grad_row(inp.x, inp.h, inp.xstar, inp.g[0], i, cfg.sigma, cfg.seed, tick)
                    oracle.async_tick(inp.x, inp.v, inp.g[0], lrc, cfg.momentum, cfg.beta, i, j)
            elif cfg.rule == "allreduce":
                oracle.step_allreduce(inp.x, inp.v, inp.g, lrc, cfg.momentum)
            else:
                oracle.step_easgd(inp.x, inp.v, inp.g, inp.center, lrc, cfg.momentum, cfg.alpha_e)
        ostep(0)
        n_cpu, t0 = 0, time.perf_counter()
        while time.perf_counter() - t0 < args.cpu_seconds:
            ostep(n_cpu + 1)
            n_cpu += 1
        cpu_wall = time.perf_counter() - t0
        cpu_value = k * n_cpu / cpu_wall * (ds / d)      # scaled to full-length rows
        cores = oracle.num_threads()
        # the same oracle on one thread, a quarter of the budget
        oracle.set_num_threads(1)
        n_one, t1 = 0, time.perf_counter()
        while time.perf_counter() - t1 < args.cpu_seconds / 4 or n_one == 0:
            ostep(n_cpu + n_one + 1)
            n_one += 1
        one_wall = time.perf_counter() - t1
        oracle.set_num_threads(cores)
        out["cpu_baseline"] = {
            "value": cpu_value, "unit": "replica-steps/s", "cores": cores, "kind": "oracle",
            "one_thread_value": k * n_one / one_wall * (ds / d),
            "sample": "%d %s steps of the C oracle on the first %d of %d columns of all %d replicas (%.1f s); "
                      "rate scaled by %d/%d to full-length rows" % (n_cpu, cfg.rule, ds, d, k, cpu_wall, ds, d),
        }
        log("cpu oracle: %.2f replica-steps/s on %d threads, %.2f on one" % (cpu_value, cores, k * n_one / one_wall * (ds / d)))

    ctx.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

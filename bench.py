"""Throughput of the gossip step on one MI355X.

Metric: replica-steps/s (= k x gossip steps per second) of gsgd_step_gossip at
ResNet-50-sized vectors (d = 25,557,032 fp32) with k = 32 replicas, a fresh
seeded peer permutation per step, x / v / g resident in HBM.  One JSON line on
stdout; progress on stderr.

In the same line:
  roofline      the dominant kernel (fused SGD + momentum + mix, HBM-bound, 20
                algorithmic bytes per replica-element) over the K timed steps,
                plus the spread of the same measurement over fresh allocations
                of x / v / g (the rate depends on where the driver places them);
  extras        the synthetic-gradient generator and the generator-fused step
                with their ALU-only and HBM-only times, the other gossip forms
                at the metric shape, the other benchmark configurations as short
                legs, and what a plain copy gets on this machine;
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published peak HBM3E bandwidth
SIMDS = 1024                   # 256 compute units x 4 SIMDs
PEAK_CLOCK_HZ = 2.4e9

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (KiB per dispatch, each scaled by what the
# same counter reads for a plain copy of known size).  These come from the profile runs summarised under profiles/,
# NOT from the run that prints them: a bench run cannot read hardware counters.  None = no such profile yet.
def _kib(fetch_size, write_size):
    """FETCH_SIZE reads half the KiB fetched, WRITE_SIZE the KiB written (both calibrated on a plain copy)."""
    return (fetch_size * 2.0 + write_size) * 1024.0


_GOSSIP_R50 = "profiles/gossip_step_kernel_gossip_r50.md"
_OTHERS = "profiles/step_kernels_other_workloads.md"
_GENERATOR = "profiles/generator_kernels_alu_vs_hbm.md"
TRAFFIC_FROM_PROFILES = {
    # name: (bytes per launch, source)
    "gossip_r50": (_kib(4792037.3, 6390778.6), _GOSSIP_R50),
    "stale_gossip_r50": (_kib(4792028.2, 6390059.6), _GOSSIP_R50),
    "pull_gossip_r50": (_kib(4792032.3, 6390840.2), _OTHERS),
    "push_gossip_r50": (_kib(4792027.0, 6390304.0), _GOSSIP_R50),
    "local_r50": (_kib(4792016.9, 6390055.1), _GOSSIP_R50),
    "allreduce_r18": (_kib(548018.5, 730983.1), _OTHERS),
    "gossip_r18": (_kib(2191852.5, 2923219.8), _OTHERS),
    "easgd_r50": (_kib(2445969.7, 3295277.8), _OTHERS),
    "seg_gossip_r50_k128": (_kib(19167946.7, 25562415.2), _OTHERS),
    "gen_grad@gossip_r50": (_kib(1697262.5, 3195443.6), _GENERATOR),
    "fused@gossip_r50": (_kib(3294575.8, 6390697.4), _GENERATOR),
}
TRAFFIC_NOTE = ("rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE, each scaled by a plain copy of known size; a separate "
                "profile run, not this run")


def traffic_of(name):
    t, src = TRAFFIC_FROM_PROFILES.get(name, (None, None))
    return {"traffic": t, "traffic_source": "%s (%s)" % (src, TRAFFIC_NOTE) if src else None}


KERNEL_OF_RULE = {"gossip": "gossip_step_kernel", "gossip_stale": "gossip_step_kernel (stale)",
                  "gossip_pull": "gossip_step_kernel (tree walk)", "gossip_push": "push_step_kernel",
                  "allreduce": "allreduce_step_kernel", "easgd": "easgd_step_kernel", "local": "local_step_kernel",
                  "async_tick": "async_tick_kernel (generator fused, one launch per tick)"}
# on blocked matrices the gossip rules run as two ascending sweeps, the local step as a row walk
KERNEL_OF_RULE_BLOCKED = {"gossip": "gossip_sweep_kernel", "gossip_stale": "gossip_sweep_kernel (stale)",
                          "gossip_pull": "gossip_sweep_kernel", "gossip_push": "push_sweep_kernel",
                          "local": "local_walk_kernel"}


def kernel_of(rule, block_columns):
    if block_columns and rule in KERNEL_OF_RULE_BLOCKED:
        return KERNEL_OF_RULE_BLOCKED[rule]
    return KERNEL_OF_RULE[rule]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def bytes_per_replica_element(rule, k):
    """Algorithmic HBM traffic of one step, fp32: x, v, g read and x, v written (+ the centre for elastic averaging)."""
    return 20.0 + (8.0 / k if rule == "easgd" else 0.0)


class Run:
    """One configuration with its state resident on the GPU."""

    def __init__(self, gsgd, W, cfg, launch_width=0, ld=0, block_columns=None):
        """block_columns: None = the blocked layout the configuration names, 0 = row-major matrices."""
        import torch
        self.gsgd, self.cfg, self.torch = gsgd, cfg, torch
        k, d = cfg.k, cfg.d
        if block_columns is None:
            block_columns = 0 if ld else cfg.block_columns           # an explicit row stride means row-major
        self.k, self.d, self.ld = k, d, (ld if ld else W.round_up(d, block_columns if block_columns else 1024))
        self.block_columns = block_columns
        seg = {}
        if cfg.layout:
            off, sc, _ = W.resnet_layout(cfg.layout)
            seg = dict(seg_offsets=off, seg_lr_scale=sc)
        self.ctx = gsgd.Context(k, d, self.ld, lr=cfg.lr, momentum=cfg.momentum, sigma=cfg.sigma, seed=cfg.seed,
                                noise_kind=gsgd.NOISE_GAUSSIAN, block_columns=block_columns, **seg)
        if launch_width:
            for kern in range(gsgd.KERNEL_COUNT):
                self.ctx.set_launch_width(kern, launch_width)
        self.h = torch.empty(self.ld, dtype=torch.float32, device="cuda")
        self.xstar = torch.empty_like(self.h)
        self.x0 = torch.empty_like(self.h)
        self.center = torch.empty_like(self.h)
        self.ctx.fill(self.h, gsgd.FILL_H)
        self.ctx.fill(self.xstar, gsgd.FILL_XSTAR)
        self.ctx.fill(self.x0, gsgd.FILL_X0)
        self.x = self.v = self.g = None
        self.allocate()
        self.ctx.set_local_step(cfg.weight_decay, cfg.nesterov)

    def allocate(self):
        """Fresh device allocations of x, v, g (the old ones go back to the driver first), initialised as the
        algorithms start: every replica at x0, momentum zero, one gradient drawn."""
        torch = self.torch
        self.x = self.v = self.g = None
        torch.cuda.empty_cache()
        self.x = torch.empty((self.k, self.ld), dtype=torch.float32, device="cuda")
        self.v = torch.empty_like(self.x)
        self.g = torch.empty_like(self.x)
        self.ctx.init_replicas(self.x, self.v, self.center, self.x0, self.gsgd.INIT_BROADCAST)
        self.ctx.gen_grad(self.x, self.h, self.xstar, self.g, 0)
        torch.cuda.synchronize()

    def step(self, t):
        gsgd, cfg, ctx, x, v, g = self.gsgd, self.cfg, self.ctx, self.x, self.v, self.g
        rule = cfg.rule if gsgd.comm_due(t, cfg.tau) else "local"
        if rule == "gossip":
            ctx.step_gossip(x, v, g, gsgd.make_perm(cfg.seed, t, self.k), cfg.beta)
        elif rule == "gossip_stale":
            ctx.step_gossip_stale(x, v, g, gsgd.make_perm(cfg.seed, t, self.k), cfg.beta)
        elif rule == "gossip_pull":
            ctx.step_gossip_pull(x, v, g, gsgd.make_targets(cfg.seed, t, self.k), cfg.beta)
        elif rule == "gossip_push":
            ctx.step_gossip_push(x, v, g, gsgd.make_targets(cfg.seed, t, self.k, True))
        elif rule == "local":
            ctx.step_local(x, v, g)
        elif rule == "async_tick":                      # k ticks of the one-node-per-tick model = k replica-steps
            ctx.run_async_ticks(x, v, self.h, self.xstar, t * self.k, self.k, cfg.beta)
        elif rule == "allreduce":
            ctx.step_allreduce(x, v, g)
        else:
            ctx.step_easgd(x, v, g, self.center, cfg.alpha_e)

    def timed(self, fn, n, t_start=0):
        """n calls of fn(t) between two HIP events on the stream the library launches on (torch's current stream),
        bracketed by synchronize; returns (wall seconds, HIP-event seconds)."""
        torch = self.torch
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

    def kernel_seconds(self, fn, n, t_start=0, repeats=3):
        """Median over `repeats` timed runs of n calls each of the HIP-event time per call: one host hiccup inside
        a timed region (the GPU idles, the events still count it) then spoils one run, not the figure."""
        per_call = []
        for r in range(repeats):
            _, ev = self.timed(fn, n, t_start + r * n)
            per_call.append(ev / n)
        return statistics.median(per_call)

    def algorithmic_bytes(self):
        cfg = self.cfg
        if cfg.rule == "async_tick":
            # per tick and element of the ticking row: x_i, v_i, h, xstar and the peer's x read (the peer's only when
            # j != i, probability 1 - 1/k), x_i and v_i written
            return (28.0 - 4.0 / self.k) * self.d
        return bytes_per_replica_element(cfg.rule, self.k) * self.k * self.d

    def launches_per_step(self):
        return self.k if self.cfg.rule == "async_tick" else 1

    def close(self):
        self.x = self.v = self.g = None
        self.ctx.close()
        self.torch.cuda.empty_cache()


def short_leg(gsgd, W, name, warmup=5, steps=30, repeats=3, fresh_allocations=0):
    """One of the other benchmark configurations as a short leg: median kernel time of `repeats` timed runs, and
    optionally the same measurement on `fresh_allocations` further allocations of x / v / g."""
    cfg = W.CONFIGS[name]
    run = Run(gsgd, W, cfg)
    try:
        def measure():
            for t in range(warmup):
                run.step(t)
            ms = []
            for r in range(repeats):
                _, ev = run.timed(run.step, steps, warmup + r * steps)
                ms.append(ev / (steps * run.launches_per_step()) * 1e3)
            return ms
        ms = measure()
        med = statistics.median(ms)
        out = {"rule": cfg.rule, "k": cfg.k, "d": cfg.d, "layout": cfg.layout or "flat",
               "block_columns": run.block_columns, "kernel_ms": med,
               "kernel_ms_min": min(ms), "kernel_ms_max": max(ms),
               "replica_steps_per_s": cfg.k / (med * run.launches_per_step() * 1e-3)}
        if name != "tiny":           # the tiny configuration lives in cache and is launch-bound: no bandwidth figure
            out["frac_of_hbm_peak"] = run.algorithmic_bytes() / (med * 1e-3) / 1e9 / HBM_PEAK_GBS
            out["algorithmic_bytes_per_launch"] = run.algorithmic_bytes()
            out.update(traffic_of(name))
            if fresh_allocations:
                fr = [out["frac_of_hbm_peak"]]
                for a in range(fresh_allocations):
                    run.allocate()
                    fr.append(run.algorithmic_bytes() / (statistics.median(measure()) * 1e-3) / 1e9 / HBM_PEAK_GBS)
                out["frac_of_hbm_peak_fresh_allocations"] = fr
        return out
    finally:
        run.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", default="gossip_r50")
    ap.add_argument("--repeats", type=int, default=5,
                    help="fresh allocations of x / v / g over which the kernel is timed (the first is the K-step run)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget for the oracle baseline (0 = skip)")
    ap.add_argument("--no-extras", action="store_true", help="time only the metric kernel")
    ap.add_argument("--no-fused", action="store_true", help="skip the fused-generator extra")
    ap.add_argument("--no-legs", action="store_true", help="skip the other benchmark configurations")
    ap.add_argument("--launch-width", type=int, default=0,
                    help="persistent workgroups per streaming kernel (0 = the library's default)")
    ap.add_argument("--ld", type=int, default=0,
                    help="row-major x / v / g with this row stride in elements (a multiple of 4, >= d)")
    ap.add_argument("--block-columns", type=int, default=-1,
                    help="columns per block of the blocked matrix layout (a power of two >= 1024); 0 = row-major "
                         "matrices with the row stride rounded up to 1024; default: what the configuration names")
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
    K, Wm = args.steps, args.warmup
    run = Run(gsgd, W, cfg, args.launch_width, args.ld, None if args.block_columns < 0 else args.block_columns)
    k, d, ld = run.k, run.d, run.ld
    ctx, h, xstar = run.ctx, run.h, run.xstar
    log("config %s: rule=%s k=%d d=%d ld=%d steps=%d warmup=%d" % (cfg.name, cfg.rule, k, d, ld, K, Wm))
    if args.calibrate_copy:
        # reads k*ld*4 bytes and writes k*ld*4 bytes; g is regenerated right after
        torch.mul(run.x, 1.0, out=run.g)
        torch.cuda.synchronize()
        log("calibration copy: %d bytes read, %d bytes written" % (k * ld * 4, k * ld * 4))
        ctx.gen_grad(run.x, h, xstar, run.g, 0)
        torch.cuda.synchronize()

    # ---- the metric: K step calls on resident x, v, g -----------------------------------
    for t in range(Wm):
        run.step(t)
    wall, ev = run.timed(run.step, K, Wm)
    ms_per_step = wall / K * 1e3
    value = k * K / wall
    alg_bytes = run.algorithmic_bytes()
    kern_s = ev / (K * run.launches_per_step())      # one kernel per launch in the timed region
    achieved = alg_bytes / kern_s / 1e9
    log("step: %.3f ms wall, %.3f ms by HIP events -> %.0f replica-steps/s, %.0f GB/s algorithmic (%.1f%% of peak)"
        "  (x, v, g at 0x%x 0x%x 0x%x)" % (ms_per_step, kern_s * 1e3, value, achieved, 100 * achieved / HBM_PEAK_GBS,
                                          run.x.data_ptr(), run.v.data_ptr(), run.g.data_ptr()))

    # ---- the same kernel on fresh allocations: the rate depends on the physical placement ----
    # (no reference to the old tensors may survive here, or the new ones are carved out next to them instead of
    # replacing them)
    fracs = [achieved / HBM_PEAK_GBS]
    n_rep = max(10, min(K, 100))
    for r in range(1, max(1, args.repeats)):
        run.allocate()
        for t in range(10):
            run.step(t)
        _, ev_r = run.timed(run.step, n_rep, 10)
        fracs.append(alg_bytes / (ev_r / (n_rep * run.launches_per_step())) / 1e9 / HBM_PEAK_GBS)
        log("  fresh allocation %d: %.1f%% of peak  (x, v, g at 0x%x 0x%x 0x%x)"
            % (r, 100 * fracs[-1], run.x.data_ptr(), run.v.data_ptr(), run.g.data_ptr()))
    x, v, g = run.x, run.v, run.g

    out = {
        "metric": "replica-steps/sec + achieved HBM GB/s, gossip step, ResNet-50-size d, k=32" if cfg.name == "gossip_r50"
                  else "replica-steps/sec, %s step" % cfg.rule,
        "value": value, "unit": "replica-steps/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: k=%d replicas, d=%d fp32 (%s), rule=%s, fresh Philox peer permutation "
                               "per step, x/v/g resident in HBM"
                               % (cfg.name, k, d, "blocks of %d columns, k x %d elements per matrix" % (run.block_columns, ld)
                                  if run.block_columns else "row-major, row stride %d" % ld, cfg.rule),
                   "k": k, "d": d, "ld": ld, "block_columns": run.block_columns, "rule": cfg.rule, "lr": cfg.lr, "momentum": cfg.momentum,
                   "beta": cfg.beta, "sigma": cfg.sigma, "layout": cfg.layout or "flat"},
        "roofline": {"bound": "hbm", "kernel": kernel_of(cfg.rule, run.block_columns), "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, **traffic_of(cfg.name),
                     "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": kern_s * 1e3,
                     "fresh_allocations": {"n": len(fracs), "steps_each": [K] + [n_rep] * (len(fracs) - 1),
                                           "frac_median": statistics.median(fracs), "frac_min": min(fracs),
                                           "frac_max": max(fracs), "frac_each": fracs}},
    }

    # ---- context: generator, full simulated iteration, other forms, other configurations -----------
    if not args.no_extras:
        n2 = min(100, max(10, K // 4))
        t_next = Wm + K
        extras = {}
        # what this machine's memory delivers to a plain device-to-device copy of the same matrices (read 4 B, write 4 B
        # per element), as context for every fraction here; g is regenerated by the next gen_grad
        scratch = torch.empty_like(g)
        copy_gbs = 8.0 * k * ld / run.kernel_seconds(lambda t: scratch.copy_(g), 10) / 1e9
        extras["plain_copy_GBps"] = copy_gbs
        del scratch
        torch.cuda.empty_cache()

        # the generator's arithmetic alone (no memory traffic): the ALU side of the generator kernels' roofline
        wgs, iters = 2048, 512
        probe_out = torch.empty(wgs * 256, dtype=torch.float32, device="cuda")
        ctx.noise_alu_probe(wgs, 8, probe_out)
        s_alu = run.kernel_seconds(lambda t: ctx.noise_alu_probe(wgs, iters, probe_out), 3)
        s_per_quad = s_alu / (wgs * 256.0 * iters)                   # seconds per Philox block + 4 noise values, whole chip
        quads = k * ((d + 3) // 4)
        alu_ms = quads * s_per_quad * 1e3
        extras["generator_alu"] = {
            "what": "Philox4x32-10 block + Box-Muller for 4 values, registers only (gsgd_noise_alu_probe)",
            "blocks_per_s": 1.0 / s_per_quad,
            "simd_cycles_per_wavefront_block_at_2.4GHz": s_per_quad * 64 * SIMDS * PEAK_CLOCK_HZ,
            "alu_only_ms_for_k_x_d": alu_ms,
        }
        del probe_out

        def roof(ms, bpe, with_generator):
            """Measured time of a kernel beside its two floors: HBM-only (algorithmic bytes at the 8 TB/s peak and at
            this box's plain-copy rate) and, for the kernels that draw noise, ALU-only (the probe above)."""
            nbytes = bpe * k * d
            r = {"kernel_ms": ms, "algorithmic_GBps": nbytes / (ms * 1e-3) / 1e9,
                 "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                 "hbm_only_ms_at_peak": nbytes / (HBM_PEAK_GBS * 1e9) * 1e3,
                 "hbm_only_ms_at_plain_copy_rate": nbytes / (copy_gbs * 1e9) * 1e3}
            if with_generator:
                r["alu_only_ms"] = alu_ms
                r["bound"] = "alu" if alu_ms > r["hbm_only_ms_at_plain_copy_rate"] else "hbm"
            else:
                r["bound"] = "hbm"
            return r

        n3 = max(5, n2 // 3)                           # per timed run of the kernels below; three runs each, median
        s_gen = run.kernel_seconds(lambda t: ctx.gen_grad(x, h, xstar, g, t), n3, t_next)
        extras["gen_grad"] = roof(s_gen * 1e3, 8.0 + 8.0 / k, True)
        extras["gen_grad"].update(traffic_of("gen_grad@" + cfg.name))

        def full(t):
            ctx.gen_grad(x, h, xstar, g, t)
            run.step(t)
        w_full, _ = run.timed(full, n2, t_next + n2)
        extras["full_iteration_ms"] = w_full / n2 * 1e3
        extras["full_iteration_replica_steps_per_s"] = k * n2 / w_full
        if cfg.rule == "gossip" and not args.no_fused:
            def fused(t):
                ctx.step_gossip_fused(x, v, h, xstar, gsgd.make_perm(cfg.seed, t, k), t, cfg.beta)
            for t in range(3):
                fused(t_next + 2 * n2 + t)
            s_fu = run.kernel_seconds(fused, n3, t_next + 2 * n2 + 3)
            extras["fused_iteration"] = roof(s_fu * 1e3, 16.0 + 8.0 / k, True)
            extras["fused_iteration"]["replica_steps_per_s"] = k / s_fu
            extras["fused_iteration"].update(traffic_of("fused@" + cfg.name))
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
                s_f = run.kernel_seconds(fn, n3, 1000)
                extras[name + "_ms"] = s_f * 1e3
                extras[name + "_frac_of_hbm_peak"] = 20.0 * k * d / s_f / 1e9 / HBM_PEAK_GBS
        # the diagnostics (not part of a step): one read of x, 4 B per replica-element
        if d <= gsgd.STATS_STATIC_MAX_D:
            stats_out = torch.empty(4, dtype=torch.float64, device="cuda")
            s_st = run.kernel_seconds(lambda t: gsgd.stats_static(k, d, ld, x, xstar, stats_out,
                                                                  block_columns=run.block_columns), n3)
            extras["stats"] = roof(s_st * 1e3, 4.0 + 4.0 / k, False)
        out["extras"] = extras
        log("extras:", json.dumps(extras))

    blocked = run.block_columns
    run.close()
    del x, v, g, run
    torch.cuda.empty_cache()

    if not args.no_extras and blocked:
        # the same step on row-major matrices (row stride rounded up to 1024), for comparison
        rm = Run(gsgd, W, cfg, args.launch_width, 0, 0)
        for t in range(5):
            rm.step(t)
        s_rm = rm.kernel_seconds(rm.step, n3, 5) / rm.launches_per_step()
        cmp_rm = {"ld": rm.ld, "kernel_ms": s_rm * 1e3, "frac_of_hbm_peak": alg_bytes / s_rm / 1e9 / HBM_PEAK_GBS}
        out["extras"]["row_major_layout"] = cmp_rm
        log("row-major layout:", json.dumps(cmp_rm))
        rm.close()
        del rm
        torch.cuda.empty_cache()

    if not args.no_extras and not args.no_legs and cfg.name == "gossip_r50":
        # the other benchmark configurations (and the gossip step at ResNet-18 size), each a short leg of its own
        legs = {}
        for name in ("tiny", "allreduce_r18", "gossip_r18", "easgd_r50", "seg_gossip_r50_k128"):
            # the 39 GB configuration is the one whose rate depends most on where its arrays land: three placements
            legs[name] = short_leg(gsgd, W, name, fresh_allocations=2 if name == "seg_gossip_r50_k128" else 0)
            log("leg %s: %s" % (name, json.dumps(legs[name])))
        out["extras"]["other_configs"] = legs

    if not args.no_extras and not args.no_legs and cfg.name == "gossip_r50":
        # Section 4.3's observation on the quadratic: gossip's consensus floor moves with the step size.  The
        # generator-fused gossip step at ResNet-18 size with the experiments' local step (Nesterov 0.9, weight decay
        # 1e-4), step size 0.1 annealed by 0.1 twice; per stage the consensus distance per parameter and replica
        # beside the second-moment prediction (paper_1611_04581_amd.theory).
        from paper_1611_04581_amd import theory
        acfg = W.CONFIGS["paper_setup_r18"]
        arun = Run(gsgd, W, acfg)
        arun.ctx.set_local_step(1e-4, True)
        hh = arun.h[:acfg.d].cpu().numpy()
        stages, t, rows = (0.1, 0.01, 0.001), 0, []
        for lr in stages:
            arun.ctx.set_lr(lr)
            for s in range(150):
                arun.ctx.step_gossip_fused(arun.x, arun.v, arun.h, arun.xstar, gsgd.make_perm(acfg.seed, t, acfg.k), t, 0.5)
                t += 1
            cons = arun.ctx.stats(arun.x, arun.xstar)[0]
            pred = acfg.k * float(theory.gossip_consensus_floor(hh, lr, acfg.momentum, acfg.sigma, acfg.k, 0.5, 1e-4, True).sum())
            rows.append({"lr": lr, "consensus_distance": cons, "predicted": pred,
                         "rms_deviation_per_parameter": (cons / (acfg.k * acfg.d)) ** 0.5})
        out["extras"]["annealing_gossip_r18_k16"] = rows
        log("annealing:", json.dumps(rows))
        arun.close()
        del arun

    if not args.no_extras and not args.no_legs and cfg.name == "gossip_r50":
        # short vectors: the k-way sums (LDS-staged block sums) and the gossip step (two sweeps) with the rows split
        # over the wavefronts of a workgroup, against one thread per four columns walking all k rows
        rows = {}
        for (ks, ds) in ((128, 16384), (128, 65536), (32, 65536)):
            scfg = W.Config("short", "allreduce", ks, ds, 0)
            srun = Run(gsgd, W, scfg)
            cell = {}
            for label, mode in (("serial_us", gsgd.ROW_SPLIT_OFF), ("row_split_us", gsgd.ROW_SPLIT_ON)):
                srun.ctx.set_row_split(mode)
                for t in range(5):
                    srun.step(t)
                cell["allreduce_" + label] = srun.kernel_seconds(srun.step, 50) * 1e6
            srun.cfg = W.Config("short", "easgd", ks, ds, 0, alpha_e=0.9 / ks)
            for label, mode in (("serial_us", gsgd.ROW_SPLIT_OFF), ("row_split_us", gsgd.ROW_SPLIT_ON)):
                srun.ctx.set_row_split(mode)
                for t in range(5):
                    srun.step(t)
                cell["easgd_" + label] = srun.kernel_seconds(srun.step, 50) * 1e6
            srun.cfg = W.Config("short", "gossip", ks, ds, 0)
            for label, form in (("walk_us", gsgd.GOSSIP_WALK), ("split_sweeps_us", gsgd.GOSSIP_SWEEP_SPLIT)):
                srun.ctx.set_gossip_form(form)
                for t in range(5):
                    srun.step(t)
                cell["gossip_" + label] = srun.kernel_seconds(srun.step, 50) * 1e6
            rows["k=%d,d=%d" % (ks, ds)] = cell
            srun.close()
        out["extras"]["short_vectors_step_us"] = rows
        log("short vectors:", json.dumps(rows))

    # ---- CPU baseline: the oracle, as it stands, on a bounded sample ---------------------
    if args.cpu_seconds > 0:
        from oracle import oracle
        ds = min(d, 1 << 20)                       # first 2^20 columns of every replica row
        inp = W.make_inputs(k, ds, seed=5)
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
            elif cfg.rule == "local":
                oracle.step_gossip(inp.x, inp.v, inp.g, lrc, cfg.momentum, 0.0, list(range(k)))
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

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark of the fused RPS round on one MI355X.

A "step" is one pass of the whole hot path over the workload: mask generation + fused local
SGD step (in-register synthetic Gaussian gradient) + Reduce-Scatter average + All-Gather
write-back, for all n workers and all N parameters, in place in HBM.

The state is held in the library's tile-major layout by default (row-major with --layout
row-major; the other layout is measured as well and reported under "other_layout").

Order of a measurement: an untimed settling phase of its own (windows of ten rounds are launched
until two consecutive windows agree within 1 % in their mean kernel duration: the first launches
after start-up run at ramping clocks), then the --warmup rounds, then the timed region of exactly
--steps rounds (wall clock between two device synchronisations: `value`, `ms_per_step`), then the
same number of rounds with
every kernel bracketed by HIP events on the library's own stream (`roofline`).

Prints ONE JSON line: worker-params averaged per second (n*N per round), the HBM roofline of
the round kernel (algorithmic bytes = 2*sizeof(dtype) per worker-param, i.e. one read and one
write of the state -- 3 with a gradient buffer -- divided by the kernel's mean duration), the same
fraction from the timed region, a measured device-copy ceiling on arrays of the state's size, and
the CPU oracle timed on the host cores on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X published HBM3E bandwidth

# HBM bytes per launch of the round kernel from rocprofv3 counters (FETCH_SIZE and WRITE_SIZE,
# each scaled by what the same counter reads for a plain 1 GiB device copy).  Counters cannot be
# read from inside this process, so the measured value is recorded here per workload and layout,
# with the profile it comes from; workloads without a counter run report null.
MEASURED_TRAFFIC = {
    ("resnet50_n32", "tiled"): (6.5539e9, "profiles/round_kernel_resnet50_n32_hbm_traffic.md"),
    ("resnet50_n32", "row-major"): (6.5540e9, "profiles/round_kernel_resnet50_n32_hbm_traffic.md"),
    ("bert_n64_bf16", "tiled"): (2.81612e10, "profiles/round_kernel_bert_n64_bf16_hbm_traffic.md"),
}


def cpu_baseline(cfg, off, budget_cols):
    """The oracle as it stands on the host cores: `budget_cols` columns of every block's start,
    all n workers, one round."""
    import numpy as np
    from oracle import rps_oracle as oracle
    threads = oracle.max_threads()
    per_block = max(8, budget_cols // cfg.n)
    cols = np.concatenate([np.arange(off[j], min(off[j] + per_block, off[j + 1])) for j in range(cfg.n)]).astype(np.int64)
    m = cols.size
    if cfg.dtype == "bf16":
        X = np.zeros((cfg.n, m), dtype=np.uint16)
    else:
        X = np.zeros((cfg.n, m), dtype=np.float32)
    G = None if cfg.gradient == "synthetic" else np.zeros_like(X)     # caller-supplied gradient buffer

    def timed(nthreads, budget_s):
        t0 = time.perf_counter()
        reps = 0
        while True:
            reps += 1
            oracle.round_(X, G, off, p=cfg.p, gamma=cfg.gamma, seed=cfg.seed, step=reps, sigma=cfg.sigma,
                          weight_decay=cfg.weight_decay, cols=cols, threads=nthreads)
            dt = time.perf_counter() - t0
            if dt > budget_s:
                return reps, dt

    timed(threads, 0.0)                                               # warm-up
    reps, dt = timed(threads, 10.0)
    reps1, dt1 = timed(1, 3.0)
    return {"value": cfg.n * m * reps / dt, "unit": "worker-params/s", "cores": threads, "kind": "oracle",
            "single_thread_value": cfg.n * m * reps1 / dt1,
            "sample": f"{reps} rounds over {m} columns ({per_block} per block) x {cfg.n} workers of the same workload, "
                      f"{dt:.1f} s on {threads} threads (+ {reps1} rounds, {dt1:.1f} s, on one)"}


def settle(ctx, launch, step, most=300):
    """Untimed: launch windows of ten rounds until the mean kernel duration of a window agrees with
    that of the window before it within 1 % (2 % for kernels shorter than 0.3 ms, whose
    launch-to-launch jitter is larger; at most `most` launches): the clock ramp after start-up is over.
    Returns (next step, launches used, whether they settled)."""
    used = 0
    before = None
    while used < most:
        ctx.set_profiling(True)
        for _ in range(10):
            launch(step); step += 1
        mean = float(ctx.get_kernel_times().mean())
        ctx.set_profiling(False)
        used += 10
        band = 0.01 if mean >= 0.3 else 0.02
        if before is not None and abs(mean - before) <= band * mean:
            return step, used, True
        before = mean
    return step, used, False


def other_paths(ctx, cfg, X, G, step, torch, rps, tiled, launches=30):
    """Kernel time (HIP events on the launch stream) of the other entry points on the same state:
    each against the bytes it has to move -- per worker-param, in units of the element size:
    local step 2 (3 with a gradient buffer), averaging alone 2 - p(1 - 1/n) (rows whose reply is
    lost are not written), fused round on a gradient buffer 3, gradient averaging 3, consensus 1
    (one read; its time includes the small final reduction), layout conversion 2."""
    elem = 2 if cfg.dtype == "bf16" else 4
    wp = cfg.n * cfg.N
    if G is not None:
        Gb = G
    else:
        Gb = torch.empty_like(X) if tiled else ctx.empty_state()
        Gb.normal_(0.0, 1e-3)
    lost = cfg.p * (1.0 - 1.0 / cfg.n)
    scratch = {}

    def convert(t):
        if tiled:
            scratch["o"] = ctx.from_tiled(X)
        else:
            scratch["o"] = ctx.to_tiled(X)

    cases = (("local_step, in-register gradient", lambda t: ctx.local_step(X, None, t), 2.0),
             ("local_step, gradient buffer", lambda t: ctx.local_step(X, Gb, t), 3.0),
             ("lossy_average alone", lambda t: ctx.lossy_average(X, t), 2.0 - lost),
             ("round, gradient buffer", lambda t: ctx.round(X, Gb, t), 3.0),
             ("round_gradient_averaging", lambda t: ctx.round_gradient_averaging(X, Gb, t), 3.0),
             ("consensus", lambda t: ctx.consensus(X), 1.0),
             ("convert_layout (to the other layout)", convert, 2.0))
    res = {}
    for name, fn, units in cases:
        for t in range(5):
            fn(step + t)
        ctx.set_profiling(True)
        for t in range(launches):
            fn(step + t)
        ms = ctx.get_kernel_times()
        ctx.set_profiling(False)
        mean = float(ms.mean())
        gbs = units * elem * wp / (mean * 1e-3) / 1e9
        res[name] = {"kernel_ms": mean, "kernel_ms_min": float(ms.min()), "bytes_per_worker_param": units * elem,
                     "achieved": gbs, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS}
        scratch.clear()
    return res


def copy_ceiling(X, torch, reps=10):
    """The simplest streaming jobs on the same buffer, timed with events on the current stream, as a
    measured ceiling next to the published peak: an in-place pass (torch's elementwise x *= 1: every
    element read once and written once, like the round) and a plain copy into a second array."""
    flat = torch.empty(0, dtype=X.dtype, device="cuda").set_(X.untyped_storage())
    nbytes = flat.numel() * flat.element_size()

    def timed(fn):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / reps

    ms_inplace = timed(lambda: flat.mul_(1.0))
    other = torch.empty_like(flat)
    ms_copy = timed(lambda: other.copy_(flat))
    del other
    torch.cuda.empty_cache()
    gbs = 2.0 * nbytes / (ms_inplace * 1e-3) / 1e9
    gbs_copy = 2.0 * nbytes / (ms_copy * 1e-3) / 1e9
    return {"achieved": gbs, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "ms": ms_inplace, "bytes_each_way": nbytes,
            "what": "torch in-place elementwise pass (x *= 1) over the state buffer",
            "copy_to_second_array": {"achieved": gbs_copy, "frac": gbs_copy / HBM_PEAK_GBS, "ms": ms_copy}}


def measure(cfg, off, layout, args, torch, rps, want_other_paths, want_copy):
    """Settling, warm-up, the timed region, then the event-bracketed pass of the round kernel, for one storage layout."""
    tiled = layout == "tiled"
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    elem = 2 if cfg.dtype == "bf16" else 4
    ctx = rps.RpsContext(cfg.n, cfg.N, cfg.p, cfg.gamma, cfg.seed,
                         rps.RPS_DTYPE_BF16 if cfg.dtype == "bf16" else rps.RPS_DTYPE_F32, block_offsets=off,
                         flags=rps.RPS_FLAG_LAYOUT_TILED if tiled else 0)
    ctx.set_synthetic_grad(cfg.sigma, cfg.weight_decay)
    pitch = None
    if tiled:
        T = rps.RPS_TILE_BYTES // elem
        X = torch.zeros(((cfg.N + T - 1) // T, cfg.n, T), device="cuda", dtype=tdt)   # Alg. 1: identical start, X_1 = 0
    else:
        # rows a little further apart than N where the row size would otherwise be a multiple of 32 KB
        # (all n rows of a tile on one memory channel); the padding is never touched
        if (cfg.N * elem) % 32768 == 0:
            pitch = rps.rps_recommended_row_pitch(cfg.N, ctx.dtype)
            ctx.set_row_pitch(pitch)
        X = ctx.empty_state(fill=0.0)
    # workloads whose gradient comes from a model (least squares, MLP): the library's part of a
    # step is the fused round on a caller-supplied gradient buffer; a fixed seeded buffer stands
    # in for it here (3 arrays of traffic instead of 2)
    G = None
    if cfg.gradient != "synthetic":
        gen = torch.Generator(device="cuda"); gen.manual_seed(1)
        G = torch.zeros_like(X) if tiled else ctx.empty_state(fill=0.0)
        G.copy_((torch.randn(tuple(G.shape), device="cuda", generator=gen) * 1e-3).to(tdt))

    def launch(t):
        ctx.round(X, G, t)

    step, settle_launches, settled = settle(ctx, launch, 0)
    for _ in range(args.warmup):
        launch(step); step += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        launch(step); step += 1
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    # the round kernel alone, bracketed by HIP events on the stream it is launched on
    ctx.set_profiling(True)
    for _ in range(args.steps):
        launch(step); step += 1
    times = ctx.get_kernel_times(max(4096, args.steps))
    ctx.set_profiling(False)
    assert len(times) == min(args.steps, 4096)
    kernel_ms = float(times.mean())

    alg_bytes = (3.0 if G is not None else 2.0) * elem * cfg.n * cfg.N   # read x (and g) once, write x' once
    res = {"value": cfg.n * cfg.N * args.steps / dt, "ms_per_step": dt / args.steps * 1e3, "kernel_ms": kernel_ms,
           "kernel_ms_median": float(sorted(times)[len(times) // 2]), "kernel_ms_min": float(times.min()),
           "alg_bytes": alg_bytes, "achieved": alg_bytes / (kernel_ms * 1e-3) / 1e9, "has_G": G is not None,
           "settle_launches": settle_launches, "settled": settled, "row_pitch": pitch}
    if want_other_paths:
        res["other_paths"] = other_paths(ctx, cfg, X, G, step, torch, rps, tiled)
    if want_copy:
        res["copy_ceiling"] = copy_ceiling(X, torch)
    ctx.destroy()
    del X, G
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", default=None, help="workload name (default: the headline config)")
    ap.add_argument("--layout", choices=("tiled", "row-major"), default=None,
                    help="storage layout of X and G (default: tiled; the other layout is measured too and "
                         "reported under other_layout)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--other-paths", action="store_true",
                    help="also time the unfused entry points, the gradient-buffer round, gradient averaging, consensus "
                         "and the layout conversion on the same workload (needs further arrays of the state's size) "
                         "and report each against its own algorithmic bytes, for both layouts")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies (a kernel of known traffic) so that one "
                         "rocprofv3 --pmc run holds both the round kernel and the reference for its counters; "
                         "measures the chosen layout only")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the n workers are simulated in one [n, N] tensor); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads
    from paper_1810_07766_amd import rps

    cfg = workloads.CONFIGS[args.config or workloads.HEADLINE]
    off = workloads.config_offsets(cfg)
    torch.cuda.set_device(0)
    layout = args.layout or "tiled"
    other = "row-major" if layout == "tiled" else "tiled"

    m = measure(cfg, off, layout, args, torch, rps, args.other_paths, want_copy=not args.pmc_calibration)
    kernel = "round_kernel_narrow" if layout == "tiled" else "round_kernel"
    traffic, traffic_source = MEASURED_TRAFFIC.get((cfg.name, layout), (None, "no rocprofv3 counter run for this workload and layout"))
    out = {
        "metric": "worker-params averaged/sec (n*N per round)",
        "value": m["value"],
        "unit": "worker-params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": m["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if cfg.dtype == "f32" else "bf16-storage/f32-math",
        "data": "synthetic",
        "config": {"workload": cfg.name, "n": cfg.n, "N": cfg.N, "p": cfg.p, "gamma": cfg.gamma,
                   "gradient": (f"in-register N(0,{cfg.sigma ** 2:.3g}) + {cfg.weight_decay}*x" if not m["has_G"]
                                else "caller-supplied buffer G[n,N] (seeded stand-in)"),
                   "blocks": "unequal" if cfg.unequal_blocks else "equal",
                   "layout": ("tile-major [N/T][n][T], T = 128 bytes" if layout == "tiled" else "row-major [n][N]"),
                   "row_pitch": m["row_pitch"],
                   "settling": f"{m['settle_launches']} untimed launches before the warm-up"
                               + ("" if m["settled"] else " (window means had not settled within 1 %)")},
        "roofline": {"bound": "hbm", "achieved": m["achieved"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": m["achieved"] / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": kernel, "kernel_ms": m["kernel_ms"], "kernel_ms_median": m["kernel_ms_median"],
                     "kernel_ms_min": m["kernel_ms_min"], "algorithmic_bytes": m["alg_bytes"],
                     "frac_timed_region": m["alg_bytes"] / (m["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }
    if "copy_ceiling" in m:
        out["copy_ceiling"] = m["copy_ceiling"]
    if "other_paths" in m:
        out["other_paths"] = m["other_paths"]
    if not args.pmc_calibration:
        o = measure(cfg, off, other, args, torch, rps, args.other_paths, want_copy=False)
        out["other_layout"] = {"layout": other, "value": o["value"], "ms_per_step": o["ms_per_step"],
                               "kernel_ms": o["kernel_ms"], "kernel_ms_median": o["kernel_ms_median"],
                               "kernel_ms_min": o["kernel_ms_min"], "achieved": o["achieved"], "unit": "GB/s",
                               "frac": o["achieved"] / HBM_PEAK_GBS, "row_pitch": o["row_pitch"],
                               "frac_timed_region": o["alg_bytes"] / (o["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBS}
        if "other_paths" in o:
            out["other_layout"]["other_paths"] = o["other_paths"]
    if args.pmc_calibration:
        src = torch.ones(1 << 28, device="cuda")          # 1 GiB of fp32
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, off, budget_cols=1 << 18)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

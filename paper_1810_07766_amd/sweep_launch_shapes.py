"""Sweep of the round kernels' launch shapes over worker counts (measurement utility; needs an MI355X).

For every (layout, dtype, n) at equal state size it times the three round entry points -- fused round
with the in-register gradient, averaging alone, fused round on a gradient buffer -- and the gradient
averaging, first with the library's built-in launch shape and then with every shape of a small grid
set through rps_set_launch_tuning (rows per load chunk, wavefronts per workgroup, occupancy cap, steps
per wavefront), and prints one markdown table row per case: the built-in shape's fraction of the HBM
peak, the best shape of the grid and its fraction.  The built-in rules (default_tuning / tiled_tuning /
gradavg_cap in csrc/rps_api.hip) were drawn from such sweeps; results never depend on the shape.

    python -m paper_1810_07766_amd.sweep_launch_shapes [--layout tiled|row-major|both]
        [--workers 2,4,8,...] [--state-gb 1.2] [--launches 30]
"""
import argparse
import sys

PEAK_GBS = 8000.0


def _grid(what, n, tiled):
    rows = (2, 4) if (n > 32 or not tiled) else (4,)
    if what == "gradient averaging":
        return [(4, 1, c, 0) for c in (0, 6, 8, 10, 12, 16, 24)]
    if tiled:
        if what == "round, in-register gradient":
            return [(r, w, 0, t) for r in rows for w in (4, 8, 12, 14) for t in (1, 2)]
        return ([(r, 1, c, 0) for r in rows for c in (8, 10, 12, 14, 16, 20)]
                + [(r, w, c, 0) for r in rows for w in (8, 12, 14) for c in (0, 16)])
    if what == "round, in-register gradient":
        return [(r, w, c, 1) for r in rows for w in (2, 4, 8) for c in (0, 12)]
    return [(r, 1, c, 0) for r in rows for c in (4, 5, 6, 8, 12)] + [(r, 4, c, 0) for r in rows for c in (0, 8, 12)]


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--layout", choices=("tiled", "row-major", "both"), default="both")
    ap.add_argument("--workers", default="2,3,4,6,8,12,16,20,24,32,40,48,64")
    ap.add_argument("--state-gb", type=float, default=1.2)
    ap.add_argument("--launches", type=int, default=30)
    args = ap.parse_args(argv)
    import torch
    from . import rps
    if not torch.cuda.is_available():
        sys.exit("sweep_launch_shapes: needs a GPU")
    workers = [int(x) for x in args.workers.split(",")]
    layouts = ("tiled", "row-major") if args.layout == "both" else (args.layout,)
    print("| layout | dtype | n | entry point | built-in shape: frac of 8 TB/s | best of the grid: frac | best shape "
          "(rows per chunk : wavefronts per workgroup : cap : steps per wavefront) |")
    print("|---|---|---|---|---|---|---|")
    for layout in layouts:
        tiled = layout == "tiled"
        for dtype, elem, tdt in ((rps.RPS_DTYPE_F32, 4, torch.float32), (rps.RPS_DTYPE_BF16, 2, torch.bfloat16)):
            T = rps.RPS_TILE_BYTES // elem
            for n in workers:
                N = (int(args.state_gb * 1e9) // elem // n // 1024) * 1024 + (0 if tiled else 1024)
                shape = ((N + T - 1) // T, n, T) if tiled else (n, N)
                X = torch.zeros(shape, device="cuda", dtype=tdt)
                G = torch.zeros(shape, device="cuda", dtype=tdt)
                off = [0] + [((N * (j + 1)) // n // 64) * 64 for j in range(n - 1)] + [N]
                for what, units in (("round, in-register gradient", 2), ("averaging alone", 2),
                                    ("round, gradient buffer", 3), ("gradient averaging", 3)):
                    ctx = rps.RpsContext(n, N, 0.1, 0.1, 0, dtype, flags=rps.RPS_FLAG_LAYOUT_TILED if tiled else 0,
                                         block_offsets=off)
                    ctx.set_synthetic_grad(0.03, 0.0)
                    call = {"round, in-register gradient": lambda t: ctx.round(X, None, t),
                            "averaging alone": lambda t: ctx.lossy_average(X, t),
                            "round, gradient buffer": lambda t: ctx.round(X, G, t),
                            "gradient averaging": lambda t: ctx.round_gradient_averaging(X, G, t)}[what]
                    nbytes = units * elem * n * N

                    def frac():
                        for t in range(12):
                            call(t)
                        ctx.set_profiling(True)
                        for t in range(args.launches):
                            call(100 + t)
                        ms = ctx.get_kernel_times().mean()
                        ctx.set_profiling(False)
                        return nbytes / ms / 1e6 / PEAK_GBS

                    for t in range(30):
                        call(t)
                    builtin = frac()
                    results = {}
                    for rep in range(2):
                        for cand in _grid(what, n, tiled):
                            ctx.set_launch_tuning(*cand)
                            results[cand] = results.get(cand, 0.0) + frac() / 2
                    best = max(results, key=results.get)
                    print(f"| {layout} | {'fp32' if elem == 4 else 'bf16'} | {n} | {what} | {builtin:.3f} | "
                          f"{results[best]:.3f} | {best[0]}:{best[1]}:{best[2]}:{best[3]} |", flush=True)
                    ctx.destroy()
                del X, G


if __name__ == "__main__":
    main()

"""Benchmark of the CSER update on one MI355X.

A "step" is one iteration of Algorithm 3 through the C ABI: block selection, the fused local step + partial
synchronisation + residual bookkeeping, and the error reset on the iterations where t mod H = 0 -- the whole
hot path.  The workload is the large-CNN-sized configuration the headline metric is quoted on
(d = 25,557,032, W = 8, block 1024, R_step 256, R_reset 16, H 32); states and two rotating gradient
buffers are resident in HBM before the timed region, gradients are synthetic N(0, 1e-3).

Prints one JSON line: whole-job param-elements/s, the HBM roofline of the fused-step kernel
(algorithmic bytes per launch / HIP-event duration per launch, measured in the same timed region),
and the CPU oracle timed on a bounded sample of the same workload.

The timed iterations always contain at least one redraw of the block-mask window and, when H > 0, at least
one error reset: with few steps the iteration counter is moved (cser_set_step) so that they do.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, vendor figure
TUNING_KEYS = {"kernel": 0, "nontemporal": 1, "fuse_reset": 2, "tile_waves_per_cu": 3, "shared_groups_per_cu": 4}
KERNEL_NAMES = {"launches_tile": "cser_step_tile_kernel", "launches_shared": "cser_step_shared_kernel",
                "launches_general": "cser_step_general_kernel",
                "launches_split": "cser_step_tile_kernel+cser_step_shared_kernel"}


def step_bytes(wl, d_sel, with_error=True, with_momentum=True):
    """Algorithmic bytes of one fused-step launch: per element and worker read g, m, x, e and write
    m, x, e (28 B); on the d_sel columns of chosen blocks e is neither read nor written (20 B)."""
    per = 4 * (1 + (2 if with_momentum else 0) + 2 + (2 if with_error else 0))
    sel = per - (8 if with_error else 0)
    return wl.W * (per * (wl.d - d_sel) + sel * d_sel)


def reset_bytes(wl, d_sel, with_error=True):
    """Algorithmic bytes of one error reset: read e, x and write x, e on the chosen columns (implementation II: x only)."""
    return (16 if with_error else 8) * wl.W * d_sel


def chosen_columns(wl, mask):
    """Number of columns in the blocks a mask selects (the last block may be short)."""
    n = int(mask.sum()) * wl.block
    if mask[-1]:
        n -= wl.B * wl.block - wl.d
    return n


def read_traffic(workload):
    """HBM bytes per fused-step launch from the committed counter summary (a constant of an earlier counter run
    of this same command, not a counter of this run), or (None, None)."""
    rel = os.path.join("profiles", f"fused_step_{workload}_hbm_traffic.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
    return (float(m.group(1)), rel) if m else (None, None)


def cpu_baseline(wl, variant_e=True, variant_m=True):
    """The oracle as it stands, one host thread, on a slice of the workload's blocks."""
    import numpy as np
    from oracle import reference as R
    steps = max(wl.H, 1)                           # one full reset period, so the reset is included
    steps = min(steps, 32)
    nb = max(1, wl.B // 4)
    ncols = min(wl.d, nb * wl.block)
    rng = np.random.default_rng(wl.seed)
    x0 = (rng.standard_normal(ncols) * np.sqrt(wl.x_var)).astype(np.float32)
    g = [(rng.standard_normal((wl.W, ncols)) * np.sqrt(wl.g_var)).astype(np.float32) for _ in range(2)]
    o = R.OracleCSER(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum if variant_m else 0.0,
                     wl.seed, x0, dtype=np.float32, b0=0, b1=nb, with_error=variant_e)
    t0 = time.perf_counter()
    for t in range(steps):
        o.step(g[t & 1])
    dt = time.perf_counter() - t0
    return {"value": ncols * steps / dt, "unit": "param-elements/s", "cores": 1, "kind": "oracle",
            "sample": f"blocks [0, {nb}) of {wl.B} ({ncols} of {wl.d} columns, all {wl.W} workers), {steps} steps "
                      f"incl. {steps // wl.H if wl.H else 0} error reset(s), block choice over all blocks; {dt:.1f} s on one host thread",
            "host_cpus": os.cpu_count()}


def place_timed_region(B, ctx, wl, steps):
    """Move the iteration counter, if need be, so that the next `steps` iterations hold a redraw of the mask
    window and (H > 0) an error reset.  Returns the first timed iteration."""
    t_now = B.cser_get_step(ctx)
    first, last = t_now + 1, t_now + steps
    has_reset = wl.H > 0 and (last // wl.H) * wl.H >= first
    if steps >= 64 and (has_reset or wl.H == 0):
        return first                                  # long enough to hold both anyway (the window is 32 iterations)
    back = (3 * steps) // 4                           # the reset falls three quarters into the region
    period = wl.H if wl.H > 0 else 32
    r = -(-(t_now + 33 + back) // period) * period    # beyond the window drawn so far: the first timed step redraws
    B.cser_set_step(ctx, r - back - 1)
    return r - back


def buffer_pool(wl, dev):
    """One set of state and gradient buffers for a series of runs of the same shape.  The time of a launch depends
    on which physical pages the buffers got (the same code at the same virtual addresses: 0.87 to 0.93 ms between
    fresh allocations, +-0.1 % within one), so a series that is to be compared point by point keeps its buffers."""
    import torch
    return {"shape": (wl.W, wl.ld),
            **{k: torch.zeros(wl.W, wl.ld, device=dev, dtype=torch.float32) for k in ("x", "e", "m", "g1", "g2")}}


def run_workload(wl, steps, warmup, tune=(), with_copy=True, variant_e=True, variant_m=True, second_pass=True, pool=None):
    """Time `steps` iterations on one workload; returns the fields of the JSON line."""
    import torch
    from paper_2007_13221_amd import binding as B
    from paper_2007_13221_amd import inputs as I

    dev = torch.device("cuda:0")
    momentum = wl.momentum if variant_m else 0.0
    cfg = B.make_config(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, momentum, wl.seed, ld=wl.ld)
    if pool is not None:
        assert pool["shape"] == (wl.W, wl.ld)
        pool["x"].zero_()
        pool["x"][:, :wl.d] = I.initial_model_row(wl, dev)
        opt = B.CSER(cfg, pool["x"], with_error=variant_e, with_momentum=variant_m, e=pool["e"], m=pool["m"])
        grads = [I.gradient(wl, t, dev, out=pool[f"g{t}"]) for t in (1, 2)]
    else:
        opt = B.CSER(cfg, I.initial_model(wl, dev), with_error=variant_e, with_momentum=variant_m)
        grads = [I.gradient(wl, t, dev) for t in (1, 2)]   # generated outside every timed region
    for item in tune:
        key, value = item.split("=")
        B.cser_set_tuning(opt.ctx, TUNING_KEYS[key], int(value))
    stream = torch.cuda.current_stream().cuda_stream
    glist = B.gradient_list([grads[t & 1] for t in range(steps)])
    torch.cuda.synchronize()

    for t in range(warmup):
        opt.step(grads[t & 1])
    torch.cuda.synchronize()

    # ---- the timed region: `steps` iterations, every fused-step and reset launch bracketed by HIP events
    t_first = place_timed_region(B, opt.ctx, wl, steps)
    before = B.cser_measure_counters(opt.ctx)
    B.cser_profile_enable(opt.ctx, True)
    B.cser_profile_clear(opt.ctx)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    B.cser_step_many(opt.ctx, glist, stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    step_ms, step_launches = B.cser_profile_read(opt.ctx, 0)
    reset_ms, reset_launches = B.cser_profile_read(opt.ctx, 1)
    B.cser_profile_enable(opt.ctx, False)
    after = B.cser_measure_counters(opt.ctx)
    delta = {k: after[k] - before[k] for k in after}

    # ---- the same iterations once more without the events (they cost host and GPU time that matters at small d)
    plain = None
    if second_pass:
        B.cser_set_step(opt.ctx, t_first - 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        B.cser_step_many(opt.ctx, glist, stream)
        torch.cuda.synchronize()
        plain = time.perf_counter() - t0

    # algorithmic bytes of the timed launches (block lists recomputed by the GPU selector afterwards)
    total_step_bytes = 0
    total_reset_bytes = 0
    synced_columns = 0
    for t in range(t_first, t_first + steps):
        _, mask = B.cser_select_blocks(opt.ctx, 0, t)
        cols = chosen_columns(wl, mask)
        synced_columns += cols
        total_step_bytes += step_bytes(wl, cols, variant_e, variant_m)
        if wl.H and t % wl.H == 0:
            _, rmask = B.cser_select_blocks(opt.ctx, 1, t)
            rcols = chosen_columns(wl, rmask)
            synced_columns += rcols
            total_reset_bytes += reset_bytes(wl, rcols, variant_e)
    # The fused-step kernel is credited with the step's bytes only, also on iterations where it carries the error
    # reset out as well (x and e of those blocks are in registers already): its figure is never overstated.
    bytes_per_launch = total_step_bytes / steps
    kernel_ms = step_ms / max(step_launches, 1)
    achieved = bytes_per_launch / (kernel_ms * 1e-3) / 1e9

    copy_gbps = None
    if with_copy:
        # a plain 128-bit copy kernel over buffers of the same size, for comparison and counter calibration
        n_copy = wl.W * wl.ld * 4
        src, dst = opt.x, torch.empty_like(opt.x)
        for _ in range(3):
            B.cser_copy_probe(dst, src, n_copy)
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(20):
            B.cser_copy_probe(dst, src, n_copy)
        ev1.record()
        torch.cuda.synchronize()
        copy_gbps = 2 * n_copy * 20 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
        del dst

    kind = ("implementation I" if variant_e else "implementation II (no e)") + ("" if variant_m else ", no momentum buffer")
    kernels = {KERNEL_NAMES[k]: delta[k] for k in KERNEL_NAMES if delta[k]}
    if wl.W > 16 and delta["launches_split"]:    # beyond 16 workers the general kernel takes the synchronised blocks of a pair
        kernels["cser_step_tile_kernel+cser_step_general_kernel"] = kernels.pop(KERNEL_NAMES["launches_split"])
    traffic, traffic_source = read_traffic(wl.name) if (variant_e and variant_m and not tune) else (None, None)
    whole_bytes = total_step_bytes + total_reset_bytes
    out = {
        "metric": "CSER step param-elements/s and achieved HBM GB/s (% of peak) at d=25.6M, W=8",
        "value": wl.d * steps / elapsed,
        "unit": "param-elements/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": elapsed * 1e3 / steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: d={wl.d}, W={wl.W}, block={wl.block}, R_step={wl.R_step}, "
                               f"R_reset={wl.R_reset}, H={wl.H}, lr={wl.lr}, momentum={momentum}, "
                               f"g~N(0,{wl.g_var}), seed={wl.seed}; steps t={t_first}..{t_first + steps - 1}; {kind}",
                   "resident": "x, e, m [W][ld] fp32 + 2 rotating g buffers", "ld": wl.ld},
        "worker_elements_per_s": wl.W * wl.d * steps / elapsed,
        "whole_path_GBps": whole_bytes / elapsed / 1e9,
        "whole_path_frac_of_peak": whole_bytes / elapsed / 1e9 / HBM_PEAK_GBPS,
        "whole_path_bytes": "algorithmic: fused step 4*W*(7d - 2 d_sel) per iteration plus 16*W*d_sel' per error reset",
        "roofline": {"bound": "hbm", "kernel": max(kernels, key=kernels.get) if kernels else None, "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "bytes_per_launch": bytes_per_launch, "ms_per_launch": kernel_ms, "launches": step_launches,
                     "launches_by_kernel": kernels},
        "selector": {"window_draws_in_timed_region": delta["window_draws"]},
        "resets": {"in_timed_region": delta["resets_fused"] + delta["resets_separate"],
                   "fused_into_step_kernel": delta["resets_fused"],
                   "separate_kernel_launches": reset_launches,
                   "separate_kernel_ms_per_launch": reset_ms / max(reset_launches, 1)},
        "overall_compression_ratio": {"counted": wl.d * steps / synced_columns if synced_columns else None,
                                      "section_5_1_formula": B.cser_overall_ratio(cfg)},
        "without_kernel_events": None if plain is None else {"ms_per_step": plain * 1e3 / steps,
                                                             "value": wl.d * steps / plain},
        "copy_kernel_GBps": copy_gbps,
    }
    opt.close()
    del opt, grads
    if pool is None:
        torch.cuda.empty_cache()
    return out


def run_explicit_resets(wl, reps, tune=(), variant_e=True):
    """Time cser_error_reset (block selection, ordered block list, reset kernel) `reps` times at t = 1, 2, ...: the
    blocks differ from call to call.  States hold random values; nothing is stepped."""
    import torch
    from paper_2007_13221_amd import binding as B
    from paper_2007_13221_amd import inputs as I

    dev = torch.device("cuda:0")
    cfg = B.make_config(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum, wl.seed, ld=wl.ld)
    opt = B.CSER(cfg, I.initial_model(wl, dev), with_error=variant_e)
    for item in tune:
        key, value = item.split("=")
        B.cser_set_tuning(opt.ctx, TUNING_KEYS[key], int(value))
    if variant_e:
        opt.e.normal_(0.0, 0.01)
    torch.cuda.synchronize()
    B.cser_set_step(opt.ctx, 0)
    opt.error_reset()
    torch.cuda.synchronize()
    B.cser_profile_enable(opt.ctx, True)
    B.cser_profile_clear(opt.ctx)
    stream = torch.cuda.current_stream().cuda_stream
    t0 = time.perf_counter()
    for r in range(reps):
        B.cser_set_step(opt.ctx, r + 1)
        B.cser_error_reset(opt.ctx, stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms, n = B.cser_profile_read(opt.ctx, 1)
    total = 0
    for r in range(reps):
        _, mask = B.cser_select_blocks(opt.ctx, 1, r + 1)
        total += reset_bytes(wl, chosen_columns(wl, mask), variant_e)
    per = total / reps
    kernel_ms = ms / max(n, 1)
    gbps = per / (kernel_ms * 1e-3) / 1e9
    out = {"mode": "explicit error resets (cser_error_reset)", "workload": f"{wl.name}: d={wl.d}, W={wl.W}, block={wl.block}, R_reset={wl.R_reset}",
           "resets": reps, "ms_per_call": elapsed * 1e3 / reps,
           "roofline": {"bound": "hbm", "kernel": "cser_reset_shared_kernel" if wl.W <= 16 and wl.block % 4 == 0 else "cser_reset_general_kernel",
                        "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS,
                        "bytes_per_launch": per, "ms_per_launch": kernel_ms, "launches": n},
           "whole_call_GBps": total / elapsed / 1e9}
    opt.close()
    return out


def compact(wl, r):
    return {"workload": wl.name, "R_step": wl.R_step, "R_reset": wl.R_reset, "block": wl.block, "H": wl.H,
            "steps": r["steps"], "ms_per_step": round(r["ms_per_step"], 4),
            "G_param_elements_per_s": round(r["value"] / 1e9, 2),
            "step_kernel_ms": round(r["roofline"]["ms_per_launch"], 4),
            "step_kernel_GBps": round(r["roofline"]["achieved"], 1),
            "step_kernel_frac_of_peak": round(r["roofline"]["frac"], 3),
            "kernels": r["roofline"]["launches_by_kernel"],
            "whole_path_GBps": round(r["whole_path_GBps"], 1),
            "whole_path_frac_of_peak": round(r["whole_path_frac_of_peak"], 3),
            "resets": r["resets"]["in_timed_region"],
            "overall_ratio_counted": round(r["overall_compression_ratio"]["counted"], 2) if r["overall_compression_ratio"]["counted"] else None,
            "overall_ratio_formula": round(r["overall_compression_ratio"]["section_5_1_formula"], 2)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="large_cnn")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--variant", choices=["I", "II", "I-nomomentum", "II-nomomentum"], default="I",
                    help="I: x, e, m (Algorithm 3); II: no residual buffer (Appendix A.4); -nomomentum: beta = 0, no m")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the one headline line: one compact line per point of the 40-point compression "
                         "sweep at the large-CNN size (50 steps each)")
    ap.add_argument("--table4", action="store_true",
                    help="one compact line per CSER row of the paper's Table 4 (compressor pair and reset interval for "
                         "each overall ratio) at the large-CNN size, max(64, 2 H) steps each")
    ap.add_argument("--workers", type=int, default=0, help="override the workload's number of workers W")
    ap.add_argument("--override", action="append", default=[], metavar="FIELD=VALUE",
                    help="override an integer field of the workload (R_step, R_reset, H, block), e.g. R_step=1")
    ap.add_argument("--explicit-resets", type=int, default=0, metavar="N",
                    help="instead of stepping: time N calls of cser_error_reset on the workload")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="cser_set_tuning(key, value) before the run (launch-shape experiments); keys: " + ", ".join(TUNING_KEYS))
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (all W worker states are resident on it and the worker "
                 "average is a reduction over rows, not a collective); --gpus must be 1")

    import torch
    from paper_2007_13221_amd import inputs as I

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    variant_e = not args.variant.startswith("II")
    variant_m = not args.variant.endswith("nomomentum")
    if args.sweep or args.table4:
        points = I.sweep_workloads() if args.sweep else I.table4_workloads()
        pool = buffer_pool(points[0], torch.device("cuda:0"))   # every point has the same W and ld
        for wl in points:
            r = run_workload(wl, wl.steps, 5, args.tune, with_copy=False, variant_e=variant_e, variant_m=variant_m,
                             second_pass=False, pool=pool)
            print(json.dumps(compact(wl, r)), flush=True)
        return
    named = dict(I.WORKLOADS)
    named.update({w.name: w for w in I.sweep_workloads()})
    named.update({w.name: w for w in I.table4_workloads()})
    wl = named[args.workload]
    from dataclasses import replace
    if args.workers:
        wl = replace(wl, W=args.workers, name=f"{wl.name}_W{args.workers}")
    for item in args.override:
        field, value = item.split("=")
        if field not in ("R_step", "R_reset", "H", "block"):
            sys.exit(f"bench.py: cannot override {field}")
        wl = replace(wl, **{field: int(value)}, name=f"{wl.name}_{field}{value}")
    if args.explicit_resets:
        print(json.dumps(run_explicit_resets(wl, args.explicit_resets, args.tune, variant_e)))
        return
    out = run_workload(wl, args.steps, args.warmup, args.tune, variant_e=variant_e, variant_m=variant_m)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, variant_e, variant_m)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

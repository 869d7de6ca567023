#!/usr/bin/env python3
"""Benchmark of the GRAWA distributed update on one MI355X.

A "step" is one complete distributed phase for all K workers resident on the GPU: gradient
norms -> weights -> center -> pull (with the local SGD step fused in where the configuration
says so), i.e. one call of grawa_lgrawa_update / grawa_mgrawa_update[_sgd].  Inputs are
synthetic, seeded, and already in HBM when the timed region starts.

Prints ONE JSON line.  `value` is the update's HBM bandwidth under the minimum-traffic byte
model (bytes every correct implementation must move: gradients read once for the norms,
parameters read once and written once, gradients read a second time when the SGD step is
fused) divided by the measured time per step.  `roofline` is the same kind of figure for the
dominant kernel alone (center+pull), from HIP start/stop events attached to that kernel's
launches while the timed steps are repeated once more (so that `value` carries no event
overhead).  `cpu_baseline` is the float64 CPU reference timed on a bounded sample of the
same workload on this machine's host cores.  The headline workload is the largest of the five
configurations (configuration 3); `roofline_by_config` and `cpu_baseline_by_config` carry the same
two objects for each of the three configurations the throughput target is stated for (2, 3, 4),
`all_configs` the timing of all five.  `phases` times the calls around the distributed phase
(local steps, Local-GRAWA round, Nesterov step, EASGD / LSGD) on the headline workload.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
HEADLINE_CONFIG = 3            # the largest single-GPU configuration (354 M parameters x 8 workers, 28 GB per update)
TARGET_CONFIGS = (2, 3, 4)     # the configurations the throughput target is stated for
TRAFFIC_FILE = os.path.join("profiles", "traffic.json")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=HEADLINE_CONFIG,
                    help="benchmark configuration 0..4 of the headline figures (default: %d)" % HEADLINE_CONFIG)
    ap.add_argument("--variant", default=None, help="lgrawa | mgrawa (default: the configuration's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="do not also time the other configurations")
    ap.add_argument("--cpu-seconds", type=float, default=10.0,
                    help="target CPU time of the reference sample, per configuration")
    ap.add_argument("--no-phases", action="store_true", help="do not also time the local-phase and Appendix F calls")
    ap.add_argument("--emit-stats", action="store_true",
                    help="time --config/--variant only and print its raw timing record (used by the sweep, which gives "
                         "every configuration a process of its own)")
    ap.add_argument("--only-phases", action="store_true",
                    help="time only the local-phase and Appendix F calls on --config (for kernel profiles)")
    return ap.parse_args()


def pick_variant(w, variant):
    if variant:
        return variant
    return "lgrawa" if "lgrawa" in w.variants else w.variants[0]


def call_update(plan, w, x, g, variant):
    P = w.P
    if variant == "lgrawa":
        if w.fused_sgd:
            plan.lgrawa_update_sgd(x[:, :P], g[:, :P], w.lam, g[:, :P], w.lr)
        else:
            plan.lgrawa_update(x[:, :P], g[:, :P], w.lam)
    else:
        if w.fused_sgd:
            plan.mgrawa_update_sgd(x[:, :P], g[:, :P], w.lam, g[:, :P], w.lr)
        else:
            plan.mgrawa_update(x[:, :P], g[:, :P], w.lam)


def spread(v):
    v = sorted(v)
    if not v:
        return None
    return {"min": v[0], "median": v[len(v) // 2] if len(v) % 2 else 0.5 * (v[len(v) // 2 - 1] + v[len(v) // 2]),
            "mean": sum(v) / len(v), "max": v[-1], "n": len(v)}


def time_config(torch, grawa, W, idx, variant, steps, warmup):
    """Returns (stats dict, x, g, w) with x, g left on the device (x has been updated)."""
    w = W.config(idx)
    variant = pick_variant(w, variant)
    x, g = W.make_inputs(w, device="cuda:0")
    x0 = None
    torch.cuda.synchronize()
    with grawa.Plan(w.K, w.P, w.offsets) as plan:
        info = plan.info()
        for _ in range(warmup):
            call_update(plan, w, x, g, variant)
        # timed region: exactly `steps` updates, bracketed by device synchronisation
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            call_update(plan, w, x, g, variant)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        # the same update recorded once into a HIP graph and replayed `steps` times (what a launch-bound
        # caller would do; reported beside the eager figure, never instead of it)
        graph_ms = None
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                call_update(plan, w, x, g, variant)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                call_update(plan, w, x, g, variant)
            graph.replay()
            torch.cuda.synchronize()
            g0 = time.perf_counter()
            for _ in range(steps):
                graph.replay()
            torch.cuda.synchronize()
            graph_ms = (time.perf_counter() - g0) * 1e3 / steps
            del graph
        except RuntimeError as e:                            # reported, not fatal: the eager figure stands
            print("bench.py: graph replay skipped: %s" % e, file=sys.stderr)
        # the same steps again with start/stop events attached to the two big kernels
        plan.profile(True)
        torch.cuda.synchronize()
        e0 = time.perf_counter()
        for _ in range(steps):
            call_update(plan, w, x, g, variant)
        torch.cuda.synchronize()
        ms_events = (time.perf_counter() - e0) * 1e3 / steps
        prof = plan.profile_read()
        per_call = [plan.profile_read_call(i) for i in range(prof["calls"])]
        plan.profile(False)
    ms = (t1 - t0) * 1e3 / steps
    model_bytes = w.update_bytes()
    pull_bytes = w.K * w.P * (8 + (w.grad_bytes if w.fused_sgd else 0))
    norm_bytes = w.K * w.P * w.grad_bytes
    n = max(1, prof["calls"])
    pull_ms = prof["pull_ms"] / n
    norm_ms = prof["norm_ms"] / n
    stats = {
        "workload": w.name, "variant": variant + ("+sgd" if w.fused_sgd else ""), "K": w.K, "L": w.L, "P": w.P,
        "grad_dtype": w.grad_dtype, "ms_per_step": ms, "updates_per_s": 1e3 / ms,
        "model_bytes": model_bytes, "GBps": model_bytes / (ms * 1e-3) / 1e9,
        "frac_of_peak": model_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "norm_kernel_ms": norm_ms, "norm_kernel_GBps": norm_bytes / (norm_ms * 1e-3) / 1e9 if norm_ms > 0 else None,
        "pull_kernel_ms": pull_ms, "pull_kernel_GBps": pull_bytes / (pull_ms * 1e-3) / 1e9 if pull_ms > 0 else None,
        "pull_kernel_bytes": pull_bytes, "tile_elems": info["tile_elems"], "n_tiles": info["n_tiles"],
        # per update, first kernel start to last kernel end on the device (the event pass)
        "graph_replay_ms_per_step": graph_ms, "ms_per_step_event_pass": ms_events,
        "device_ms": spread([c["span_ms"] for c in per_call]),
        "pull_kernel_ms_spread": spread([c["pull_ms"] for c in per_call]),
    }
    del x0
    return stats, x, g, w


def copy_ceiling(torch, grawa, nbytes=1 << 31, reps=10):
    """Read+write bandwidth of a plain 128-bit copy kernel over nbytes (twice nbytes of traffic)."""
    src = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda:0").normal_()
    dst = torch.empty_like(src)
    for _ in range(2):
        grawa.stream_copy(dst, src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        grawa.stream_copy(dst, src)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    ok = bool(torch.equal(dst, src))
    return {"GBps": 2 * nbytes / (ms * 1e-3) / 1e9, "ms": ms, "bytes_moved": 2 * nbytes, "verified": ok}


def time_phases(torch, grawa, W, idx, steps, warmup):
    """The calls around the distributed phase, on the same workload: local steps of Algorithms 1 and 2
    (SGD, + proximity step, + the running norm estimate of Appendix G), the local optimizer of the
    experiments (Nesterov momentum, Appendix B.2.2), one Local-GRAWA round, and the EASGD / LSGD
    phases of Appendix F.  GB/s under each call's minimum-traffic byte model, from events on the
    stream the kernels are launched on (torch's current stream)."""
    w = W.config(idx)
    x, g = W.make_inputs(w, device="cuda:0")
    K, P, sg = w.K, w.P, w.grad_bytes
    xv, gv = x[:, :P], g[:, :P]
    cen = torch.zeros(W.round_up(P, 256), device="cuda:0")
    losses = torch.rand(K, device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(1))
    lr = 1e-3
    out = {}

    def run(name, nbytes, fn):
        for _ in range(warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        out[name] = {"ms": ms, "bytes": nbytes, "GBps": nbytes / (ms * 1e-3) / 1e9,
                     "frac_of_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}

    step = K * P * (8 + sg)
    with grawa.Plan(K, P, w.offsets) as plan:
        def local_round():
            plan.local_step_scored(xv, gv, lr, 0.9)
            plan.local_lgrawa_update(xv, w.lam)

        run("local_sgd", step, lambda: grawa.local_sgd(xv, gv, lr))
        run("local_sgd_prox", step + 4 * P, lambda: grawa.local_sgd_prox(xv, gv, lr, cen, 0.05, 16.0))
        run("local_step_scored", step, lambda: plan.local_step_scored(xv, gv, lr, 0.9))
        run("local_step_scored_prox", step + 4 * P,
            lambda: plan.local_step_scored(xv, gv, lr, 0.9, center=cen, mu=0.05, tau=16.0))
        plan.local_scores_reset()
        run("local_round_1step_lgrawa", step + K * P * 8, local_round)
        run("easgd_update", K * P * 8 + 8 * P, lambda: plan.easgd_update(xv, w.lam, 0.5, cen))
        run("lsgd_update", K * P * 8, lambda: plan.lsgd_update(xv, losses, w.lam))
    del cen
    buf = torch.zeros_like(x)
    run("local_nesterov", K * P * (16 + sg), lambda: grawa.local_nesterov(xv, gv, buf[:, :P], lr, 0.9, 5e-4))
    del buf, x, g
    torch.cuda.empty_cache()
    return {"workload": w.name, "steps": steps, "calls": out}


def cpu_baseline(torch, W, w, variant, target_seconds):
    """The float64 CPU reference, as it stands, on the first n columns of the same seeded
    workload (all K workers, layers clipped to the sample); n is chosen from a short trial so
    that the run takes about target_seconds.  One thread: the reference is plain sequential C."""
    import numpy as np
    from oracle import grawa_oracle as orc

    x_dev, g_dev = W.make_inputs(w, device="cuda:0")

    def run(n):
        off = np.unique(np.clip(w.offsets, 0, n))
        x = W.to_numpy_params(x_dev[:, :n].contiguous())
        g = W.to_numpy_grads(g_dev[:, :n].contiguous())
        t0 = time.perf_counter()
        kw = dict(g_sgd=g, lr=w.lr) if w.fused_sgd else {}
        if variant == "lgrawa":
            orc.lgrawa_update(x, g, off, w.lam, **kw)
        else:
            orc.mgrawa_update(x, g, off, w.lam, **kw)
        return time.perf_counter() - t0

    n = min(w.P, 1 << 18)
    t = run(n)
    n_full = int(min(w.P, n * target_seconds / max(t, 1e-6)))
    n_full -= n_full % 8
    def run_all_cores(n, threads):
        """The same reference functions, the column range split over a thread pool: per-chunk partial
        sums of squares are added up, the weights follow once, center and pull are column-local.
        The slices are copied out beforehand so that only reference calls are timed."""
        from concurrent.futures import ThreadPoolExecutor
        off = np.unique(np.clip(w.offsets, 0, n))
        Ln = off.size - 1
        per = -(-n // (4 * threads))
        per += -per % 8
        jobs = []
        for i0 in range(0, n, per):
            i1 = min(n, i0 + per)
            l0 = int(np.searchsorted(off, i0, side="right") - 1)
            l1 = int(np.searchsorted(off, i1, side="left"))
            sub = np.clip(off[l0:l1 + 1], i0, i1) - i0
            jobs.append((l0, l1, sub, W.to_numpy_params(x_dev[:, i0:i1].contiguous()),
                         W.to_numpy_grads(g_dev[:, i0:i1].contiguous())))
        t0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=threads) as pool:
            S = np.zeros((w.K, Ln))
            for (l0, l1, _, _, _), part in zip(jobs, pool.map(lambda j: orc.grad_sumsq(j[4], j[2]), jobs)):
                S[:, l0:l1] += part
            if variant == "lgrawa":
                beta = orc.weights(orc.layer_norms(S))
            else:
                beta = orc.weights(orc.model_norms(S, "layersum"))

            def pull(j):
                l0, l1, sub, xs, gs = j
                kw = dict(g_sgd=gs, lr=w.lr) if w.fused_sgd else {}
                b = np.ascontiguousarray(beta[:, l0:l1]) if beta.ndim == 2 else beta
                orc.center_pull(xs, b, sub, w.lam, **kw)
                return 0
            list(pool.map(pull, jobs))
        return time.perf_counter() - t0

    reps = 1
    if n_full > n:
        n, t = n_full, run(n_full)
        if n == w.P - w.P % 8 and t < 0.6 * target_seconds:      # the whole workload is short: repeat it
            reps = int(min(50, max(1, round(target_seconds / t)) ))
            t = sum(run(n) for _ in range(reps)) / reps
    threads = max(1, min(16, os.cpu_count() or 1))
    t_all = run_all_cores(n, threads) if threads > 1 else None
    del x_dev, g_dev
    per = w.grad_bytes + 8 + (w.grad_bytes if w.fused_sgd else 0)
    sample_bytes = w.K * n * per
    all_cores = None
    if t_all:
        all_cores = {"value": sample_bytes / t_all / 1e9, "unit": "GB/s", "cores": threads, "seconds": t_all,
                     "how": "same reference functions, column range split over a thread pool, one update"}
    return {
        "all_cores": all_cores,
        "value": sample_bytes / t / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": "first %d of %d columns of %s, all %d workers, layers clipped to the sample, %d update(s); "
                  "%.1f s of CPU time in the reference; same byte model as value" % (n, w.P, w.name, w.K, reps, t * reps),
        "seconds": t * reps, "updates_per_s_extrapolated": 1.0 / (t * w.P / n), "host_cores_available": os.cpu_count(),
    }


def kernel_source_hash():
    """Hash of the library's kernel and host sources: counter figures taken from an older build are not
    reported for a newer one."""
    src = os.path.join(ROOT, "paper_2403_04206_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(src)):
        with open(os.path.join(src, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload, variant):
    """(bytes, source): HBM bytes per launch of the center+pull kernel from the committed rocprofv3
    counter runs (profiles/traffic.json: FETCH_SIZE and WRITE_SIZE, each scaled by what it reads for the
    plain copy kernel in the same run).  bytes is None when there is no entry for this workload or the
    library sources have changed since the counters were taken."""
    try:
        with open(os.path.join(ROOT, TRAFFIC_FILE)) as f:
            tj = json.load(f)
    except (OSError, ValueError):
        return None, "no %s" % TRAFFIC_FILE
    have, now = tj.get("source_hash"), kernel_source_hash()
    if have != now:
        return None, "%s was taken from library sources %s, this build is %s" % (TRAFFIC_FILE, have, now)
    entry = tj.get("workloads", {}).get(workload)
    if not entry or entry.get("variant") != variant:
        return None, "%s has no entry for %s (%s)" % (TRAFFIC_FILE, workload, variant)
    k = entry.get("kernels", {}).get("k_center_pull")
    if not k:
        return None, "%s has no center+pull entry for %s" % (TRAFFIC_FILE, workload)
    return k["total_bytes"], ("%s: rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE runs of this file, scaled by the "
                              "copy kernel of the same run (x%.3f, x%.3f); library sources %s; not re-measured in this "
                              "run" % (TRAFFIC_FILE, entry["fetch_scale"], entry["write_scale"], have))


def roofline_of(stats):
    """The roofline object of one timed configuration: the center+pull kernel (dominant), with the norm kernel
    beside it."""
    traffic, source = measured_traffic(stats["workload"], stats["variant"])
    return {
        "bound": "hbm", "kernel": "k_center_pull", "achieved": stats["pull_kernel_GBps"], "peak": HBM_PEAK_GBPS,
        "unit": "GB/s", "frac": (stats["pull_kernel_GBps"] or 0.0) / HBM_PEAK_GBPS,
        "traffic": traffic, "traffic_source": source,
        "bytes_per_launch": stats["pull_kernel_bytes"], "avg_launch_ms": stats["pull_kernel_ms"],
        "launch_ms": stats["pull_kernel_ms_spread"],
        "norm_kernel": {"kernel": "k_sumsq", "achieved": stats["norm_kernel_GBps"], "avg_launch_ms": stats["norm_kernel_ms"],
                        "bytes_per_launch": stats["K"] * stats["P"] * (2 if stats["grad_dtype"] == "bf16" else 4),
                        "frac": (stats["norm_kernel_GBps"] or 0.0) / HBM_PEAK_GBPS},
        "whole_update": {"GBps": stats["GBps"], "frac": stats["frac_of_peak"], "ms_per_step": stats["ms_per_step"],
                         "updates_per_s": stats["updates_per_s"], "bytes_per_update": stats["model_bytes"]},
    }


def time_config_in_child(idx, variant, steps, warmup):
    """One configuration timed in a fresh process: device memory that has been freed and allocated again in
    the same process is served a few percent slower (measured: 3 % on the norm kernel), and a job that
    runs this update allocates its arrays once, at its start."""
    import subprocess
    cmd = [sys.executable, os.path.abspath(__file__), "--config", str(idx), "--variant", variant, "--steps", str(steps),
           "--warmup", str(warmup), "--emit-stats"]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=600)
    if res.returncode != 0:
        raise RuntimeError("bench.py child for configuration %d failed:\n%s" % (idx, res.stderr[-2000:]))
    for line in res.stdout.splitlines():
        if line.startswith("{") and '"stats"' in line:
            return json.loads(line)["stats"]
    raise RuntimeError("bench.py child for configuration %d printed no record" % idx)


SWEEP_KEYS = ("workload", "variant", "ms_per_step", "updates_per_s", "GBps", "frac_of_peak", "pull_kernel_GBps",
              "norm_kernel_GBps", "graph_replay_ms_per_step", "ms_per_step_event_pass")


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: the GRAWA update runs on ONE GPU (all K workers of a configuration "
              "live on it); --gpus %d is not supported." % a.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2403_04206_amd import buildlib, grawa, workloads as W
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if not os.path.exists(grawa.LIB_PATH):
        buildlib.build(force=True)

    if a.only_phases:
        print(json.dumps({"metric": "grawa_phase_calls_hbm_bandwidth", "unit": "GB/s", "n_gpus": 1, "steps": a.steps,
                          "warmup": a.warmup, "data": "synthetic", "dtype": "f32",
                          "phases": time_phases(torch, grawa, W, a.config, a.steps, a.warmup),
                          "copy_kernel": copy_ceiling(torch, grawa)}), flush=True)   # calibrates hardware counters
        return
    stats, x, g, w = time_config(torch, grawa, W, a.config, a.variant, a.steps, a.warmup)
    del x, g
    torch.cuda.empty_cache()
    variant = pick_variant(w, a.variant)
    if a.emit_stats:
        print(json.dumps({"stats": stats}), flush=True)
        return

    out = {
        "metric": "grawa_update_hbm_bandwidth", "value": stats["GBps"], "unit": "GB/s", "n_gpus": 1,
        "steps": a.steps, "warmup": a.warmup, "ms_per_step": stats["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "variant": stats["variant"], "K": w.K, "L": w.L, "P": w.P,
                   "grad_dtype": w.grad_dtype, "lambda": w.lam, "bytes_per_update": stats["model_bytes"],
                   "tile_elems": stats["tile_elems"]},
        "frac_of_hbm_peak": stats["frac_of_peak"], "updates_per_s": stats["updates_per_s"],
        "device_ms_per_update": stats["device_ms"], "graph_replay_ms_per_step": stats["graph_replay_ms_per_step"],
        "ms_per_step_event_pass": stats["ms_per_step_event_pass"],
        "roofline": roofline_of(stats),
    }
    out["copy_kernel"] = copy_ceiling(torch, grawa)
    out["frac_of_copy_kernel"] = stats["GBps"] / out["copy_kernel"]["GBps"]     # against this machine's own copy rate
    torch.cuda.empty_cache()
    by_config = {w.name + "/" + stats["variant"]: roofline_of(stats)} if a.config in TARGET_CONFIGS else {}
    if not a.no_sweep:
        sweep = []
        for i in range(W.N_CONFIGS):
            for var in W.config(i).variants:
                if i == a.config and var == variant:
                    sweep.append({k: stats[k] for k in SWEEP_KEYS})
                    continue
                try:
                    s = time_config_in_child(i, var, a.steps, a.warmup)
                except Exception as e:        # reported; the configuration is then timed in this process instead
                    print("bench.py: %s; timing configuration %d here" % (e, i), file=sys.stderr)
                    s, x, g, _ = time_config(torch, grawa, W, i, var, a.steps, a.warmup)
                    del x, g
                    torch.cuda.empty_cache()
                sweep.append({k: s[k] for k in SWEEP_KEYS})
                if i in TARGET_CONFIGS and var == pick_variant(W.config(i), None):
                    by_config[s["workload"] + "/" + s["variant"]] = roofline_of(s)
        out["all_configs"] = sweep
        out["roofline_by_config"] = by_config
    if not a.no_phases and not a.no_sweep:
        out["phases"] = time_phases(torch, grawa, W, a.config, a.steps, a.warmup)
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(torch, W, w, variant, a.cpu_seconds)
        if not a.no_sweep:
            cb = {w.name: out["cpu_baseline"]}
            for i in TARGET_CONFIGS:
                if i != a.config:
                    wi = W.config(i)
                    cb[wi.name] = cpu_baseline(torch, W, wi, pick_variant(wi, None), a.cpu_seconds)
            out["cpu_baseline_by_config"] = cb
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

"""Turn rocprofv3 CSV output of bench.py runs into the short text summaries kept under
profiles/ and into profiles/traffic.txt (HBM bytes per launch of the update kernels).

Expected input, one directory per run (any parent folder):
    <dir>/prof_cfg<N>_stats   from  rocprofv3 --kernel-trace --stats -d <that dir> --output-format csv
                                    -- python3 bench.py --config <N> --no-sweep --no-cpu-baseline
    <dir>/prof_cfg<N>_fetch   same command with  --pmc FETCH_SIZE   instead of --kernel-trace --stats
    <dir>/prof_cfg<N>_write   same command with  --pmc WRITE_SIZE
    <dir>/prof_cfg<N>_phases  (optional) --kernel-trace --stats of
                                    python3 bench.py --config <N> --only-phases
    <dir>/prof_cfg<N>_phases_fetch, _phases_write  (optional) the same with --pmc FETCH_SIZE / WRITE_SIZE

FETCH_SIZE / WRITE_SIZE are reported in KiB per dispatch.  Each is scaled by what the same
counter reads, in the same run, for the library's plain copy kernel (bench.py launches it over
2 GiB: 2 GiB read, 2 GiB written), because the raw counters do not weigh every request size
correctly (streaming loads are counted at half their size on this part).

usage: python -m paper_2403_04206_amd.profile_summary <dir with prof_cfg*_*> [configs...]
"""
from __future__ import annotations

import collections
import csv
import glob
import hashlib
import json
import os
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
COPY_BYTES = 1 << 31


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    for name in sorted(os.listdir(os.path.join(PKG, "csrc"))):
        with open(os.path.join(PKG, "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def short(name: str) -> str:
    name = name.strip('"')
    if name.startswith("void "):
        name = name[5:]
    return name.split("(")[0]


def read_counters(run_dir: str, counter: str):
    files = glob.glob(os.path.join(run_dir, "*", "*counter_collection.csv"))
    if not files:
        raise FileNotFoundError("no counter_collection.csv under " + run_dir)
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(files[0])):
        if r["Counter_Name"] == counter:
            agg[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return {k: (sum(v) / len(v), len(v)) for k, v in agg.items()}


def read_stats(run_dir: str):
    files = glob.glob(os.path.join(run_dir, "*", "*kernel_stats.csv"))
    if not files:
        raise FileNotFoundError("no kernel_stats.csv under " + run_dir)
    return [(short(r["Name"]), int(r["Calls"]), float(r["AverageNs"]), float(r["MinNs"]), float(r["MaxNs"]),
             float(r["Percentage"])) for r in csv.DictReader(open(files[0]))]


def bench_line(run_dir: str):
    with open(os.path.join(run_dir, "run.log")) as f:
        for line in f:
            if line.startswith("{") and '"metric"' in line:
                return json.loads(line)
    return None


def summarize(base: str, cfg: int, out_dir: str):
    stats_dir = os.path.join(base, "prof_cfg%d_stats" % cfg)
    stats = read_stats(stats_dir)
    bl = bench_line(stats_dir)
    fetch = read_counters(os.path.join(base, "prof_cfg%d_fetch" % cfg), "FETCH_SIZE")
    write = read_counters(os.path.join(base, "prof_cfg%d_write" % cfg), "WRITE_SIZE")
    copy_f = fetch["k_stream_copy"][0] * 1024.0
    copy_w = write["k_stream_copy"][0] * 1024.0
    f_scale, w_scale = COPY_BYTES / copy_f, COPY_BYTES / copy_w
    w = bl["config"]
    K, P = w["K"], w["P"]
    gb = 2 if w["grad_dtype"] == "bf16" else 4
    fused = w["variant"].endswith("+sgd")
    algo = {"k_sumsq": K * P * gb, "k_center_pull": K * P * (8 + (gb if fused else 0))}

    lines = []
    lines.append("# rocprofv3 summary: GRAWA update kernels, %s (%s)" % (w["workload"], w["variant"]))
    lines.append("")
    lines.append("K=%d workers, L=%d layers, P=%d parameters, gradients %s, library source hash %s." %
                 (K, w["L"], P, w["grad_dtype"], kernel_source_hash()))
    lines.append("")
    lines.append("Commands (run from /tmp with TMPDIR=/tmp, repository root = $R):")
    lines.append("")
    for args in ("--kernel-trace --stats", "--pmc FETCH_SIZE", "--pmc WRITE_SIZE"):
        lines.append("    rocprofv3 %s -d <out> --output-format csv -- python3 $R/bench.py --config %d --no-sweep "
                     "--no-cpu-baseline" % (args, cfg))
    lines.append("")
    lines.append("The CSV output of the three runs was turned into this file by "
                 "`python -m paper_2403_04206_amd.profile_summary <dir holding the three output folders> %d`." % cfg)
    lines.append("")
    lines.append("bench.py line of the --kernel-trace run: value %.0f GB/s (%.1f%% of 8 TB/s), %.4f ms/update, "
                 "%.0f updates/s; center+pull kernel from HIP events %.4f ms/launch." %
                 (bl["value"], 100 * bl["frac_of_hbm_peak"], bl["ms_per_step"], bl["updates_per_s"],
                  bl["roofline"]["avg_launch_ms"]))
    lines.append("")
    lines.append("## --kernel-trace --stats (library kernels only)")
    lines.append("")
    lines.append("| kernel | calls | avg us | min us | max us | algorithmic bytes/launch | GB/s at avg | % of 8 TB/s |")
    lines.append("|---|---|---|---|---|---|---|---|")
    traffic = {}
    for name, calls, avg, mn, mx, _pct in stats:
        base_name = name.split("<")[0]
        if not base_name.startswith(("k_", "grawa")):
            continue
        ab = algo.get(base_name)
        if base_name == "k_stream_copy":
            ab = 2 * COPY_BYTES
        gbps = "%.0f" % (ab / avg) if ab else "-"
        frac = "%.1f" % (100 * ab / avg / 8000.0) if ab else "-"
        lines.append("| %s | %d | %.1f | %.1f | %.1f | %s | %s | %s |" %
                     (name, calls, avg / 1e3, mn / 1e3, mx / 1e3, ab if ab else "-", gbps, frac))
    lines.append("")
    lines.append("## HBM traffic per launch (--pmc FETCH_SIZE, --pmc WRITE_SIZE; KiB per dispatch, averaged)")
    lines.append("")
    lines.append("Calibration on the plain copy kernel of the same run (2 GiB read + 2 GiB written): FETCH_SIZE reads "
                 "%.0f KiB (scale %.4f), WRITE_SIZE reads %.0f KiB (scale %.4f)." %
                 (copy_f / 1024, f_scale, copy_w / 1024, w_scale))
    lines.append("")
    lines.append("| kernel | FETCH_SIZE KiB | WRITE_SIZE KiB | scaled read bytes | scaled written bytes | scaled total | "
                 "algorithmic bytes | total / algorithmic |")
    lines.append("|---|---|---|---|---|---|---|---|")
    for name in sorted(fetch):
        base_name = name.split("<")[0]
        if base_name not in algo:
            continue
        fr = fetch[name][0] * 1024 * f_scale
        wr = write.get(name, (0.0, 0))[0] * 1024 * w_scale
        tot = fr + wr
        lines.append("| %s | %.0f | %.0f | %.4g | %.4g | %.4g | %d | %.4f |" %
                     (name, fetch[name][0], write.get(name, (0.0, 0))[0], fr, wr, tot, algo[base_name],
                      tot / algo[base_name]))
        traffic[base_name] = {"kernel": name, "read_bytes": fr, "written_bytes": wr, "total_bytes": tot,
                              "algorithmic_bytes": algo[base_name]}
    lines.append("")
    name = "update_kernels_%s.md" % w["workload"]
    with open(os.path.join(out_dir, name), "w") as f:
        f.write("\n".join(lines) + "\n")
    return w["workload"], {"variant": w["variant"], "fetch_scale": f_scale, "write_scale": w_scale, "kernels": traffic}


def template_args(name: str):
    if "<" not in name or ">" not in name or name.rindex(">") < name.index("<"):
        return []
    return [a.strip() for a in name[name.index("<") + 1:name.rindex(">")].split(",")]


def summarize_phases(base: str, cfg: int, out_dir: str):
    """Kernel table of the calls around the distributed phase (bench.py --only-phases)."""
    run_dir = os.path.join(base, "prof_cfg%d_phases" % cfg)
    if not os.path.isdir(run_dir):
        return None
    stats = read_stats(run_dir)
    bl = bench_line(run_dir)
    ph = bl["phases"]
    from . import workloads as W
    w = W.config(cfg)
    K, P, gb = w.K, w.P, w.grad_bytes
    lines = ["# rocprofv3 summary: local-phase, Nesterov and Appendix F kernels, %s" % ph["workload"], "",
             "K=%d workers, L=%d layers, P=%d parameters, gradients %s, library source hash %s." %
             (K, w.L, P, w.grad_dtype, kernel_source_hash()), "",
             "Command (run from /tmp with TMPDIR=/tmp, repository root = $R):", "",
             "    rocprofv3 --kernel-trace --stats -d <out> --output-format csv -- python3 $R/bench.py --config %d "
             "--only-phases" % cfg, "",
             "(and the same command under `--pmc FETCH_SIZE` and `--pmc WRITE_SIZE` for the traffic table); turned "
             "into this file by `python -m paper_2403_04206_amd.profile_summary <dir> %d`." % cfg, "",
             "## Calls, from stream events inside bench.py (minimum-traffic byte model of each call)", "",
             "| call | ms | bytes | GB/s | % of 8 TB/s |", "|---|---|---|---|---|"]
    for name, c in ph["calls"].items():
        lines.append("| %s | %.4f | %d | %.0f | %.1f |" % (name, c["ms"], c["bytes"], c["GBps"], 100 * c["frac_of_peak"]))
    lines += ["", "## --kernel-trace --stats (library kernels only)", "",
              "k_row_step<grad type, V, U, streaming, PROX, SCORE>: SGD (+ proximity step) (+ per-tile gradient "
              "sums of squares), one worker per block.  k_center_pull here serves the Local-GRAWA communication "
              "and the EASGD and LSGD phases together.", "",
              "| kernel | calls | avg us | min us | max us | algorithmic bytes/launch | GB/s at avg | % of 8 TB/s |",
              "|---|---|---|---|---|---|---|---|"]
    for name, calls, avg, mn, mx, _pct in stats:
        base_name = name.split("<")[0]
        if not base_name.startswith("k_"):
            continue
        ta = template_args(name)
        ab = None
        if base_name == "k_nesterov":
            ab = K * P * (16 + gb)
        elif base_name == "k_row_step":
            ab = K * P * (8 + gb) + (4 * P if len(ta) > 4 and ta[4] == "true" else 0)
        elif base_name == "k_center_pull":
            ab = K * P * 8
        gbps = "%.0f" % (ab / avg) if ab else "-"
        frac = "%.1f" % (100 * ab / avg / 8000.0) if ab else "-"
        lines.append("| %s | %d | %.1f | %.1f | %.1f | %s | %s | %s |" %
                     (name, calls, avg / 1e3, mn / 1e3, mx / 1e3, ab if ab else "-", gbps, frac))
    fdir, wdir = run_dir + "_fetch", run_dir + "_write"
    if os.path.isdir(fdir) and os.path.isdir(wdir):
        fetch, write = read_counters(fdir, "FETCH_SIZE"), read_counters(wdir, "WRITE_SIZE")
        f_scale = COPY_BYTES / (fetch["k_stream_copy"][0] * 1024.0)
        w_scale = COPY_BYTES / (write["k_stream_copy"][0] * 1024.0)
        lines += ["", "## HBM traffic per launch (--pmc FETCH_SIZE, --pmc WRITE_SIZE of the same command)", "",
                  "Scaled by what the counters read for the plain copy kernel in the same run (scales %.4f and %.4f). "
                  "The proximity center is read by every worker's blocks but fetched from HBM about once: the "
                  "launch order keeps it in cache." % (f_scale, w_scale), "",
                  "| kernel | scaled read bytes | scaled written bytes | total | algorithmic bytes | total / algorithmic |",
                  "|---|---|---|---|---|---|"]
        for name in sorted(fetch):
            base_name = name.split("<")[0]
            ta = template_args(name)
            if base_name == "k_nesterov":
                ab = K * P * (16 + gb)
            elif base_name == "k_row_step":
                ab = K * P * (8 + gb) + (4 * P if len(ta) > 4 and ta[4] == "true" else 0)
            else:
                continue
            fr = fetch[name][0] * 1024 * f_scale
            wr = write.get(name, (0.0, 0))[0] * 1024 * w_scale
            lines.append("| %s | %.4g | %.4g | %.4g | %d | %.4f |" % (name, fr, wr, fr + wr, ab, (fr + wr) / ab))
    lines.append("")
    out = os.path.join(out_dir, "phase_kernels_%s.md" % ph["workload"])
    with open(out, "w") as f:
        f.write("\n".join(lines) + "\n")
    return out


def main(argv):
    base = argv[1]
    cfgs = [int(a) for a in argv[2:]] or [2, 3, 4]
    out_dir = os.path.join(ROOT, "profiles")
    os.makedirs(out_dir, exist_ok=True)
    tj = {"source_hash": kernel_source_hash(), "workloads": {}}
    for c in cfgs:
        name, t = summarize(base, c, out_dir)
        tj["workloads"][name] = t
        print("wrote summary for", name)
        if summarize_phases(base, c, out_dir):
            print("wrote phase summary for", name)
    with open(os.path.join(out_dir, "traffic.txt"), "w") as f:
        json.dump(tj, f, indent=1)


if __name__ == "__main__":
    main(sys.argv)

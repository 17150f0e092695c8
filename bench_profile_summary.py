"""Turns the output of a rocprofv3 run of bench.py into the short summaries kept under profiles/.

    python bench_profile_summary.py stats   <rocprofv3 output dir> <bench stdout log> <out.md> "<command>"
    python bench_profile_summary.py traffic <FETCH_SIZE output dir> <WRITE_SIZE output dir> <out.md> <out.json> "<command>"
    python bench_profile_summary.py counters <out.md> "<command>" <kernel name parts, comma separated, or -> <output dir> ...

`stats` lists the per-kernel rows of a `--kernel-trace --stats` run beside bench.py's own line.  `traffic` sums
FETCH_SIZE / WRITE_SIZE per kernel, scales them by what the same counters read for the known-size calibration
copy, and writes the gate/up GEMM's bytes per launch (with a hash of the kernel's source) to the JSON that
bench.py reads for `roofline.traffic`.  `counters` sums any other --pmc counters per kernel.
"""
import collections
import csv
import glob
import json
import os
import sys
import time


def _short(name):
    name = name.replace("void keep::", "").replace("keep::", "")
    return name[:name.index("(")] if "(" in name else name


def _counter_rows(d, after_calibration=True):
    """Rows of the counter CSV.  With after_calibration, only the dispatches that follow bench.py's calibration copy
    (--calib-copy-mib: the longest-running device-to-device copy), i.e. without the set-up launches (weights,
    group caches), but including that copy itself; the profiler cannot be paused in a --pmc run."""
    f = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
    if not f:
        raise SystemExit("no counter_collection.csv under " + d)
    rows = list(csv.DictReader(open(f[0])))
    if after_calibration:
        copies = [r for r in rows if "copyBuffer" in r["Kernel_Name"]]
        if copies:
            dur = lambda r: int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
            mark = max(copies, key=dur)
            if dur(mark) >= 50000:      # ns: a copy of hundreds of MiB, not a table upload
                first = int(mark["Dispatch_Id"])
                rows = [r for r in rows if int(r["Dispatch_Id"]) >= first]
    return rows


def _per_kernel(rows):
    """counter -> kernel -> [calls, total, max] (one row per dispatch and counter)."""
    out = collections.defaultdict(lambda: collections.defaultdict(lambda: [0, 0.0, 0.0]))
    for r in rows:
        e = out[r["Counter_Name"]][_short(r["Kernel_Name"])]
        v = float(r["Counter_Value"])
        e[0] += 1
        e[1] += v
        e[2] = max(e[2], v)
    return out


def stats(argv):
    d, benchlog, out, cmd = argv
    f = glob.glob(os.path.join(d, "**", "*kernel_stats.csv"), recursive=True)
    rows = list(csv.DictReader(open(f[0])))
    bench = json.loads([l for l in open(benchlog) if l.startswith("{")][-1])
    with open(out, "w") as o:
        o.write("# rocprofv3 kernel stats: keep_prefill, %s (one MI355X)\n\n" % bench["config"]["workload"].split(":")[0])
        o.write("Command (from /tmp with TMPDIR=/tmp on the GPU box):\n\n    %s\n\n" % cmd)
        o.write("bench.py pauses the profiler during set-up (roctxProfilerPause/Resume, honoured with --marker-trace), so "
                "the rows cover the warm-up, the timed steps and the one fully instrumented step.\n\n")
        o.write("| kernel | calls | total ms | avg us | % | min us | max us |\n|---|---|---|---|---|---|---|\n")
        for r in rows:
            if float(r["Percentage"]) < 0.01:
                continue
            o.write("| `%s` | %s | %.2f | %.1f | %s | %.1f | %.1f |\n" % (
                _short(r["Name"])[:70], r["Calls"], int(r["TotalDurationNs"]) / 1e6, float(r["AverageNs"]) / 1e3,
                r["Percentage"], int(r["MinNs"]) / 1e3, int(r["MaxNs"]) / 1e3))
        n_calls = sum(int(r["Calls"]) for r in rows)
        o.write("\nKernel launches in all: %d.\n" % n_calls)
        o.write("\nbench.py line of the same run (HIP-event timings on the compute stream):\n\n")
        o.write("    TTFT %.1f ms (median %.1f, min %.1f), %.0f tokens/s; roofline kernel: avg launch %.4f ms, %.1f TFLOP/s = %.3f of 2500\n" % (
            bench["ms_per_step"], bench.get("ttft_ms_median", 0), bench.get("ttft_ms_min", 0), bench["value"],
            bench["roofline"]["avg_launch_ms"], bench["roofline"]["achieved"], bench["roofline"]["frac"]))
        for k, v in bench["kernels"].items():
            if "achieved" in v:
                o.write("    %-24s %8.2f ms/step  %9.2f %s  (%.3f of peak)\n" % (k, v["ms_per_step"], v["achieved"], v["unit"], v["frac"]))
            else:
                o.write("    %-24s %s\n" % (k, json.dumps(v)))


def traffic(argv):
    d_fetch, d_write, out_md, out_json, cmd = argv
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    import bench
    pk = {"FETCH_SIZE": _per_kernel(_counter_rows(d_fetch))["FETCH_SIZE"],
          "WRITE_SIZE": _per_kernel(_counter_rows(d_write))["WRITE_SIZE"]}
    # calibration: the largest device-to-device copy of the run moved a known number of bytes
    calib = {}
    for c in pk:
        copies = [v for k, v in pk[c].items() if "copyBuffer" in k]
        calib[c] = max(v[2] for v in copies) if copies else 0.0
    copy_kib = None
    for part in cmd.split():
        if part.isdigit():
            copy_kib = int(part) * 1024
    f_scale = copy_kib / calib["FETCH_SIZE"] if calib["FETCH_SIZE"] else 0.0
    w_scale = copy_kib / calib["WRITE_SIZE"] if calib["WRITE_SIZE"] else 0.0
    gu = lambda c: sum(v[1] for k, v in pk[c].items() if k.startswith("k_gemm_mfma<256, 256, 4, 2, 2") or k.startswith("k_gemm_fixup<256, 256, 4, 2, 2"))
    launches = sum(v[0] for k, v in pk["FETCH_SIZE"].items() if k.startswith("k_gemm_mfma<256, 256, 4, 2, 2"))
    bytes_per_launch = (gu("FETCH_SIZE") * f_scale + gu("WRITE_SIZE") * w_scale) * 1024.0 / max(1, launches)
    with open(out_json, "w") as o:
        json.dump({"bytes_per_launch": int(bytes_per_launch), "launches": launches, "fetch_scale": round(f_scale, 4),
                   "write_scale": round(w_scale, 4), "sources_sha16": bench.sources_sha16(),
                   "measured_at": time.strftime("%Y-%m-%d"), "command": cmd}, o, indent=1)
        o.write("\n")
    with open(out_md, "w") as o:
        o.write("# rocprofv3 counters FETCH_SIZE / WRITE_SIZE: keep_prefill, workload qwen14b_32k (one MI355X)\n\n")
        o.write("Commands (each from /tmp with TMPDIR=/tmp on the GPU box, one counter per run):\n\n    %s\n    %s\n\n"
                % (cmd.replace("COUNTER", "FETCH_SIZE"), cmd.replace("COUNTER", "WRITE_SIZE")))
        o.write("Calibration (same runs): the %d KiB device-to-device copy reads %.0f KiB by FETCH_SIZE and writes %.0f KiB "
                "by WRITE_SIZE, so true bytes = %.2f x FETCH_SIZE and %.2f x WRITE_SIZE.  The counters sit between L2 and "
                "the fabric: they count L2 misses, whether the Infinity Cache or HBM serves them.\n\n"
                % (copy_kib, calib["FETCH_SIZE"], calib["WRITE_SIZE"], f_scale, w_scale))
        o.write("Gate/up GEMM (k_gemm_mfma<256,256,4,2,SWIGLU> + its fix-up): %d launches, %.3f GB per launch (scaled).\n\n"
                % (launches, bytes_per_launch / 1e9))
        att = [pk[c].get("k_attn_mfma", (0, 0.0, 0.0)) for c in ("FETCH_SIZE", "WRITE_SIZE")]
        if att[0][0]:
            o.write("Attention (k_attn_mfma, %d launches: the step's 48 plus the on-demand launches of layer 0 and the launches "
                    "of the row-sparse diagnostic): %.1f MB fetched and %.1f MB written per launch on average (scaled); K and V "
                    "of one layer are 135 MB.\n\n"
                    % (att[0][0], att[0][1] * f_scale * 1024.0 / att[0][0] / 1e6, att[1][1] * w_scale * 1024.0 / att[0][0] / 1e6))
        o.write("```\n")
        for c in ("FETCH_SIZE", "WRITE_SIZE"):
            o.write(c + " (KiB as counted)\n")
            for k, v in sorted(pk[c].items(), key=lambda kv: -kv[1][1])[:16]:
                o.write("  %-64s calls %5d  total %12.0f  max %10.0f\n" % (k[:64], v[0], v[1], v[2]))
        o.write("```\n")


def counters(argv):
    out_md, cmd, part = argv[0], argv[1], argv[2]
    dirs = argv[3:]
    want = [w for w in part.split(",") if w and w != "-"]
    with open(out_md, "w") as o:
        o.write("# rocprofv3 --pmc counters per kernel (one MI355X)\n\nCommand (from /tmp with TMPDIR=/tmp on the GPU box; "
                "one run per counter set, COUNTERS = the names listed under each kernel):\n\n    %s\n\nValues are sums over all "
                "dispatches of the kernel in the run and over the chip's counter instances (SQ counters: all CUs).\n\n" % cmd)
        merged = collections.defaultdict(dict)
        for d in dirs:
            pk = _per_kernel(_counter_rows(d))
            for c, per in pk.items():
                for k, v in per.items():
                    merged[k][c] = v
        for k in sorted(merged, key=lambda k: -max(v[1] for v in merged[k].values())):
            if want and not any(w in k for w in want):
                continue
            o.write("`%s`\n\n" % k[:100])
            for c in sorted(merged[k]):
                o.write("    %-34s calls %5d  total %.6g\n" % (c, merged[k][c][0], merged[k][c][1]))
            cs = merged[k]
            if "SQ_VALU_MFMA_BUSY_CYCLES" in cs and "SQ_BUSY_CU_CYCLES" in cs and cs["SQ_BUSY_CU_CYCLES"][1] > 0:
                # MFMA busy cycles are counted per SIMD (4 per CU), CU busy cycles per CU
                o.write("    -> matrix pipe busy %.3f of the cycles its CUs were busy\n"
                        % (cs["SQ_VALU_MFMA_BUSY_CYCLES"][1] / (4.0 * cs["SQ_BUSY_CU_CYCLES"][1])))
            if "SQ_WAIT_ANY" in cs and "SQ_WAVE_CYCLES" in cs and cs["SQ_WAVE_CYCLES"][1] > 0:
                o.write("    -> waves waiting %.3f of their cycles (LDS: %.3f)\n"
                        % (cs["SQ_WAIT_ANY"][1] / cs["SQ_WAVE_CYCLES"][1],
                           cs.get("SQ_WAIT_INST_LDS", [0, 0.0])[1] / cs["SQ_WAVE_CYCLES"][1]))
            o.write("\n")


if __name__ == "__main__":
    modes = {"stats": stats, "traffic": traffic, "counters": counters}
    if len(sys.argv) < 2 or sys.argv[1] not in modes:
        print(__doc__)
        sys.exit(0 if len(sys.argv) > 1 and sys.argv[1] in ("-h", "--help") else 2)
    modes[sys.argv[1]](sys.argv[2:])

"""Turns the raw output of profile.sh (rocprofv3 kernel trace and counter passes of bench.py) into the
short text summaries kept under profiles/.

usage: python -m paper_2603_14303_amd.profile_summary <tag> <dir written by profile.sh> [bench.py arguments]
writes <dir>/<tag>_kernel_stats.md, <dir>/hbm_traffic_<tag>.txt, <dir>/<tag>_sq_counters.md
"""
from __future__ import annotations

import csv
import glob
import json
import os
import sqlite3
import sys


def _last_json(path):
    if not os.path.exists(path):
        return None
    for line in reversed(open(path).read().strip().splitlines()):
        if line.startswith("{"):
            return json.loads(line)
    return None


def _short(name):
    return name.replace("void ", "").split("(")[0]


def _counters(dirname, largest=False):
    """{(kernel, counter): (dispatches, mean value)} from the .db of one counter pass; with `largest`, the
    largest value of a dispatch instead of the mean (a kernel launched on buffers of several sizes)."""
    out = {}
    for db_path in glob.glob(os.path.join(dirname, "**", "*.db"), recursive=True):
        db = sqlite3.connect(db_path)
        q = "select kernel_name, counter_name, count(*), %s(value) from counters_collection group by kernel_name, counter_name" % ("max" if largest else "avg")
        for k, c, n, v in db.execute(q):
            out[(_short(k), c)] = (n, v)
    return out


def main():
    tag, out = sys.argv[1], sys.argv[2]
    bench_args = " ".join(sys.argv[3:])
    root_cmd = "python3 $R/bench.py --no-cpu-baseline"
    # ------------------------------------------------------------------ kernel trace
    stats = glob.glob(os.path.join(out, "trace", "**", "*kernel_stats.csv"), recursive=True)
    rows = list(csv.DictReader(open(stats[0]))) if stats else []
    bj = _last_json(os.path.join(out, "bench_traced.json"))
    pj = _last_json(os.path.join(out, "bench_plain.json"))
    lines = ["# rocprofv3 kernel-trace summary: bench.py %s" % (bench_args or "(default workload layer32k)"), ""]
    lines += ["Workload: %s" % (bj or pj)["config"]["workload"], ""]
    lines += ["Command (run from /tmp with TMPDIR=/tmp, repository root in $R; `paper_2603_14303_amd/profile.sh %s %s` runs it):" % (tag, bench_args), "",
              "    rocprofv3 --kernel-trace --stats --output-format csv -d $R/gpurun_out/prof_%s/trace -o run -- \\" % tag,
              "        %s --steps 10 --warmup 3 %s" % (root_cmd, bench_args), ""]
    lines += ["Kernel statistics (`run_kernel_stats.csv`; microseconds; kernels of this library and the runtime's copy kernel):", "",
              "| kernel | calls | avg us | min us | max us | stddev us | % of GPU time |", "|---|---:|---:|---:|---:|---:|---:|"]
    for r in rows:
        if "sc::" in r["Name"] or "copyBuffer" in r["Name"]:
            lines.append("| `%s` | %s | %.2f | %.2f | %.2f | %.2f | %s |" % (_short(r["Name"]), r["Calls"], float(r["AverageNs"]) / 1e3,
                         float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3, float(r["StdDev"]) / 1e3, r["Percentage"]))
    def bench_lines(j, title):
        rl, rd = j["roofline"], j["roofline_decode"]
        return ["", title, "",
                "* `sc_gsc_merge` call (its kernels back to back): %.2f us; `sc_segment` %.2f us; `sc_decode_attn` %.2f us per call" % (rl["us"], j["sc_segment_ms"] * 1e3, rd["us"]),
                "* value %.1f Mtok/s (stack: %.1f); roofline of the merge call %.0f GB/s of %d algorithmic bytes = %.3f of 8 TB/s; decode %.0f GB/s of %d B = %.3f"
                % (j["value"], j["stack_Mtok_per_s"], rl["achieved"], rl["algorithmic_bytes"], rl["frac"], rd["achieved"], rd["algorithmic_bytes"], rd["frac"]),
                "* attainable on this device: streaming read %.0f GB/s, device-to-device copy %.0f GB/s" % (j["attainable"]["stream_read_GBps"], j["attainable"]["d2d_copy_GBps"])]
    if bj:
        lines += bench_lines(bj, "What bench.py measured with HIP events in the traced run (graph replays; tracing adds time to every launch):")
    if pj:
        lines += bench_lines(pj, "The same command without the profiler (`%s %s`):" % (root_cmd, bench_args))
    open(os.path.join(out, "%s_kernel_stats.md" % tag), "w").write("\n".join(lines) + "\n")

    # ------------------------------------------------------------------ HBM traffic
    F, W = _counters(os.path.join(out, "pmc1")), _counters(os.path.join(out, "pmc2"))
    j1 = _last_json(os.path.join(out, "bench_pmc1.json")) or pj
    # the runtime's copy kernel also moves smaller buffers (uploads of the inputs): its largest dispatch is the 512 MiB copy
    Fmax, Wmax = _counters(os.path.join(out, "pmc1"), True), _counters(os.path.join(out, "pmc2"), True)
    copy_f = [v for (k, c), (n, v) in Fmax.items() if "copyBuffer" in k and c == "FETCH_SIZE"]
    copy_w = [v for (k, c), (n, v) in Wmax.items() if "copyBuffer" in k and c == "WRITE_SIZE"]
    read_f = [v for (k, c), (n, v) in F.items() if "stream_read_kernel" in k and c == "FETCH_SIZE"]
    COPY_KIB = 512.0 * 1024.0     # bench.py copies 512 MiB device to device
    READ_KIB = 1024.0 * 1024.0    # and streams 1 GiB through sc_stream_read_probe
    ff = READ_KIB / max(read_f) if read_f else float("nan")
    ff_copy = COPY_KIB / max(copy_f) if copy_f else float("nan")
    wf = COPY_KIB / max(copy_w) if copy_w else float("nan")
    t = ["# HBM traffic per launch from rocprofv3 hardware counters: bench.py %s" % bench_args,
         "# workload: %s" % j1["config"]["workload"],
         "# Commands (from /tmp with TMPDIR=/tmp, repository root in $R), one counter per run:",
         "#   rocprofv3 --pmc FETCH_SIZE -d $R/gpurun_out/prof_%s/pmc1 -o run -- %s --eager --steps 2 --warmup 1 %s" % (tag, root_cmd, bench_args),
         "#   rocprofv3 --pmc WRITE_SIZE -d $R/gpurun_out/prof_%s/pmc2 -o run -- %s --eager --steps 2 --warmup 1 %s" % (tag, root_cmd, bench_args),
         "# Counter values are KiB per dispatch, averaged over the dispatches of the run.",
         "# Calibration with kernels of known size that bench.py launches in the same run.  Reads: sc::stream_read_kernel",
         "# (16 bytes per lane like the kernels here) over 1 GiB reads FETCH_SIZE = %.1f KiB -> fetch_scale = 1048576 / reading" % (max(read_f) if read_f else float("nan")),
         "# (the FETCH_SIZE formula prices the wide read requests of 16-byte-per-lane kernels at half their size).",
         "# Writes: the runtime's device-to-device copy kernel (__amd_rocclr_copyBuffer) on 512 MiB, its largest dispatch:",
         "# WRITE_SIZE = %.1f KiB -> write_scale = 524288 / reading.  (The same copy reads FETCH_SIZE = %.1f KiB, a factor %.3f.)"
         % (max(copy_w) if copy_w else float("nan"), max(copy_f) if copy_f else float("nan"), ff_copy),
         "workload_tokens %d" % j1["config"]["tokens"], "tau %s" % bench_args_tau(sys.argv[3:], j1),
         "compressed_rows %d" % j1["config"]["compressed_rows"],
         "fetch_scale %.5f" % ff, "write_scale %.5f" % wf]
    total = {}
    for key, pats in (("gsc_compress", ("gsc_compress_kernel",)), ("gsc_scan", ("gsc_scan_kernel",)), ("gsc_relocate", ("gsc_relocate_kernel",)),
                      ("decode", ("decode_bf16_kernel",)), ("decode_mfma", ("multi_attn_kernel",)), ("decode_mfma_combine", ("multi_attn_combine_kernel",)),
                      ("segment", ("segment_kernel",))):
        f = [(n, v) for (k, c), (n, v) in F.items() if c == "FETCH_SIZE" and all(p in k for p in pats)]
        wv = [(n, v) for (k, c), (n, v) in W.items() if c == "WRITE_SIZE" and all(p in k for p in pats)]
        if not f or not wv:
            continue
        fn, fv = max(f); wn, wvv = max(wv)
        t.append("%s_fetch_kib_raw %.1f   # %d dispatches" % (key, fv, fn))
        t.append("%s_write_kib_raw %.1f   # %d dispatches" % (key, wvv, wn))
        total[key] = (fv * ff + wvv * wf) * 1024.0
        t.append("%s_bytes %d" % (key, total[key]))
    gm = sum(total.get(k, 0.0) for k in ("gsc_compress", "gsc_scan", "gsc_relocate"))
    t.append("gsc_merge_bytes %d   # all kernels of the call; algorithmic bytes %d" % (gm, j1["roofline"]["algorithmic_bytes"]))
    dk = total.get("decode", 0.0) or (total.get("decode_mfma", 0.0) + total.get("decode_mfma_combine", 0.0))
    t.append("decode_bytes %d   # algorithmic bytes %d" % (dk, j1["roofline_decode"]["algorithmic_bytes"]))
    open(os.path.join(out, "hbm_traffic_%s.txt" % tag), "w").write("\n".join(t) + "\n")

    # ------------------------------------------------------------------ SQ counters
    A, B = _counters(os.path.join(out, "pmc3")), _counters(os.path.join(out, "pmc4"))
    s = ["# Shader-engine counters per launch (rocprofv3 --pmc): bench.py %s" % bench_args, "",
         "Workload: %s" % j1["config"]["workload"], "",
         "Commands (from /tmp with TMPDIR=/tmp, repository root in $R), eight SQ counters per run:", "",
         "    rocprofv3 --pmc SQ_WAVES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_INSTS_VALU SQ_INSTS_MFMA SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_INSTS_VMEM \\",
         "        -d $R/gpurun_out/prof_%s/pmc3 -o run -- %s --eager --steps 2 --warmup 1 %s" % (tag, root_cmd, bench_args),
         "    rocprofv3 --pmc SQ_ACTIVE_INST_ANY SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS SQ_ACTIVE_INST_VMEM SQ_WAIT_ANY SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS SQ_INSTS_LDS \\",
         "        -d $R/gpurun_out/prof_%s/pmc4 -o run -- %s --eager --steps 2 --warmup 1 %s" % (tag, root_cmd, bench_args), "",
         "Values are sums over the chip per dispatch, averaged over the dispatches of the run.  SQ_BUSY_CYCLES counts per",
         "shader engine (32 of them), the wave-level cycle counters (SQ_WAVE_CYCLES, SQ_ACTIVE_*, SQ_WAIT_*) count in units",
         "of four clocks per resident wavefront, SQ_VALU_MFMA_BUSY_CYCLES counts busy clocks of the matrix pipes summed",
         "over the SIMDs (1024 of them).", ""]
    kernels = sorted({k for (k, c) in list(A) + list(B) if k.startswith("sc::")})
    for k in kernels:
        a = {c: v for (kk, c), (n, v) in A.items() if kk == k}
        b = {c: v for (kk, c), (n, v) in B.items() if kk == k}
        n = max([n for (kk, c), (n, v) in list(A.items()) + list(B.items()) if kk == k] or [0])
        s.append("## `%s` (%d dispatches)" % (k, n))
        s.append("")
        for c, v in sorted(a.items()) + sorted(b.items()):
            s.append("    %-32s %16.1f" % (c, v))
        derived = []
        if a.get("SQ_BUSY_CYCLES") and a.get("SQ_VALU_MFMA_BUSY_CYCLES") is not None:
            # busy clocks of the kernel = SQ_BUSY_CYCLES / 32 engines; matrix-pipe utilisation = busy pipe clocks / (1024 SIMDs x kernel clocks)
            clocks = a["SQ_BUSY_CYCLES"] / 32.0
            derived.append("matrix-core utilisation = SQ_VALU_MFMA_BUSY_CYCLES / (1024 SIMDs x SQ_BUSY_CYCLES / 32) = %.3f" % (a["SQ_VALU_MFMA_BUSY_CYCLES"] / (1024.0 * clocks)))
            if a.get("SQ_WAVE_CYCLES"):
                derived.append("resident wavefronts on average = 4 x SQ_WAVE_CYCLES / kernel clocks = %.0f" % (4.0 * a["SQ_WAVE_CYCLES"] / clocks))
        if a.get("SQ_WAVE_CYCLES") and b.get("SQ_ACTIVE_INST_ANY") is not None:
            derived.append("share of wavefront time issuing = SQ_ACTIVE_INST_ANY / SQ_WAVE_CYCLES = %.2f; waiting (SQ_WAIT_ANY / SQ_WAVE_CYCLES) = %.2f; "
                           "waiting for an instruction to issue (SQ_WAIT_INST_ANY) = %.2f"
                           % (b["SQ_ACTIVE_INST_ANY"] / a["SQ_WAVE_CYCLES"], b.get("SQ_WAIT_ANY", 0.0) / a["SQ_WAVE_CYCLES"], b.get("SQ_WAIT_INST_ANY", 0.0) / a["SQ_WAVE_CYCLES"]))
        for dline in derived:
            s.append("    -> " + dline)
        s.append("")
    open(os.path.join(out, "%s_sq_counters.md" % tag), "w").write("\n".join(s) + "\n")
    print("wrote", out)


def bench_args_tau(argv, j):
    if "--tau" in argv:
        return argv[argv.index("--tau") + 1]
    w = j["config"]["workload"]
    return w.split("tau=")[1].split(",")[0]


if __name__ == "__main__":
    main()

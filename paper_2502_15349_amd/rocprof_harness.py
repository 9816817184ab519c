"""rocprofv3 harness: one command that profiles a bench.py run and reports, per kernel, the launch
durations, the matrix-pipe (MFMA) busy fraction, the HBM traffic and GB/s, and the flop cross-check.

    python bench.py --profile [--workload NAME | --backward --only S | --recurrent --only S] [--profile-dir DIR]

This module never touches the GPU itself: it starts `rocprofv3 ... -- python3 bench.py <args>` child
processes, one per pass (rocprofv3 does not split counters over passes, and trace and counter collection do
not share a run), parses the CSV files they leave and writes a text summary:

  pass 1  --kernel-trace --stats            calls and average / min / max duration per kernel
  pass 2  --pmc FETCH_SIZE                  bytes read from HBM per dispatch   (counter units)
  pass 3  --pmc WRITE_SIZE                  bytes written to HBM per dispatch  (counter units)
  pass 4,5  the same two counters for a plain device copy of 1 GiB (`bench.py --calib-copy 1024`):
          the size of a counter unit in bytes on this machine (documented as KiB, measured otherwise)
  pass 6  --pmc SQ_* GRBM_GUI_ACTIVE        MFMA busy cycles, MFMA operations, vector / LDS instruction
                                            counts, LDS bank conflicts, active cycles

Derived figures per kernel: MFMA busy fraction = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE / 8 XCDs x
1024 SIMDs); issued MFMA flop = SQ_INSTS_VALU_MFMA_MOPS_BF16 x 512; shader clock = GRBM_GUI_ACTIVE / 8 /
duration; HBM GB/s = (fetch + write bytes) / average duration; vector instructions per 32x32x16 MFMA.
The summary ends with a machine-readable line per kernel,
    traffic_bytes_per_launch <kernel> fetch=<bytes> write=<bytes>
which bench.py reads back (from the tracked copy under profiles/) for `roofline.traffic`.
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import re
import subprocess
import sys
import time

SQ_COUNTERS = ["SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CU_CYCLES", "SQ_INSTS_VALU_MFMA_MOPS_BF16", "GRBM_GUI_ACTIVE",
               "SQ_LDS_BANK_CONFLICT", "SQ_LDS_IDX_ACTIVE", "SQ_INSTS_LDS", "SQ_INSTS_VALU"]
# kernels of this library (everything else in a trace -- torch's fills and copies -- is listed but not analysed)
OURS = ("attn_fwd_kernel", "attn_bwd_kernel", "attn_bwd_delta_kernel", "attn_merge_kernel", "rec_state_kernel", "rec_step_kernel",
        "rec_scan_kernel", "rec_fused_kernel", "gated_", "calib_mfma_kernel")
N_XCD, N_SIMD = 8, 1024
GIB = 1 << 30


def short_name(kernel: str) -> str:
    """A compact, stable name for a kernel symbol (template arguments kept, namespaces and argument lists dropped)."""
    k = re.sub(r"\(anonymous namespace\)::", "", kernel)
    k = re.sub(r"^void\s+", "", k)
    k = re.sub(r"\(.*\)$", "", k).strip()
    k = k.replace("ae::", "").replace(" ", "")
    return k


def _is_ours(kernel: str) -> bool:
    return any(t in kernel for t in OURS)


def _run(cmd, log, limit_s):
    print(f"[profile] {' '.join(cmd)}", flush=True)
    t0 = time.time()
    with open(log, "w") as f:
        r = subprocess.run(cmd, stdout=f, stderr=subprocess.STDOUT, cwd="/tmp", env=dict(os.environ, TMPDIR="/tmp"),
                           timeout=limit_s)
    print(f"[profile]   -> exit {r.returncode} after {time.time() - t0:.0f} s", flush=True)
    if r.returncode != 0:
        tail = "".join(open(log).readlines()[-25:])
        raise RuntimeError(f"profiling pass failed ({' '.join(cmd)}):\n{tail}")


def _find(out_dir, pattern):
    hits = sorted(glob.glob(os.path.join(out_dir, "**", pattern), recursive=True))
    if not hits:
        raise RuntimeError(f"no {pattern} under {out_dir}")
    return hits[-1]


def _pmc_means(out_dir):
    """{kernel: {counter: (mean per dispatch, dispatches)}} of one --pmc pass."""
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(_find(out_dir, "*counter_collection.csv"))):
        agg[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: {c: (sum(v) / len(v), len(v)) for c, v in d.items()} for k, d in agg.items()}


def profile(bench_py: str, child_args: list, out_dir: str, name: str, trace_args=("--steps", "50", "--warmup", "10"),
            pmc_args=("--steps", "3", "--warmup", "1"), rocprof: str = "rocprofv3") -> str:
    """Runs the passes and returns the path of the summary it wrote (out_dir/<name>.txt)."""
    os.makedirs(out_dir, exist_ok=True)
    raw = os.path.join(out_dir, name + "_raw")
    os.makedirs(raw, exist_ok=True)
    py = [sys.executable, bench_py]
    cmds = []

    def rp(tag, opts, args, limit):
        d = os.path.join(raw, tag)
        cmd = [rocprof, *opts, "-d", d, "-o", tag, "--output-format", "csv", "--", *py, *args]
        cmds.append(" ".join(cmd).replace(out_dir, "$OUT").replace(bench_py, "$R/bench.py").replace(sys.executable, "python3"))
        _run(cmd, os.path.join(raw, tag + ".log"), limit)
        return d

    d_trace = rp("trace", ["--kernel-trace", "--stats"], [*child_args, *trace_args], 600)
    d_pmc = {}
    for c in ("FETCH_SIZE", "WRITE_SIZE"):
        d_pmc[c] = rp(c.lower(), ["--pmc", c], [*child_args, *pmc_args], 300)
        d_pmc["copy_" + c] = rp("copy_" + c.lower(), ["--pmc", c], ["--calib-copy", "1024"], 300)
    d_sq = rp("sq", ["--pmc", *SQ_COUNTERS], [*child_args, *pmc_args], 300)

    L = [f"# rocprofv3 summary: {name}",
         f"# made by: python3 bench.py --profile {' '.join(child_args)}   (paper_2502_15349_amd/rocprof_harness.py), which ran,",
         "# from /tmp with TMPDIR=/tmp ($R = repository root, $OUT = the output directory):"]
    L += ["#   " + c for c in cmds]
    L += ["# Counters are means per dispatch.  The trace's call counts include the launches bench.py issues while the clock",
          "# settles; a trace of the default mode also holds its 2 s pure-MFMA calibration kernel.",
          "# GRBM_GUI_ACTIVE sums the 8 XCDs: / 8 = shader clocks per launch."]
    stats = list(csv.DictReader(open(_find(d_trace, "*kernel_stats.csv"))))
    L.append("== rocprofv3 --kernel-trace --stats (kernel, calls, avg ns, min ns, max ns, % of traced time)")
    avg_ns = {}
    for r in stats:
        avg_ns[r["Name"]] = float(r["AverageNs"])
        L.append(f"{short_name(r['Name'])[:100]:100s} {r['Calls']:>6s} {float(r['AverageNs']):13.1f} {r['MinNs']:>11s} {r['MaxNs']:>11s} "
                 f"{float(r['Percentage']):6.2f}")
    unit = {}
    L.append("== size of a counter unit, from a plain 1 GiB device copy (reads 1 GiB, writes 1 GiB)")
    for c in ("FETCH_SIZE", "WRITE_SIZE"):
        m = _pmc_means(d_pmc["copy_" + c])
        best = max(((v[c][0], v[c][1], k) for k, v in m.items() if c in v), default=None)   # the copy kernel moves the most
        if best is None or best[0] <= 0:
            raise RuntimeError(f"no {c} reading for the copy kernel")
        unit[c] = GIB / best[0]
        L.append(f"{c}: copy kernel {short_name(best[2])[:60]} reads {best[0]:.1f} (n={best[1]}) -> {unit[c]:.1f} bytes per unit")
    fetch, write, sq = _pmc_means(d_pmc["FETCH_SIZE"]), _pmc_means(d_pmc["WRITE_SIZE"]), _pmc_means(d_sq)
    tail = []
    for k in sorted(set(fetch) | set(write) | set(sq)):
        if not _is_ours(k):
            continue
        sn = short_name(k)
        L.append(f"== {sn}")
        ns = avg_ns.get(k)
        if ns:
            L.append(f"   average duration (trace pass): {ns / 1e3:.1f} us")
        fb = wb = None
        if k in fetch and "FETCH_SIZE" in fetch[k]:
            v, n = fetch[k]["FETCH_SIZE"]
            fb = v * unit["FETCH_SIZE"]
            L.append(f"   FETCH_SIZE {v:.1f} (n={n}) = {fb / 1e6:.1f} MB read from HBM per launch")
        if k in write and "WRITE_SIZE" in write[k]:
            v, n = write[k]["WRITE_SIZE"]
            wb = v * unit["WRITE_SIZE"]
            L.append(f"   WRITE_SIZE {v:.1f} (n={n}) = {wb / 1e6:.1f} MB written to HBM per launch")
        if fb is not None and wb is not None:
            if ns:
                L.append(f"   HBM traffic {(fb + wb) / 1e6:.1f} MB per launch = {(fb + wb) / ns:.1f} GB/s over the average duration")
            tail.append(f"traffic_bytes_per_launch {sn} fetch={fb:.0f} write={wb:.0f}")
        m = {c: v[0] for c, v in sq.get(k, {}).items()}
        for c in sorted(m):
            L.append(f"   {c}: {m[c]:.1f}")
        if m.get("GRBM_GUI_ACTIVE") and "SQ_VALU_MFMA_BUSY_CYCLES" in m:
            cyc = m["GRBM_GUI_ACTIVE"] / N_XCD
            L.append(f"   MFMA busy fraction = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE / {N_XCD} x {N_SIMD} SIMDs) = "
                     f"{m['SQ_VALU_MFMA_BUSY_CYCLES'] / (cyc * N_SIMD):.3f}")
            if ns:
                L.append(f"   shader clock under this kernel = GRBM_GUI_ACTIVE / {N_XCD} / duration = {cyc / ns:.2f} GHz "
                         "(the counter pass's launches; the nominal peak assumes 2.4)")
        if m.get("SQ_INSTS_VALU_MFMA_MOPS_BF16"):
            flop = m["SQ_INSTS_VALU_MFMA_MOPS_BF16"] * 512
            L.append(f"   issued MFMA flop = SQ_INSTS_VALU_MFMA_MOPS_BF16 x 512 = {flop:.4e}" +
                     (f" = {flop / ns / 1e3:.1f} TFLOP/s over the average duration" if ns else ""))
            n_mfma = flop / 32768.0   # one v_mfma_f32_32x32x16_bf16 per wavefront = 32768 flop
            if m.get("SQ_INSTS_VALU"):
                L.append(f"   vector instructions per 32x32x16 MFMA = {m['SQ_INSTS_VALU'] / n_mfma:.2f}; LDS instructions per MFMA = "
                         f"{m.get('SQ_INSTS_LDS', 0.0) / n_mfma:.2f}")
        if m.get("SQ_LDS_IDX_ACTIVE"):
            L.append(f"   LDS bank conflict cycles / LDS active cycles = {m.get('SQ_LDS_BANK_CONFLICT', 0.0) / m['SQ_LDS_IDX_ACTIVE']:.4f}")
    L.append("== bench.py output of the traced run")
    for line in open(os.path.join(raw, "trace.log")):
        if line.startswith("{") or line.startswith("# "):
            L.append(line.rstrip()[:3000])
    L.append("== machine-readable")
    L += tail
    path = os.path.join(out_dir, name + ".txt")
    with open(path, "w") as f:
        f.write("\n".join(L) + "\n")
    print("\n".join(L))
    return path


def read_traffic(summary_path: str, kernel_substr: str):
    """(fetch bytes, write bytes) per launch of the first kernel whose name contains kernel_substr, from a summary
    written by profile(); None if the file or the line is missing."""
    try:
        for line in open(summary_path):
            m = re.match(r"traffic_bytes_per_launch (\S+) fetch=(\d+) write=(\d+)", line)
            if m and kernel_substr in m.group(1):
                return int(m.group(2)), int(m.group(3))
    except OSError:
        pass
    return None

"""rocprofv3 summaries of bench.py, written as short text files under profiles/.

    python -m paper_2604_10103_amd.profile_summary [--workload step_832x480] [--out profiles] [--scratch gpurun_out/prof]

Three runs of the same bench command (counters are collected in runs of their own):
  1. --kernel-trace --stats                       -> <out>/bench_<workload>_kernel_trace.txt
  2. --pmc FETCH_SIZE, 3. --pmc WRITE_SIZE        -> <out>/bench_<workload>_hbm_traffic.txt
     (KiB per dispatch, scaled by what the same counter reads for a plain device copy of known size that
      bench.py runs on request)
  4. two --pmc passes of SQ counters              -> <out>/bench_<workload>_sq_counters.txt
Each file starts with the commands that made it and ends with `key=value` lines that bench.py reads back
(`a4_avg_us`, `a4_hbm_bytes_per_launch`): the figures in the benchmark's JSON line then come from the profile
of the code as it stands, not from constants kept by hand.  Raw profiler output stays in the scratch folder.

This module starts the profiler as a child process and never touches the GPU itself.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import re
import os
import shutil
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_MIB = 256


def short(name: str) -> str:
    name = name.replace("void ", "").replace("hf::(anonymous namespace)::", "hf::")
    return name.split("(")[0][:70]


def run(cmd, log):
    with open(log, "w") as f:
        r = subprocess.run(cmd, stdout=f, stderr=subprocess.STDOUT, cwd=ROOT)
    if r.returncode != 0:
        sys.stderr.write(open(log).read()[-3000:])
        raise SystemExit(f"failed: {' '.join(cmd)}")


def newest(pattern):
    files = sorted(glob.glob(pattern, recursive=True), key=os.path.getmtime)
    if not files:
        raise SystemExit(f"no profiler output matches {pattern}")
    return files[-1]


def counters(folder, names):
    """{kernel: {counter: [values per dispatch]}} from a --pmc run."""
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(newest(os.path.join(folder, "**", "*counter_collection.csv")))):
        if r["Counter_Name"] in names:
            agg[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return agg


def is_attention(name):   # the forward kernels of Eq. 5 (not the backward pass's)
    return "attn_" in name and "bwd" not in name


def main():
    p = argparse.ArgumentParser()
    p.add_argument("--workload", default="step_832x480")
    p.add_argument("--out", default=os.path.join(ROOT, "profiles"))
    p.add_argument("--scratch", default=os.path.join(ROOT, "gpurun_out", "prof"))
    p.add_argument("--skip-sq", action="store_true")
    a = p.parse_args()
    rocprof = shutil.which("rocprofv3") or "/opt/rocm/bin/rocprofv3"
    os.makedirs(a.out, exist_ok=True)
    os.makedirs(a.scratch, exist_ok=True)
    os.environ.setdefault("TMPDIR", "/tmp")
    tag = f"bench_{a.workload}"
    bench = ["python3", "bench.py", "--workload", a.workload, "--no-cpu-baseline", "--no-extras"]

    # ---- 1. kernel trace of the default timed run (HIP graphs), dense comparator left out (it shares the kernel's name)
    d = os.path.join(a.scratch, "kt")
    shutil.rmtree(d, ignore_errors=True)
    cmd1 = [rocprof, "--kernel-trace", "--stats", "-d", d, "-o", "kt", "--output-format", "csv", "--"] + bench + ["--no-dense"]
    run(cmd1, os.path.join(a.scratch, "kt.log"))
    rows = list(csv.DictReader(open(newest(os.path.join(d, "**", "*kernel_stats.csv")))))
    lines = ["# " + " ".join(cmd1).replace(ROOT + "/", ""), "# (bench.py launches the step as HIP graphs; times are per kernel launch)", ""]
    best = None
    for r in rows:
        n = short(r["Name"])
        lines.append(f"{n:62s} calls {int(r['Calls']):5d}  avg {float(r['AverageNs']) / 1e3:9.2f} us  min {float(r['MinNs']) / 1e3:9.2f} us"
                     f"  max {float(r['MaxNs']) / 1e3:9.2f} us  {float(r['Percentage']):6.2f} %")
        if is_attention(n) and (best is None or float(r["TotalDurationNs"]) > float(best["TotalDurationNs"])):
            best = r
    # bench.py's roofline times the launch without a history term (state = NULL): where the kernel has an instance
    # of its own for that (template arguments <.., 0, 0>: no history term, list given), that instance is the one to compare with; the timed step's
    # launches carry the history epilogue and are listed above as well
    plain = [r for r in rows if re.search(r"attn_mfma_kernel<\d+, 0, 0>$", short(r["Name"]))]
    if plain:
        best = max(plain, key=lambda r: float(r["TotalDurationNs"]))
    lines += ["", f"a4_kernel={short(best['Name'])}", f"a4_avg_us={float(best['AverageNs']) / 1e3:.3f}"]
    open(os.path.join(a.out, tag + "_kernel_trace.txt"), "w").write("\n".join(lines) + "\n")

    # ---- 2./3. HBM-side bytes: FETCH_SIZE and WRITE_SIZE in runs of their own, eager launches, calibration copy
    res = {}
    cmds = []
    for ctr in ("FETCH_SIZE", "WRITE_SIZE"):
        d = os.path.join(a.scratch, ctr.lower())
        shutil.rmtree(d, ignore_errors=True)
        cmd = [rocprof, "--pmc", ctr, "-d", d, "-o", "p", "--output-format", "csv", "--"] + bench + [
            "--eager", "--steps", "6", "--warmup", "2", "--no-backward", "--calibration-copy-mib", str(COPY_MIB)]
        cmds.append(cmd)
        run(cmd, os.path.join(a.scratch, ctr.lower() + ".log"))
        res[ctr] = counters(d, {ctr})
    lines = ["# " + " ".join(c).replace(ROOT + "/", "") for c in cmds]
    lines += ["# KiB per dispatch as the counters read; `scaled MB` = value x (bytes of the calibration copy / what the",
              f"# same counter reads for it): a plain device copy of {COPY_MIB} MiB reads and writes {COPY_MIB} MiB.", ""]
    scale = {}
    for ctr in ("FETCH_SIZE", "WRITE_SIZE"):
        copies = [(k, v[ctr]) for k, v in res[ctr].items() if "copy" in k.lower() or "Copy" in k]
        # the calibration copy is the dispatch with the largest reading among copy kernels
        val = max((max(v) for _, v in copies), default=None)
        scale[ctr] = (COPY_MIB * 1024.0 / val) if val else 1.0
        lines.append(f"{ctr}: calibration copy reads {val} KiB for {COPY_MIB * 1024} KiB moved -> factor {scale[ctr]:.4f}")
    lines.append("")
    a4_bytes = None
    for k in sorted(set(res["FETCH_SIZE"]) | set(res["WRITE_SIZE"])):
        f = res["FETCH_SIZE"].get(k, {}).get("FETCH_SIZE", [])
        w = res["WRITE_SIZE"].get(k, {}).get("WRITE_SIZE", [])
        fm = sum(f) / len(f) * scale["FETCH_SIZE"] * 1024 / 1e6 if f else 0.0
        wm = sum(w) / len(w) * scale["WRITE_SIZE"] * 1024 / 1e6 if w else 0.0
        lines.append(f"{k:62s} n {max(len(f), len(w)):4d}  fetch {fm:9.2f} MB  write {wm:9.2f} MB  total {fm + wm:9.2f} MB (scaled, per launch)")
        if k == short(best["Name"]):
            a4_bytes = (fm + wm) * 1e6
    lines += ["", f"a4_kernel={short(best['Name'])}", f"a4_hbm_bytes_per_launch={a4_bytes if a4_bytes is not None else 'nan'}"]
    open(os.path.join(a.out, tag + "_hbm_traffic.txt"), "w").write("\n".join(lines) + "\n")

    # ---- 4. SQ counters (instruction mix, waits, matrix-pipe busy share) of the attention kernel
    if not a.skip_sq:
        passes = ["SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS SQ_INSTS_MFMA SQ_INSTS_VMEM_RD SQ_WAVE_CYCLES SQ_BUSY_CU_CYCLES SQ_VALU_MFMA_BUSY_CYCLES",
                  "SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS SQ_ACTIVE_INST_ANY SQ_WAIT_ANY SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS SQ_ACTIVE_INST_SCA SQ_ACTIVE_INST_VMEM"]
        lines, merged = [], collections.defaultdict(dict)
        for i, ps in enumerate(passes):
            d = os.path.join(a.scratch, f"sq{i}")
            shutil.rmtree(d, ignore_errors=True)
            cmd = [rocprof, "--pmc"] + ps.split() + ["-d", d, "-o", "p", "--output-format", "csv", "--"] + bench + [
                "--eager", "--steps", "6", "--warmup", "2", "--no-backward", "--no-dense"]
            run(cmd, os.path.join(a.scratch, f"sq{i}.log"))
            lines.append("# " + " ".join(cmd).replace(ROOT + "/", ""))
            for k, v in counters(d, set(ps.split())).items():
                for c, vals in v.items():
                    merged[k][c] = sum(vals) / len(vals)
        lines += ["# means per dispatch, summed over the chip; *_CYCLES of SQ_WAVE / SQ_ACTIVE / SQ_WAIT count quad-cycles", ""]
        for k in sorted(merged):
            if not is_attention(k):
                continue
            lines.append(k)
            for c in sorted(merged[k]):
                lines.append(f"   {c:28s} {merged[k][c]:16.1f}")
            m = merged[k]
            if "SQ_VALU_MFMA_BUSY_CYCLES" in m and "SQ_BUSY_CU_CYCLES" in m and m["SQ_BUSY_CU_CYCLES"] > 0:
                # four matrix pipes per compute unit
                lines.append(f"   matrix pipes busy / compute-unit busy = {m['SQ_VALU_MFMA_BUSY_CYCLES'] / (4.0 * m['SQ_BUSY_CU_CYCLES']):.3f}")
            if "SQ_INSTS_MFMA" in m and m["SQ_INSTS_MFMA"] > 0:
                lines.append("   per MFMA: " + ", ".join(f"{c[9:].lower()} {m[c] / m['SQ_INSTS_MFMA']:.2f}" for c in
                                                      ("SQ_INSTS_VALU", "SQ_INSTS_SALU", "SQ_INSTS_LDS") if c in m))
            lines.append("")
        open(os.path.join(a.out, tag + "_sq_counters.txt"), "w").write("\n".join(lines) + "\n")
    print("wrote", ", ".join(sorted(f for f in os.listdir(a.out) if f.startswith(tag))))


if __name__ == "__main__":
    main()

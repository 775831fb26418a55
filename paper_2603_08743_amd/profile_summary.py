"""Turn raw rocprofv3 output (a scratch directory of CSV files) into the short summaries kept under profiles/.

    python -m paper_2603_08743_amd.profile_summary traffic --tables T --slab-layers N --fetch DIR --write DIR --name cfg2 --command "..."
    python -m paper_2603_08743_amd.profile_summary sq      --a DIR --b DIR --name cfg2 --command "..."
    python -m paper_2603_08743_amd.profile_summary stats   --csv FILE --bench-log FILE --name cfg2 --command "..."
    python -m paper_2603_08743_amd.profile_summary resources          (no GPU: compiles the kernels and records the compiler's resource remarks)

`traffic` also records the scaled HBM bytes per launch in profiles/traffic.json together with a hash of the kernel
sources; bench.py reports that figure as roofline.traffic only while the sources still hash to the same value.
"""
from __future__ import annotations

import argparse
import csv
import datetime
import glob
import hashlib
import json
import os
import subprocess

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
PROFILES = os.path.join(ROOT, "profiles")
TRAFFIC_JSON = os.path.join(PROFILES, "traffic.json")


def source_sha() -> str:
    """Hash of every kernel and API source the library is built from (the counter driver and the unbuilt split kernel excluded)."""
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(HERE, "csrc", "*"))):
        if f.endswith((".h", ".hip")) and not f.endswith("zp_prof_driver.hip") and not os.path.basename(f).startswith("zp_split"):   # what the library is built from
            h.update(os.path.basename(f).encode())
            h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def git_head() -> str:
    try:
        return subprocess.run(["git", "-C", ROOT, "rev-parse", "--short=12", "HEAD"], capture_output=True, text=True, timeout=10).stdout.strip()
    except Exception:
        return ""


def counter_rows(d: str):
    out = []
    for f in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
        out += list(csv.DictReader(open(f)))
    return out


def short(name: str) -> str:
    name = name.replace("void ", "").replace("zp::", "")
    return name.split("(")[0]


def read_tables_header(path: str):
    hd = np.fromfile(path, dtype=np.int32, count=16)
    keys = ("magic", "cfg", "seed", "B", "max_blocks", "N_max", "L", "h_kv", "h_q", "d", "b", "w", "N_total", "M", "has_keep", "has_dst")
    return dict(zip(keys, (int(x) for x in hd)))


def cmd_traffic(a):
    hd = read_tables_header(a.tables)
    Ls = a.slab_layers or hd["L"]
    copy_bytes = Ls * hd["N_total"] * hd["b"] * hd["h_kv"] * hd["d"] * 2
    strided_bytes = Ls * hd["N_total"] * hd["b"] * hd["d"] * 2
    per = {}
    lines = []
    for d, c in ((a.fetch, "FETCH_SIZE"), (a.write, "WRITE_SIZE")):
        for r in counter_rows(d):
            if r["Counter_Name"] != c:
                continue
            n = short(r["Kernel_Name"])
            if not (n.startswith("unit_") or n in ("plain_copy", "strided_read")):
                continue
            raw = float(r["Counter_Value"]) * 1024.0
            ms = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6
            per.setdefault((n, c), []).append((raw, ms))
            lines.append("%s | %s | %.3f | %.3f | %s | %s | %s" % (n, c, raw / 1e9, ms, r["VGPR_Count"], r["LDS_Block_Size"], r["Scratch_Size"]))
    mean = lambda k: float(np.mean([x[0] for x in per[k]]))
    f_copy, w_copy = copy_bytes / mean(("plain_copy", "FETCH_SIZE")), copy_bytes / mean(("plain_copy", "WRITE_SIZE"))
    f_str = strided_bytes / mean(("strided_read", "FETCH_SIZE"))
    unit = sorted({k[0] for k in per if k[0].startswith("unit_")})
    assert len(unit) == 1, unit
    fetch, write = mean((unit[0], "FETCH_SIZE")) * f_copy, mean((unit[0], "WRITE_SIZE")) * w_copy
    ms = float(np.mean([x[1] for x in per[(unit[0], "FETCH_SIZE")] + per[(unit[0], "WRITE_SIZE")]]))
    units = hd["B"] * Ls * hd["h_kv"]
    md = ["# HBM-side traffic of the fused kernel, %s (B=%d, %d layers per launch, %d units), MI355X" % (a.name, hd["B"], Ls, units),
          "Commands (TMPDIR=/tmp; zp_prof_driver and the tables file come from paper_2603_08743_amd/build.py and dump_workload.py):"]
    md += ["  " + c for c in a.command]
    md += ["", "FETCH_SIZE / WRITE_SIZE are KiB per dispatch (shown in GB = 1e9 bytes); they count what the L2 requests from / sends to the",
           "fabric, so reads served by the Infinity Cache are included.", "",
           "Kernel | counter | raw GB | duration ms | VGPRs | LDS bytes | scratch bytes", "---|---|---|---|---|---|---"] + lines
    md += ["", "Calibration against dispatches of known size: plain_copy reads and writes %.3f GB (contiguous), strided_read fetches %.3f GB" % (copy_bytes / 1e9, strided_bytes / 1e9),
           "(256-byte pieces of one kv head at the token stride, 16 bytes per lane: the kernel's own read pattern).",
           "  FETCH_SIZE factor: contiguous %.3f, strided %.3f.  WRITE_SIZE factor: %.3f." % (f_copy, f_str, w_copy),
           "%s, scaled with the contiguous factors: fetch %.2f GB + write %.2f GB = %.2f GB per launch (%.3f ms under the counters => %.2f TB/s)." %
           (unit[0], fetch / 1e9, write / 1e9, (fetch + write) / 1e9, ms, (fetch + write) / ms / 1e9)]
    os.makedirs(PROFILES, exist_ok=True)
    path = os.path.join(PROFILES, "unit_mfma_%s_hbm_traffic.md" % a.name)
    open(path, "w").write("\n".join(md) + "\n")
    entries = json.load(open(TRAFFIC_JSON)) if os.path.exists(TRAFFIC_JSON) else []
    entries = [e for e in entries if not (e["name"] == a.name)]
    entries.append({"name": a.name, "config": hd["cfg"], "B": hd["B"], "slab_layers": Ls, "kernel": unit[0], "traffic_bytes": fetch + write,
                    "fetch_bytes": fetch, "write_bytes": write, "fetch_factor_contiguous": f_copy, "fetch_factor_strided": f_str,
                    "write_factor": w_copy, "ms_under_counters": ms, "source_sha": source_sha(), "head": git_head(),
                    "date": datetime.date.today().isoformat(), "summary": os.path.relpath(path, ROOT)})
    json.dump(sorted(entries, key=lambda e: e["name"]), open(TRAFFIC_JSON, "w"), indent=1)
    print("\n".join(md[-5:]))


def cmd_sq(a):
    v = {}
    kernel = None
    for d in (a.a, a.b):
        for r in counter_rows(d):
            n = short(r["Kernel_Name"])
            if n.startswith("unit_"):
                kernel = n
                v.setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
                regs = (r["VGPR_Count"], r["Accum_VGPR_Count"], r["LDS_Block_Size"], r["Scratch_Size"])
    v = {k: x[-1] for k, x in v.items()}                      # the last dispatch of each run
    md = ["# SQ counters of the fused kernel, %s, MI355X" % a.name, "Commands (TMPDIR=/tmp; one counter set per run; the last dispatch of each run is shown):"]
    md += ["  " + c for c in a.command]
    md += ["", "Kernel: %s (VGPRs %s, AGPRs %s, LDS %s bytes, scratch %s bytes)" % ((kernel,) + regs), "", "Counter | value", "---|---"]
    md += ["%s | %.4g" % (k, x) for k, x in sorted(v.items())]
    if "SQ_BUSY_CYCLES" in v and "SQ_WAVES" in v:
        cyc = v["SQ_BUSY_CYCLES"] / 32.0                          # 32 shader engines' worth of counters on this chip
        md += ["", "Derived (1024 SIMDs; SQ_BUSY_CYCLES / 32 = %.3g cycles of the launch):" % cyc]
        w = v["SQ_WAVES"]
        if "SQ_INSTS_VALU" in v:
            md.append("  per wave: %.0f vector ALU, %.0f matrix-core, %.0f transcendental instructions" %
                      (v["SQ_INSTS_VALU"] / w, v.get("SQ_INSTS_MFMA", 0) / w, v.get("SQ_INSTS_VALU_TRANS_F32", 0) / w))
        if "SQ_ACTIVE_INST_VALU" in v:
            md.append("  vector ALU busy %.1f %% of the SIMD cycles (SQ_ACTIVE_INST_VALU x 4 / (cycles x 1024))" % (100 * v["SQ_ACTIVE_INST_VALU"] * 4 / (cyc * 1024)))
        if "SQ_VALU_MFMA_BUSY_CYCLES" in v:
            md.append("  matrix cores busy %.1f %% (SQ_VALU_MFMA_BUSY_CYCLES / (cycles x 1024))" % (100 * v["SQ_VALU_MFMA_BUSY_CYCLES"] / (cyc * 1024)))
        if "SQ_WAVE_CYCLES" in v:
            md.append("  resident waves per SIMD %.2f (SQ_WAVE_CYCLES x 4 / (cycles x 1024))" % (v["SQ_WAVE_CYCLES"] * 4 / (cyc * 1024)))
            if "SQ_WAIT_ANY" in v:
                md.append("  waiting %.0f %% of the wave cycles (SQ_WAIT_ANY / SQ_WAVE_CYCLES)" % (100 * v["SQ_WAIT_ANY"] / v["SQ_WAVE_CYCLES"]))
        if "SQ_LDS_BANK_CONFLICT" in v and "SQ_ACTIVE_INST_LDS" in v:
            md.append("  LDS bank-conflict cycles %.0f %% of the LDS-active cycles" % (100 * v["SQ_LDS_BANK_CONFLICT"] / v["SQ_ACTIVE_INST_LDS"]))
    path = os.path.join(PROFILES, "unit_mfma_%s_sq_counters.md" % a.name)
    open(path, "w").write("\n".join(md) + "\n")
    print("\n".join(md[-9:]))


def cmd_stats(a):
    rows = list(csv.DictReader(open(a.csv)))
    j = None
    if a.bench_log:
        cand = [l for l in open(a.bench_log) if l.startswith("{")]
        j = json.loads(cand[-1]) if cand else None
    md = ["# rocprofv3 kernel stats - %s, MI355X" % a.name, "Command (from the repository root, TMPDIR=/tmp):"]
    md += ["  " + c for c in a.command]
    if j:
        md.append("bench.py's own line for the same run: ms_per_step %.2f (%d launches), ms_per_launch %.3f from HIP events, roofline.frac %.3f." %
                  (j["ms_per_step"], j["config"]["launches_per_step"], j["roofline"]["ms_per_launch"], j["roofline"]["frac"]))
    md += ["", "Name | Calls | AverageNs | MinNs | MaxNs | % of GPU time", "---|---|---|---|---|---"]
    for r in rows:
        if "zp::" in r["Name"]:
            md.append("%s | %s | %s | %s | %s | %s" % (r["Name"][:70], r["Calls"], r["AverageNs"], r["MinNs"], r["MaxNs"], r["Percentage"]))
    md += ["", "Calls of the fused kernel = (warm-up + timed steps) x launches per step + 1 untimed launch with the kept-list output (used for the",
           "algorithmic byte count).  Every other kernel in the trace belongs to the seeded input generator, the pool restore or the checks, outside",
           "the timed region."]
    path = os.path.join(PROFILES, "unit_mfma_%s_kernel_stats.md" % a.name)
    open(path, "w").write("\n".join(md) + "\n")
    print("\n".join(md))


def cmd_resources(a):
    """Registers, spills, scratch and occupancy of every kernel instantiation, from hipcc's own remarks."""
    import re
    from .build import CSRC, FLAGS
    files = ["zp_mfma_d128_wide.hip", "zp_mfma_d128.hip", "zp_mfma_d64_wide.hip", "zp_mfma_d64.hip", "zp_kernels.hip", "zp_check.hip"]
    rows = []
    from concurrent.futures import ThreadPoolExecutor
    compile_one = lambda f: subprocess.run(["hipcc", *FLAGS, "--cuda-device-only", "-Rpass-analysis=kernel-resource-usage", "-c", os.path.join(CSRC, f),
                                            "-o", os.devnull], capture_output=True, text=True)
    with ThreadPoolExecutor(max_workers=len(files)) as ex:
        results = list(ex.map(compile_one, files))
    for f, r in zip(files, results):
        assert r.returncode == 0, r.stderr[-2000:]
        for blk in re.split(r"remark: Function Name: ", r.stderr)[1:]:
            mangled = blk.split()[0]
            name = subprocess.run(["c++filt", mangled], capture_output=True, text=True).stdout.strip() or mangled
            v = dict(re.findall(r"remark:\s+([A-Za-z ]+(?:\[[A-Za-z/ ]*\])?): (\S+)", blk))
            g = lambda k: next((x for kk, x in v.items() if kk.strip().startswith(k)), "?")
            rows.append((f, short(name), g("VGPRs"), g("AGPRs"), g("VGPRs Spill"), g("SGPRs Spill"), g("ScratchSize"), g("Occupancy")))
    md = ["# Compiler resource usage of every kernel instantiation (gfx950)", "Command (no GPU needed):",
          "  python -m paper_2603_08743_amd.profile_summary resources",
          "  (per source file: hipcc <build flags> --cuda-device-only -Rpass-analysis=kernel-resource-usage -c csrc/<file>)", "",
          "unit_mfma<D, RB, NW, G, RED>: head dimension, 32-row query blocks per wave, waves per workgroup, group size (0 = run time), RED = redundancy",
          "taken from the key tiles of sweep 2.  VGPR spills go to scratch memory; SGPR spills go to spare vector-register lanes and cost no memory traffic.", "",
          "File | kernel | VGPRs | AGPRs | VGPR spills | SGPR spills | scratch bytes/lane | waves/SIMD", "---|---|---|---|---|---|---|---"]
    md += ["%s | %s | %s | %s | %s | %s | %s | %s" % r for r in rows]
    used = {"cfg1": "unit_mfma<128, 1, 8, 7, false>", "cfg2 / cfg3": "unit_mfma<128, 1, 8, 4, false>", "cfg2 with redundancy": "unit_mfma<128, 1, 8, 4, true>",
            "cfg4": "unit_mfma<128, 3, 8, 5, false>", "paper geometry": "unit_mfma<128, 1, 2, 4, false>", "cfg0 (fp32)": "unit_generic<0>"}
    md += ["", "Instantiations the benchmark workloads run: " + "; ".join("%s: %s" % kv for kv in used.items()) + "."]
    path = os.path.join(PROFILES, "kernel_resource_usage.md")
    open(path, "w").write("\n".join(md) + "\n")
    want = set(used.values())
    for r in rows:
        if r[1] in want:
            print(" | ".join(r))


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="what", required=True)
    t = sub.add_parser("traffic")
    t.add_argument("--tables", required=True)
    t.add_argument("--slab-layers", type=int, default=0)
    t.add_argument("--fetch", required=True)
    t.add_argument("--write", required=True)
    s = sub.add_parser("sq")
    s.add_argument("--a", required=True)
    s.add_argument("--b", required=True)
    k = sub.add_parser("stats")
    k.add_argument("--csv", required=True)
    k.add_argument("--bench-log", default="")
    sub.add_parser("resources")
    for p in (t, s, k):
        p.add_argument("--name", required=True)
        p.add_argument("--command", action="append", default=[])
    a = ap.parse_args()
    {"traffic": cmd_traffic, "sq": cmd_sq, "stats": cmd_stats, "resources": cmd_resources}[a.what](a)


if __name__ == "__main__":
    main()

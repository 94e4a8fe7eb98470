"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2306_15799_amd.profile_summary trace   <r_kernel_stats.csv> <out.txt> "<command>"
    python -m paper_2306_15799_amd.profile_summary traffic <raw_dir> <workload> [<workload> ...]
    python -m paper_2306_15799_amd.profile_summary pmc     <out.txt> "<command>" <r_counter_collection.csv> [...]

`traffic` reads <raw_dir>/pmc_fetch_<W>/r_counter_collection.csv and
<raw_dir>/pmc_write_<W>/r_counter_collection.csv (one counter per rocprofv3
run, raw_dir relative to the repository root), scales both counters by what they report for a copy of known size in the
same run (torch's fp32 -> bf16 conversion of Q when bench.py uploads the
inputs) and writes profiles/hbm_traffic_<W>.txt plus the machine-readable
profiles/hbm_traffic.json that bench.py reads.  The JSON is stamped with a hash
of the kernel sources it was measured on; bench.py drops the figures when the
sources have changed since.
"""
from __future__ import annotations

import collections
import csv
import hashlib
import json
import os
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)

# kernel name in a rocprofv3 trace (template arguments vary) -> name the library's stage timer uses
TIMER_NAME_RULES = [
    ("gemm_mfma_kernel<ProjPolicy", "gemm_mfma_proj"),
    ("gemm_mfma_pair_kernel", "gemm_mfma_grads"),
    ("gemm_mfma_kernel<GradXPolicy", "gemm_mfma_gradx"),
    ("gemm_mfma_kernel<GradEPolicy", "gemm_mfma_grade"),
    ("proj_finish_kernel", "proj_finish"),
    ("key_state_kernel", "key_state"),
    ("merge_pack_kernel", "merge_pack"),
    ("query_stream_kernel", "query_stream"),
    ("bwd_query_x", "bwd_query_x"),
    ("bwd_query_y_kernel", "bwd_query_y"),
    ("bwd_merge_kernel", "bwd_merge"),
    ("bwd_key_kernel", "bwd_key"),
    ("sum_splits_bf16_kernel", "sum_splits"),
]


def timer_name(trace_name: str):
    for prefix, name in TIMER_NAME_RULES:
        if trace_name.startswith(prefix):
            return name
    return None


def source_hash() -> str:
    """sha256 over the library's sources (csrc/ and the public header), in name order."""
    h = hashlib.sha256()
    files = [os.path.join(PKG_DIR, "csrc", f) for f in sorted(os.listdir(os.path.join(PKG_DIR, "csrc")))]
    files.append(os.path.join(ROOT, "include", "flurka.h"))
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()


def short(name: str) -> str:
    return name.split("(")[0].replace("void ", "").replace("flurka::", "")


def trace(path: str, out: str, cmd: str) -> None:
    rows = list(csv.DictReader(open(path)))
    with open(out, "w") as f:
        f.write("rocprofv3 kernel-trace summary\ncommand (run from the repository root on the GPU box):\n  " + cmd + "\n\n")
        f.write(f"{'kernel':90s} {'calls':>6s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'pct':>6s}\n")
        for r in rows:
            if "flurka" not in r["Name"]:
                continue
            f.write(f"{short(r['Name'])[:90]:90s} {r['Calls']:>6s} {float(r['AverageNs']) / 1e3:10.2f} "
                    f"{float(r['MinNs']) / 1e3:10.2f} {float(r['MaxNs']) / 1e3:10.2f} {float(r['Percentage']):6.2f}\n")
    print(open(out).read())


def traffic(raw_dir, workloads) -> None:
    from paper_2306_15799_amd import inputs
    jpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    out_json = json.load(open(jpath)) if os.path.exists(jpath) else {}
    stamp = source_hash()
    for w in workloads:
        wl = {**inputs.WORKLOADS, **inputs.DERIVED_WORKLOADS}[w]
        vals = {}
        for f in ["fetch", "write"]:
            p = os.path.join(ROOT, raw_dir, f"pmc_{f}_{w}/r_counter_collection.csv")
            d = collections.defaultdict(list)
            for r in csv.DictReader(open(p)):
                d[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
            vals[f] = d
        # calibration: torch's fp32 -> bf16 copy of Q reads 4 B and writes 2 B per element
        copy = [k for k in vals["fetch"] if "bfloat16_copy" in k][0]
        elems = wl.B * wl.H * wl.n * wl.d
        ffac = elems * 4 / 1024 / vals["fetch"][copy][0]
        wfac = elems * 2 / 1024 / vals["write"][copy][0]
        cmd = ("rocprofv3 --pmc {c} --output-format csv -d " + raw_dir.rstrip("/") + "/pmc_{f}_{w} -o r -- python3 bench.py "
               "--workload {w} --steps 3 --warmup 1 --no-cpu-baseline --no-measured-peaks --no-configs")
        lines = [f"HBM traffic per dispatch, workload {w} (rocprofv3 --pmc, KiB per dispatch, mean over dispatches)",
                 "commands (run from the repository root on the GPU box, one counter per run):",
                 "  " + cmd.format(c="FETCH_SIZE", f="fetch", w=w),
                 "  " + cmd.format(c="WRITE_SIZE", f="write", w=w),
                 f"calibration: torch's fp32->bf16 copy of Q ({elems} elements) reads {elems * 4 // 1024} KiB and writes {elems * 2 // 1024} KiB;",
                 f"  FETCH_SIZE reported {vals['fetch'][copy][0]:.0f} -> factor {ffac:.3f}; WRITE_SIZE reported {vals['write'][copy][0]:.0f} -> factor {wfac:.3f}",
                 f"library sources at measurement: sha256 {stamp[:16]}",
                 "", f"{'kernel':50s} {'FETCH_SIZE':>12s} {'WRITE_SIZE':>12s} {'read MiB':>10s} {'write MiB':>10s}"]
        out_json[w] = {"fetch_factor": round(ffac, 3), "write_factor": round(wfac, 3), "source_sha256": stamp,
                       "kernels": {}}
        for k in vals["fetch"]:
            tn = timer_name(k)
            if tn is None:
                continue
            fv = sum(vals["fetch"][k]) / len(vals["fetch"][k])
            wv = sum(vals["write"][k]) / len(vals["write"][k])
            lines.append(f"{k[:50]:50s} {fv:12.0f} {wv:12.0f} {fv * ffac / 1024:10.1f} {wv * wfac / 1024:10.1f}")
            out_json[w]["kernels"][tn] = {"trace_name": k, "read_bytes": int(fv * ffac * 1024),
                                          "write_bytes": int(wv * wfac * 1024)}
        open(os.path.join(ROOT, f"profiles/hbm_traffic_{w}.txt"), "w").write("\n".join(lines) + "\n")
        print("\n".join(lines))
    json.dump(out_json, open(jpath, "w"), indent=1)


def pmc(out: str, cmd: str, paths) -> None:
    """Mean counter values per kernel from one or more rocprofv3 --pmc runs (one run per counter group)."""
    d = collections.defaultdict(lambda: collections.defaultdict(list))
    for path in paths:
        for r in csv.DictReader(open(path)):
            n = short(r["Kernel_Name"])
            if timer_name(n) is None:
                continue
            d[n][r["Counter_Name"]].append(float(r["Counter_Value"]))
    with open(out, "w") as f:
        f.write("rocprofv3 --pmc summary (mean per dispatch)\ncommands (run from the repository root on the GPU box, "
                "one run per counter group):\n")
        for c in cmd.split(";;"):
            f.write("  " + c.strip() + "\n")
        f.write("\n")
        for n, c in d.items():
            f.write(n + "\n")
            for k, v in sorted(c.items()):
                f.write(f"   {k:32s} {sum(v) / len(v):18.1f}   ({len(v)} dispatches)\n")
    print(open(out).read())


if __name__ == "__main__":
    if len(sys.argv) < 2:
        sys.exit(__doc__)
    if sys.argv[1] == "trace":
        trace(*sys.argv[2:5])
    elif sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3:])
    elif sys.argv[1] == "pmc":
        pmc(sys.argv[2], sys.argv[3], sys.argv[4:])
    else:
        sys.exit(__doc__)

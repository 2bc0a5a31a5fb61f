"""Turn rocprofv3 output of `bench.py` runs into the short summaries kept under profiles/.

    python -m paper_2405_01481_amd.profile_summary trace <kernel_stats.csv> [top]
        the --kernel-trace --stats table as markdown rows (calls, total ms, average / min / max us, share)

    python -m paper_2405_01481_amd.profile_summary traffic <fetch counter csv> <write counter csv> <workload> <out.json>
        HBM-side bytes per launch of the kernel classes from two --pmc runs (FETCH_SIZE, WRITE_SIZE; KiB per
        dispatch), each scaled by what the same counter reads for the 1 GiB device copies that
        `bench.py --calib-copy` runs first; merged into <out.json> under the workload's name together with the
        current commit, which is where bench.py takes `roofline.traffic` from.

Reads files only; runs nothing on the GPU.
"""
from __future__ import annotations

import collections
import csv
import json
import os
import re
import subprocess
import sys

# kernel name pattern -> class of bench.py's roofline entries (the LM-head GEMM is the tile kernel with epilogue 5)
CLASSES = {r"gemm_ring_kernel": "gemm_decode", r"attn_decode_kernel": "attn_decode",
           r"gemm_dma8?_kernel<[0-4][,>]": "gemm_prefill", r"gemm_dma8?_kernel<5[,>]": "lmhead_score",
           r"attn_prefill_kernel": "attn_prefill"}


def trace_table(path, top=24):
    rows = list(csv.DictReader(open(path)))
    print("| kernel | calls | total ms | avg us | % | min us | max us |")
    print("|---|---|---|---|---|---|---|")
    for r in rows[:top]:
        name = re.sub(r"\(.*", "", r["Name"])[:64]
        print(f"| {name} | {r['Calls']} | {float(r['TotalDurationNs']) / 1e6:.1f} | {float(r['AverageNs']) / 1e3:.1f} | "
              f"{float(r['Percentage']):.2f} | {float(r['MinNs']) / 1e3:.1f} | {float(r['MaxNs']) / 1e3:.1f} |")


def _per_kernel(path, counter):
    """kernel name (without arguments) -> list of counter values, one per dispatch"""
    per = collections.defaultdict(dict)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        name = re.sub(r"^void ", "", re.sub(r"\(.*", "", r["Kernel_Name"]))
        per[name][r["Dispatch_Id"]] = per[name].get(r["Dispatch_Id"], 0.0) + float(r["Counter_Value"])
    return {k: list(v.values()) for k, v in per.items()}


def traffic(fetch_csv, write_csv, workload, out_json):
    out = {}
    fetch, write = _per_kernel(fetch_csv, "FETCH_SIZE"), _per_kernel(write_csv, "WRITE_SIZE")
    gib_kib = float(1 << 20)

    def scale(per, what):
        copies = [v for k, v in per.items() if "copyBuffer" in k]
        if not copies:
            raise SystemExit(f"no calibration copies in the {what} run (bench.py --calib-copy)")
        first = copies[0][:3]          # --calib-copy runs its three 1 GiB copies before anything else
        return gib_kib / (sum(first) / len(first))
    sf, sw = scale(fetch, "FETCH_SIZE"), scale(write, "WRITE_SIZE")
    res = {}
    for pattern, cls in CLASSES.items():
        f = [x for k, v in fetch.items() if re.match(pattern, k) for x in v]
        w = [x for k, v in write.items() if re.match(pattern, k) for x in v]
        if not f or not w:
            continue
        res[cls] = {"context_dependent": cls.startswith("attn_"),   # per-launch bytes grow with the sequences: only
                    # comparable with a run of the same prompt and generation lengths
                    "bytes_per_launch": (sum(f) / len(f) * sf + sum(w) / len(w) * sw) * 1024.0,
                    "fetch_bytes_per_launch": sum(f) / len(f) * sf * 1024.0,
                    "write_bytes_per_launch": sum(w) / len(w) * sw * 1024.0, "dispatches": len(f)}
    try:
        out = json.load(open(out_json))
    except Exception:
        out = {}
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    try:
        commit = subprocess.run(["git", "-C", root, "rev-parse", "--short", "HEAD"], capture_output=True, text=True).stdout.strip()
    except Exception:
        commit = ""
    out["commit"] = commit or out.get("commit", "")
    out["scale_factors"] = {"FETCH_SIZE": sf, "WRITE_SIZE": sw}
    out[workload] = res
    json.dump(out, open(out_json, "w"), indent=1, sort_keys=True)
    print(json.dumps(out[workload], indent=1))


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "trace":
        trace_table(sys.argv[2], int(sys.argv[3]) if len(sys.argv) > 3 else 24)
    elif len(sys.argv) == 6 and sys.argv[1] == "traffic":
        traffic(*sys.argv[2:])
    else:
        raise SystemExit(__doc__)

"""Turn rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2602_12128_amd.profile_tools stats   <dir-with-*_kernel_stats.csv>
    python -m paper_2602_12128_amd.profile_tools traffic <fetch-dir> <write-dir> <copy-MiB> [out.json]

`traffic` reads two --pmc runs (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch) of
`bench.py --calib-copy-mib M`, takes the per-byte scale of each counter from the calibration copy
(a device-to-device copy of M MiB: M MiB read, M MiB written) and prints scaled HBM bytes per
launch for every kernel of the library; with out.json it also stores them for bench.py.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import re
import sys

_KERNEL = re.compile(r"(k_[a-z_0-9]+|__amd_rocclr_\w+)")

# kernel symbol -> name used by the library's launch records / bench.py
LAUNCH_NAMES = {
    "k_phi_fwd<": "mfma_phi_forward", "k_phi_bwd<": "mfma_phi_backward",
    "k_state<": "mfma_state", "k_query<": "mfma_query", "k_bwd_query<": "mfma_bwd_query",
    "k_bwd_key<": "mfma_bwd_key", "k_reduce<": "mfma_reduce",
    "k_phi_wgrad<128,": "mfma_phi_weight_grads", "k_phi_wgrad<64,": "mfma_phi_weight_grads",
    "k_wgrad_reduce": "phi_weight_grads_reduce",
}


def _short(name: str) -> str:
    """`k_name<template arguments>` out of a demangled symbol (nested brackets kept whole,
    namespaces dropped)."""
    m = _KERNEL.search(name)
    if not m:
        return name[:40]
    end = m.end()
    if name[end:end + 1] == "<":
        depth = 0
        for i in range(end, len(name)):
            depth += {"<": 1, ">": -1}.get(name[i], 0)
            if depth == 0:
                end = i + 1
                break
    return name[m.start():end].replace("hla::mf::", "").replace("hla::", "")


def stats(d: str) -> None:
    path = glob.glob(d + "/*kernel_stats.csv")[0]
    print("| kernel | calls | total us | avg us | % |\n|---|---|---|---|---|")
    for r in csv.DictReader(open(path)):
        print(f"| `{_short(r['Name'])}` | {r['Calls']} | {float(r['TotalDurationNs']) / 1e3:.1f} | "
              f"{float(r['AverageNs']) / 1e3:.2f} | {r['Percentage']} |")


def _per_kernel(d: str, counter: str):
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(glob.glob(d + "/*counter_collection.csv")[0])):
        if r["Counter_Name"] == counter:
            acc[_short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return acc


def traffic(fetch_dir: str, write_dir: str, copy_mib: float, out: str | None) -> None:
    f = _per_kernel(fetch_dir, "FETCH_SIZE")
    w = _per_kernel(write_dir, "WRITE_SIZE")
    # the calibration copy is the largest copyBuffer dispatch of the run
    cf = max(f.get("__amd_rocclr_copyBuffer", [0.0]))
    cw = max(w.get("__amd_rocclr_copyBuffer", [0.0]))
    if cf <= 0 or cw <= 0:
        raise SystemExit("no calibration copy found: run bench.py with --calib-copy-mib")
    sf, sw = copy_mib * 1024.0 / cf, copy_mib * 1024.0 / cw   # true KiB per counted KiB
    print(f"calibration copy {copy_mib:g} MiB: FETCH_SIZE read {cf / 1024:.1f} MiB (scale {sf:.3f}), "
          f"WRITE_SIZE read {cw / 1024:.1f} MiB (scale {sw:.3f})")
    print("| kernel | HBM read MiB/launch | HBM write MiB/launch |\n|---|---|---|")
    result = {}
    for k in f:
        if not k.startswith("k_"):
            continue
        rd = sum(f[k]) / len(f[k]) * sf / 1024.0
        wr = sum(w.get(k, [0.0])) / max(len(w.get(k, [])), 1) * sw / 1024.0
        print(f"| `{k}` | {rd:.1f} | {wr:.1f} |")
        for prefix, launch in LAUNCH_NAMES.items():
            if k.startswith(prefix):
                result[launch] = {"read_bytes": rd * 2 ** 20, "write_bytes": wr * 2 ** 20}
    if out:
        json.dump(result, open(out, "w"), indent=1, sort_keys=True)


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "stats":
        stats(sys.argv[2])
    elif len(sys.argv) >= 5 and sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3], float(sys.argv[4]), sys.argv[5] if len(sys.argv) > 5 else None)
    else:
        raise SystemExit(__doc__)

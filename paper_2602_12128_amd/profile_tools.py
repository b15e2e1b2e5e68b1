"""Turn rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2602_12128_amd.profile_tools stats   <dir-with-*_kernel_stats.csv>
    python -m paper_2602_12128_amd.profile_tools traffic <fetch-dir> <write-dir> <copy-MiB> [out.json]
    python -m paper_2602_12128_amd.profile_tools counters <pmc-dir> [<pmc-dir> ...]

`counters` averages every counter of one or more --pmc runs per kernel and dispatch, and derives
the occupancy figures of the vector ALU and the matrix pipe from the SQ counters when present.
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
    "k_query_causal<": "mfma_query_causal", "k_prefix<": "mfma_state_prefix",
    "k_vmod_forward<": "vmod_forward", "k_vmod_backward<": "vmod_backward", "k_add_rows<": "vmod_add_dv",
    "k_vmod_fwd_mfma<": "vmod_forward", "k_vmod_bwd_map<": "vmod_backward",
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


def _find(d: str, pattern: str) -> str:
    hits = glob.glob(d + "/**/" + pattern, recursive=True)
    if not hits:
        raise SystemExit(f"no {pattern} under {d}")
    return hits[0]


def counters(dirs) -> None:
    """Per kernel: average per dispatch of every counter found in the given --pmc output folders.
    SQ cycle counters (ACTIVE_INST_*, WAVE_CYCLES, WAIT_*) come in units of four cycles summed
    over waves; SQ_VALU_MFMA_BUSY_CYCLES / COEXEC_CYCLES in cycles summed over SIMDs."""
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    dur = collections.defaultdict(list)
    for d in dirs:
        seen = set()
        for r in csv.DictReader(open(_find(d, "*counter_collection.csv"))):
            k = _short(r["Kernel_Name"])
            if not k.startswith("k_"):
                continue
            acc[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
            if r["Dispatch_Id"] not in seen:
                seen.add(r["Dispatch_Id"])
                dur[k].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    for k, cs in acc.items():
        avg = {c: sum(v) / len(v) for c, v in cs.items()}
        print(f"`{k}`: {len(dur[k])} dispatches, {sum(dur[k]) / len(dur[k]):.1f} us each under the counters")
        print("    " + "  ".join(f"{c}={x:.4g}" for c, x in sorted(avg.items())))
        g = lambda c: avg.get(c, 0.0)
        if g("SQ_WAVE_CYCLES") and g("SQ_ACTIVE_INST_VALU"):
            wc = g("SQ_WAVE_CYCLES")
            line = f"    per wave: VALU issuing {g('SQ_ACTIVE_INST_VALU') / wc:.1%} of its cycles"
            if g("SQ_WAIT_INST_ANY"):
                line += f", waiting to issue {g('SQ_WAIT_INST_ANY') / wc:.1%}"
            if g("SQ_WAIT_ANY"):
                line += f", in s_waitcnt {g('SQ_WAIT_ANY') / wc:.1%}"
            print(line)
        if g("SQ_VALU_MFMA_BUSY_CYCLES"):
            mb = g("SQ_VALU_MFMA_BUSY_CYCLES")
            print(f"    matrix pipe busy {mb:.4g} SIMD-cycles, {g('SQ_VALU_MFMA_COEXEC_CYCLES') / mb:.1%} of them "
                  f"with a vector-ALU instruction executing beside it; VALU instructions per MFMA "
                  f"{g('SQ_INSTS_VALU') / max(g('SQ_INSTS_MFMA'), 1):.1f}")
        if g("SQ_LDS_IDX_ACTIVE") and g("SQ_INSTS_LDS"):
            print(f"    LDS: {g('SQ_LDS_BANK_CONFLICT') / g('SQ_LDS_IDX_ACTIVE'):.1%} of active cycles in bank conflicts, "
                  f"{g('SQ_LDS_IDX_ACTIVE') / g('SQ_INSTS_LDS'):.1f} index cycles per instruction")


def stats(d: str) -> None:
    path = _find(d, "*kernel_stats.csv")
    print("| kernel | calls | total us | avg us | % |\n|---|---|---|---|---|")
    for r in csv.DictReader(open(path)):
        print(f"| `{_short(r['Name'])}` | {r['Calls']} | {float(r['TotalDurationNs']) / 1e3:.1f} | "
              f"{float(r['AverageNs']) / 1e3:.2f} | {r['Percentage']} |")


def _per_kernel(d: str, counter: str):
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(_find(d, "*counter_collection.csv"))):
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
    elif len(sys.argv) >= 3 and sys.argv[1] == "counters":
        counters(sys.argv[2:])
    elif len(sys.argv) >= 5 and sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3], float(sys.argv[4]), sys.argv[5] if len(sys.argv) > 5 else None)
    else:
        raise SystemExit(__doc__)

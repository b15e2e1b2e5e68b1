#!/usr/bin/env python3
"""Throughput of the HLA hot path (feature maps -> key-side state -> query contraction, and
the matching backward) on one MI355X, on synthetic video-DiT-shaped inputs.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--features]

A step is one forward + backward of the whole path over the configuration's batch, inputs
resident in HBM.  Prints ONE JSON line: tokens/s (all heads of a token count once), the nominal
TFLOP/s, a `roofline` object for the kernel that takes the most time (HIP-event durations taken
inside the library around every launch) and a `cpu_baseline` object (the fp64 oracle timed on
this host's cores over a bounded sample of the same workload).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, help="workload configuration 2..5 (default 3: the headline one); 6 = 12600-token resolution, 7 = two-factor variant")
    ap.add_argument("--features", action="store_true",
                    help="feature-level interface (Q,K already phi-mapped): times the core alone")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="before the warm-up, run one device-to-device copy of this many MiB: the "
                         "known-size kernel that scales rocprofv3's FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--path", choices=["auto", "generic", "mfma"], default="auto")
    ap.add_argument("--weight-grads", action="store_true",
                    help="also produce the feature-map weight gradients in every backward (a "
                         "different workload from the headline one: named in config)")
    ap.add_argument("--value-modulation", action="store_true",
                    help="switch on the value modulation of Sec. 4.5 (a different workload: named in config)")
    ap.add_argument("--causal", action="store_true",
                    help="the causal variant of Sec. 4.4 (a different workload: named in config)")
    ap.add_argument("--decay", type=float, default=1.0,
                    help="with --causal: decay factor of the mask (Sec. 4.4), 1 = none")
    return ap.parse_args()


def measured_traffic(workload: str, kernel: str):
    """(HBM bytes per launch of `kernel`, where the figure comes from): the committed rocprofv3
    counter summary of this workload (profiles/hbm_traffic_<workload>.json, written by
    profile_tools.py from two --pmc runs of this script), not a measurement of the present run."""
    rel = os.path.join("profiles", f"hbm_traffic_{workload}.json")
    try:
        t = json.load(open(os.path.join(ROOT, rel))).get(kernel)
        if t is None:
            return None, None
        return t["read_bytes"] + t["write_bytes"], f"{rel} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, an earlier run of this command)"
    except (OSError, ValueError, KeyError):
        return None, None


def cpu_baseline(w, phi, backward, features, causal=False, decay=1.0, vmod=None):
    """Oracle (as it stands) on a bounded sample: the first heads of batch row / sequence 0, in
    the variant the run times (causal: the state recursions, about 10 s per 32760-token head)."""
    import numpy as np
    import torch

    from oracle import hla_oracle as orc
    from tests import parity_utils as pu

    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    H = w.H
    n_seq = w.N if w.cu_seqlens is None else w.cu_seqlens[1] - w.cu_seqlens[0]
    # about 1 s per 32760-token head (fwd+bwd) on 16 cores: take enough heads for 10 s or more
    heads = max(1, min(H, int(round((2 if causal else 12) * 32760 / max(n_seq, 1)))))
    sl = (slice(0, 1), slice(0, heads), slice(0, n_seq))
    t = {k: pu.to_np(v[sl]) for k, v in w.tensors.items()}
    ophi = None if features else pu.oracle_phi(phi)
    ovm = pu.oracle_vmod(vmod, 1e-5)
    t0 = time.perf_counter()
    orc.hla_operator_forward(t["Q"], t["K"], t["V"], w.F, w.d_phi, w.eps, phi=ophi, vmod=ovm, causal=causal, decay=decay)
    if backward:
        orc.hla_operator_backward(t["Q"], t["K"], t["V"], t["dO"], w.F, w.d_phi, w.eps, phi=ophi, vmod=ovm,
                                  causal=causal, decay=decay)
    dt = time.perf_counter() - t0
    # whole-job rate: a token counts once all H heads are done
    value = n_seq / (dt * H / heads)
    return {"value": value, "unit": "tokens/s", "cores": int(cores), "kind": "oracle", "blas": True,
            "sample": f"{heads} of {H} heads of one {n_seq}-token sequence, "
                      f"{'fwd+bwd' if backward else 'fwd'}, fp64 numpy, {dt:.1f} s"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2602_12128_amd as hla
    from paper_2602_12128_amd import flops
    from paper_2602_12128_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    hla.load_library()
    dev = torch.device("cuda:0")
    w = wl.make_workload(args.config)
    backward = w.backward
    phi = w.phi
    if args.features:
        ft = wl.make_feature_inputs(w.seed, w.B, w.H, w.N, w.d, w.F, w.d_phi, w.dtype)
        w.tensors["Q"], w.tensors["K"] = ft["Q"], ft["K"]
        phi = None
    t = {k: v.to(dev) for k, v in w.tensors.items()}
    nseq = w.B if w.cu_seqlens is None else len(w.cu_seqlens) - 1
    path = {"auto": hla.HLA_PATH_AUTO, "generic": hla.HLA_PATH_GENERIC, "mfma": hla.HLA_PATH_MFMA}[args.path]
    h = hla.HLA(head_dim=w.d, feature_dim=w.d_phi, degree=w.F, eps=w.eps,
                io_dtype=hla.HLA_F32 if w.dtype == torch.float32 else hla.HLA_BF16,
                phi_mode=hla.HLA_PHI_NONE if phi is None else hla.HLA_PHI_MLP, kernel_path=path,
                max_heads=w.H, max_tokens=w.B * w.N, max_seqs=nseq, causal=args.causal, decay=args.decay if args.causal else 1.0)
    if phi is not None:
        h.set_phi_weights([{k: v.to(dev) for k, v in m.items()} for m in phi])
    if args.value_modulation:
        vm = wl.draw_vmod_weights(torch.Generator("cpu").manual_seed(w.seed + 100), w.d, w.dtype)
        h.set_value_modulation([{k: v.to(dev) for k, v in m.items()} for m in vm])
    O = torch.empty_like(t["V"])
    grads = [torch.empty_like(t[k]) for k in ("Q", "K", "V")] if backward else None
    wgrads = None
    if args.weight_grads:
        if phi is None or not backward:
            print("bench.py: --weight-grads needs feature maps and a backward pass", file=sys.stderr)
            sys.exit(2)
        wgrads = [{"d" + k: torch.empty(v.shape, dtype=torch.float32, device=dev) for k, v in m.items()}
                  for m in phi]
        h.set_phi_weight_grads(wgrads)
        if args.value_modulation:  # the modulation's own weights, too
            vwgrads = [{"d" + k: torch.empty(v.shape, dtype=torch.float32, device=dev) for k, v in m.items()}
                       for m in vm]
            h.set_value_modulation_grads(vwgrads)

    def step():
        h.forward(t["Q"], t["K"], t["V"], O, cu_seqlens=w.cu_seqlens)
        if backward:
            h.backward(t["Q"], t["K"], t["V"], O, t["dO"], *grads, cu_seqlens=w.cu_seqlens)

    if args.calib_copy_mib > 0:
        src = torch.zeros(args.calib_copy_mib * 2 ** 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    # The oracle leg runs first (the GPU idles meanwhile), then the per-kernel pass, then warm-up
    # and the timed steps back to back: the first ~10 ms of load after an idle period run up to
    # 15 % slower (clock / power management settling: steps 6-30 of a cold start), and that
    # transient is not part of the steady-state step this line reports.
    cpu = None if args.no_cpu else cpu_baseline(w, phi, backward, args.features, args.causal, args.decay,
                                                vm if args.value_modulation else None)

    # per-kernel durations: HIP event pairs inside the library around every launch
    prof_steps = max(args.steps, 60) if args.steps >= 10 else args.steps  # short runs: counter collection
    h.profile_enable(True)
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    prof = h.profile_read()
    h.profile_enable(False)
    kernels = {p["kernel"]: {"avg_us": 1e3 * p["total_ms"] / p["launches"],
                             "launches_per_step": p["launches"] / prof_steps} for p in prof}
    sum_us = sum(k["avg_us"] * k["launches_per_step"] for k in kernels.values())

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps

    tokens = w.N * w.B
    th = w.token_heads
    tok_s = tokens / (elapsed / args.steps)
    fl = flops.path_flops(w.d, w.d_phi, w.F, backward, phi is not None) * th
    by = flops.path_bytes(w.d, w.d_phi, w.F, backward, phi is not None) * th
    tflops = fl / (elapsed / args.steps) / 1e12

    mfma_path = h.active_path == hla.HLA_PATH_MFMA
    fl_exec = flops.executed_path_flops(w.d, w.d_phi, w.F, backward, phi is not None) * th if mfma_path else None
    roofline = None
    if kernels:
        dom = max(kernels, key=lambda k: kernels[k]["avg_us"] * kernels[k]["launches_per_step"])
        model = flops.kernel_model(dom, w.d, w.d_phi, w.F)
        if model is not None:
            kb, kf, bound = model
            dur = kernels[dom]["avg_us"] * 1e-6
            traffic, traffic_source = measured_traffic(w.name, dom)
            roofline = {"kernel": dom, "avg_launch_us": kernels[dom]["avg_us"],
                        "algorithmic_bytes_per_launch": kb * th, "nominal_flops_per_launch": kf * th,
                        "traffic": traffic, "traffic_source": traffic_source}
            if bound == "alu":
                peak, unit = flops.PEAKS["alu"]
                roofline.update(bound="alu", achieved=kf * th / dur / 1e12, peak=peak, unit=unit)
            else:
                # against both roofs; the one the kernel is nearer to is reported as its bound
                ke = flops.executed_kernel_flops(dom, w.d, w.d_phi, w.F)
                frac_hbm = kb * th / dur / 1e9 / flops.PEAKS["hbm"][0]
                frac_mfma = kf * th / dur / 1e12 / flops.PEAKS["mfma"][0]
                roofline.update(frac_hbm=frac_hbm, frac_mfma_nominal=frac_mfma,
                                frac_mfma_executed=ke * th / dur / 1e12 / flops.PEAKS["mfma"][0],
                                executed_flops_per_launch=ke * th)
                bound = "hbm" if frac_hbm >= frac_mfma else "mfma"
                peak, unit = flops.PEAKS[bound]
                roofline.update(bound=bound, peak=peak, unit=unit,
                                achieved=(kb * th / dur / 1e9) if bound == "hbm" else (kf * th / dur / 1e12))
            roofline["frac"] = roofline["achieved"] / roofline["peak"]

    out = {
        "metric": "HLA fwd+bwd tokens/s" if backward else "HLA fwd tokens/s",
        "value": tok_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if w.dtype == torch.bfloat16 else "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "N": w.N, "d": w.d, "F": w.F,
                   "d_phi": w.d_phi, "phi": "mlp" if phi is not None else "none",
                   "packed_seqs": nseq if w.cu_seqlens else 0,
                   "path": "mfma" if h.active_path == hla.HLA_PATH_MFMA else "generic",
                   "weight_grads": wgrads is not None, "value_modulation": args.value_modulation, "decay": args.decay if args.causal else None,
                   "causal": args.causal},
        "tflops_nominal": tflops,
        "mfma_peak_frac_nominal": tflops / 2500.0,
        "tflops_executed": None if fl_exec is None else fl_exec / (elapsed / args.steps) / 1e12,
        "mfma_peak_frac_executed": None if fl_exec is None else fl_exec / (elapsed / args.steps) / 1e12 / 2500.0,
        "hbm_frac_whole_path": by / (elapsed / args.steps) / 8e12,
        "kernels_us": {k: round(v["avg_us"] * v["launches_per_step"], 2) for k, v in kernels.items()},
        "kernels_sum_us": round(sum_us, 2),
        "roofline": roofline,
    }
    out["untimed_before"] = f"per-kernel event pass of {prof_steps} steps, then {args.warmup} warm-up steps"
    if cpu is not None:
        out["cpu_baseline"] = cpu
    h.destroy()
    print(json.dumps(out))


if __name__ == "__main__":
    main()

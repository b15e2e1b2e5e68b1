"""Helpers shared by the GPU parity tests: run the library through its C ABI (Python binding),
run the CPU oracle on the same tensors, and compare with the build's error measure."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

import paper_2602_12128_amd as hla
from oracle import hla_oracle as orc

TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}


def max_rel_err(got, ref) -> float:
    """max_i |got_i - ref_i| / max_i |ref_i| over one tensor (0 when both are all-zero)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    scale = np.abs(ref).max() if ref.size else 0.0
    diff = np.abs(got - ref).max() if ref.size else 0.0
    if scale == 0.0:
        return 0.0 if diff == 0.0 else float("inf")
    return float(diff / scale)


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


def oracle_phi(phi: Optional[Sequence[Dict[str, torch.Tensor]]]):
    if phi is None:
        return None
    return [orc.PhiWeights(*(to_np(m[k]) for k in ("W1", "b1", "W2", "b2"))) for m in phi]


def make_handle(tensors, F, d_phi, eps, phi, cu_seqlens, path=hla.HLA_PATH_AUTO, max_scale=1):
    V = tensors["V"]
    B, H, N, d = V.shape
    nseq = B if cu_seqlens is None else len(cu_seqlens) - 1
    h = hla.HLA(head_dim=d, feature_dim=d_phi, degree=F, eps=eps,
                io_dtype=hla.HLA_F32 if V.dtype == torch.float32 else hla.HLA_BF16,
                phi_mode=hla.HLA_PHI_NONE if phi is None else hla.HLA_PHI_MLP,
                kernel_path=path, max_heads=max(H, 1), max_tokens=max(B * N, 1) * max_scale,
                max_seqs=max(nseq, 1))
    return h


def run_gpu(tensors: Dict[str, torch.Tensor], F: int, d_phi: int, eps: float,
            phi=None, cu_seqlens=None, backward=True, path=hla.HLA_PATH_AUTO, handle=None):
    """Returns dict of CPU tensors O (and dQ, dK, dV) computed by the HIP library."""
    dev = torch.device("cuda:0")
    t = {k: v.to(dev) for k, v in tensors.items()}
    h = handle or make_handle(tensors, F, d_phi, eps, phi, cu_seqlens, path)
    if phi is not None:
        phi_dev = [{k: v.to(dev) for k, v in m.items()} for m in phi]
        h.set_phi_weights(phi_dev)
    out = {"O": torch.full_like(t["V"], float("nan"))}
    h.forward(t["Q"], t["K"], t["V"], out["O"], cu_seqlens=cu_seqlens)
    if backward:
        for n, src in (("dQ", "Q"), ("dK", "K"), ("dV", "V")):
            out[n] = torch.full_like(t[src], float("nan"))
        h.backward(t["Q"], t["K"], t["V"], out["O"], t["dO"], out["dQ"], out["dK"], out["dV"],
                   cu_seqlens=cu_seqlens)
    torch.cuda.synchronize()
    res = {k: v.cpu() for k, v in out.items()}
    res["_path"] = h.active_path
    if handle is None:
        h.destroy()
    return res


def run_oracle(tensors, F, d_phi, eps, phi=None, cu_seqlens=None, backward=True,
               route="factorized"):
    Q, K, V = (to_np(tensors[k]) for k in ("Q", "K", "V"))
    ophi = oracle_phi(phi)
    out = {"O": orc.hla_operator_forward(Q, K, V, F, d_phi, eps, phi=ophi, cu_seqlens=cu_seqlens,
                                         route=route)}
    if backward:
        dQ, dK, dV = orc.hla_operator_backward(Q, K, V, to_np(tensors["dO"]), F, d_phi, eps,
                                               phi=ophi, cu_seqlens=cu_seqlens, route=route)
        out.update(dQ=dQ, dK=dK, dV=dV)
    return out


def relu_kink_masks(tensors, phi, F, band):
    """Token masks (True = compare) for dQ and dK.  The ReLU of the feature maps makes the
    gradient discontinuous where a pre-activation u crosses zero; a token whose |u| is within
    the arithmetic's error `band` of zero may take the other branch on the GPU (which decides in
    its own precision), so its gradient row is compared only through the finiteness check."""
    ophi = oracle_phi(phi)
    Q, K = to_np(tensors["Q"]), to_np(tensors["K"])
    uq = np.abs(orc.phi_forward(Q, *ophi[0].astuple())[2]).min(-1)
    uk = np.minimum.reduce([np.abs(orc.phi_forward(K, *ophi[1 + f].astuple())[2]).min(-1)
                            for f in range(F)])
    return {"dQ": uq > band, "dK": uk > band}


def assert_parity(gpu, ref, tol, what="", row_masks=None):
    errs = {}
    for k, r in ref.items():
        g = to_np(gpu[k])
        assert np.isfinite(g).all(), f"{what}: {k} has non-finite entries"
        if row_masks is not None and k in row_masks:
            m = row_masks[k]
            assert m.mean() > 0.8, f"{what}: kink band excludes too many rows of {k}"
            scale = np.abs(r).max()
            errs[k] = float(np.abs(g - r)[m].max() / scale) if m.any() else 0.0
            continue
        errs[k] = max_rel_err(g, r)
    msg = ", ".join(f"{k}={e:.2e}" for k, e in errs.items())
    print(f"[parity] {what}: {msg} (tol {tol:g})", flush=True)
    bad = {k: e for k, e in errs.items() if not e <= tol}
    assert not bad, f"{what}: max relative error above {tol:g}: {bad}"
    return errs

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


WG_KEYS = ("dW1", "db1", "dW2", "db2")


def run_gpu(tensors: Dict[str, torch.Tensor], F: int, d_phi: int, eps: float,
            phi=None, cu_seqlens=None, backward=True, path=hla.HLA_PATH_AUTO, handle=None,
            weight_grads=False, per_head=False):
    """Returns dict of CPU tensors O (and dQ, dK, dV) computed by the HIP library; with
    weight_grads also 'wg': per map a dict of the fp32 weight gradients.  per_head: the weights
    carry a leading head dimension."""
    dev = torch.device("cuda:0")
    t = {k: v.to(dev) for k, v in tensors.items()}
    h = handle or make_handle(tensors, F, d_phi, eps, phi, cu_seqlens, path)
    wg = None
    if phi is not None:
        phi_dev = [{k: v.to(dev) for k, v in m.items()} for m in phi]
        h.set_phi_weights(phi_dev, per_head=per_head)
        if weight_grads:
            wg = [{"d" + k: torch.full(v.shape, float("nan"), dtype=torch.float32, device=dev)
                   for k, v in m.items()} for m in phi_dev]
            h.set_phi_weight_grads(wg)
    out = {"O": torch.full_like(t["V"], float("nan"))}
    h.forward(t["Q"], t["K"], t["V"], out["O"], cu_seqlens=cu_seqlens)
    if backward:
        for n, src in (("dQ", "Q"), ("dK", "K"), ("dV", "V")):
            out[n] = torch.full_like(t[src], float("nan"))
        h.backward(t["Q"], t["K"], t["V"], out["O"], t["dO"], out["dQ"], out["dK"], out["dV"],
                   cu_seqlens=cu_seqlens)
    torch.cuda.synchronize()
    res = {k: v.cpu() for k, v in out.items()}
    if wg is not None:
        res["wg"] = [{k: v.cpu() for k, v in m.items()} for m in wg]
        # the library's own ReLU decisions (feature > 0), for an oracle that differentiates the
        # same branches: [B, H, N, (1+F)*d_phi]
        B, H, N = t["V"].shape[:3]
        nfeat = (1 + F) * d_phi
        feats = h.read_workspace(hla.binding.HLA_WS_FEATURES, B * H * N * nfeat)
        res["relu_open"] = feats.reshape(B, H, N, nfeat) > 0
    res["_path"] = h.active_path
    if handle is None:
        h.destroy()
    return res


RELU_BAND = 1e-2  # |pre-activation| below this: the library may decide the ReLU either way


def assert_relu_decisions_valid(tensors, phi, F, relu_open, band=RELU_BAND):
    """The ReLU decisions read back from the library (feature > 0) are only handed to the oracle
    after the oracle has confirmed them: wherever its own fp64 pre-activation is further than
    `band` from zero (the rounding error of the library's bf16/fp16 feature maps) the decision
    must be the oracle's own; inside the band either branch is a valid one."""
    ophi = oracle_phi(phi)
    Q, K = to_np(tensors["Q"]), to_np(tensors["K"])
    u = [orc.phi_forward(Q, *ophi[0].astuple())[2]]
    u += [orc.phi_forward(K, *ophi[1 + f].astuple())[2] for f in range(F)]
    u = np.concatenate(u, axis=-1)
    relu_open = np.asarray(relu_open)
    assert relu_open.shape == u.shape, (relu_open.shape, u.shape)
    clear = np.abs(u) > band
    wrong = clear & (relu_open != (u > 0))
    assert not wrong.any(), f"{int(wrong.sum())} ReLU decisions differ from the oracle's outside the band"
    assert clear.mean() > 0.9, "the band covers too many pre-activations to mean anything"


def run_oracle(tensors, F, d_phi, eps, phi=None, cu_seqlens=None, backward=True,
               route="factorized", weight_grads=False, relu_open=None):
    Q, K, V = (to_np(tensors[k]) for k in ("Q", "K", "V"))
    ophi = oracle_phi(phi)
    if relu_open is not None and phi is not None:
        assert_relu_decisions_valid(tensors, phi, F, relu_open)
    out = {"O": orc.hla_operator_forward(Q, K, V, F, d_phi, eps, phi=ophi, cu_seqlens=cu_seqlens,
                                         route=route)}
    if backward:
        res = orc.hla_operator_backward(Q, K, V, to_np(tensors["dO"]), F, d_phi, eps,
                                        phi=ophi, cu_seqlens=cu_seqlens, route=route,
                                        weight_grads=weight_grads, relu_open=relu_open)
        out.update(dQ=res[0], dK=res[1], dV=res[2])
        if weight_grads:
            out["wg"] = [dict(zip(WG_KEYS, m)) for m in res[3]]
    return out


def run_oracle_per_head(tensors, F, d_phi, eps, phi, cu_seqlens=None, weight_grads=True,
                        relu_open=None):
    """Oracle for weights that carry a leading head dimension: the oracle's maps are shared by
    the heads it is given, so every head is run on its own with its own weights."""
    H = tensors["V"].shape[1]
    outs = []
    for h in range(H):
        th = {k: v[:, h:h + 1] for k, v in tensors.items()}
        ph = [{k: v[h] for k, v in m.items()} for m in phi]
        outs.append(run_oracle(th, F, d_phi, eps, phi=ph, cu_seqlens=cu_seqlens,
                               weight_grads=weight_grads,
                               relu_open=None if relu_open is None else relu_open[:, h:h + 1]))
    out = {k: np.concatenate([o[k] for o in outs], axis=1) for k in ("O", "dQ", "dK", "dV")}
    if weight_grads:
        out["wg"] = [{k: np.stack([o["wg"][m][k] for o in outs]) for k in WG_KEYS}
                     for m in range(len(phi))]
    return out


def assert_weight_grad_parity(gpu_wg, ref_wg, tol, what=""):
    """Every weight-gradient array of every map against the oracle with the build's error
    measure (max |diff| / max |ref| per array)."""
    worst = {}
    for m, (g, r) in enumerate(zip(gpu_wg, ref_wg)):
        for k in WG_KEYS:
            got = to_np(g[k])
            assert np.isfinite(got).all(), f"{what}: map {m} {k} has non-finite entries"
            assert got.shape == r[k].shape, f"{what}: map {m} {k} shape {got.shape} vs {r[k].shape}"
            worst[f"{k}[{m}]"] = max_rel_err(got, r[k])
    msg = ", ".join(f"{k}={e:.2e}" for k, e in worst.items())
    print(f"[parity] {what}: {msg} (tol {tol:g})", flush=True)
    bad = {k: e for k, e in worst.items() if not e <= tol}
    assert not bad, f"{what}: weight gradients above {tol:g}: {bad}"
    return worst


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
        if k == "wg":
            continue
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

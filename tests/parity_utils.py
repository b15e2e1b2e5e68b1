"""Helpers shared by the GPU parity tests: run the library through its C ABI (Python binding),
run the CPU oracle on the same tensors, and compare with the build's error measure.

Every reference value comes from the oracle alone; nothing the library computes is ever handed to
it.  Where the final ReLU of the feature maps (App. A.1) makes a gradient discontinuous, the
oracle enumerates the branch choices that are open to an implementation in lower precision and
the comparison asks the library's result to match one of them."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

import paper_2602_12128_amd as hla
from oracle import hla_oracle as orc

TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}

# |pre-ReLU value| below which the library (bf16 first layer, fp16 GELU and second layer) may
# take either branch of the ReLU.  test_gpu_mfma.py::test_features_match_oracle asserts that
# the library's features stay within this distance of the oracle's, which is what makes the
# band wide enough: outside it both sides decide alike.
RELU_BAND = 1e-2


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


def make_handle(tensors, F, d_phi, eps, phi, cu_seqlens, path=hla.HLA_PATH_AUTO, max_scale=1,
                causal=False, decay=1.0):
    V = tensors["V"]
    B, H, N, d = V.shape
    nseq = B if cu_seqlens is None else len(cu_seqlens) - 1
    h = hla.HLA(head_dim=d, feature_dim=d_phi, degree=F, eps=eps,
                io_dtype=hla.HLA_F32 if V.dtype == torch.float32 else hla.HLA_BF16,
                phi_mode=hla.HLA_PHI_NONE if phi is None else hla.HLA_PHI_MLP,
                kernel_path=path, max_heads=max(H, 1), max_tokens=max(B * N, 1) * max_scale,
                max_seqs=max(nseq, 1), causal=causal, decay=decay)
    return h


WG_KEYS = ("dW1", "db1", "dW2", "db2")
VWG_KEYS = ("dW1", "db1", "dW2", "db2", "dgamma", "dbeta")


def run_gpu(tensors: Dict[str, torch.Tensor], F: int, d_phi: int, eps: float,
            phi=None, cu_seqlens=None, backward=True, path=hla.HLA_PATH_AUTO, handle=None,
            weight_grads=False, per_head=False, features=False, vmod=None, ln_eps=1e-5,
            vmod_weight_grads=False, causal=False, decay=1.0):
    """Returns dict of CPU tensors O (and dQ, dK, dV) computed by the HIP library; with
    weight_grads also 'wg': per map a dict of the fp32 weight gradients.  per_head: the weights
    carry a leading head dimension.  features: also '_features' [B,H,N,(1+F)*d_phi], the
    library's own feature workspace (an output to be compared, like the others).  vmod: the two
    value-modulation maps (Sec. 4.5), switched on for the call; with vmod_weight_grads also
    'vwg': per map a dict of the fp32 gradients of its weights.  causal / decay: the masked
    variant of Sec. 4.4 (a property of the handle)."""
    dev = torch.device("cuda:0")
    t = {k: v.to(dev) for k, v in tensors.items()}
    h = handle or make_handle(tensors, F, d_phi, eps, phi, cu_seqlens, path, causal=causal, decay=decay)
    wg = None
    if phi is not None:
        phi_dev = [{k: v.to(dev) for k, v in m.items()} for m in phi]
        h.set_phi_weights(phi_dev, per_head=per_head)
        if weight_grads:
            wg = [{"d" + k: torch.full(v.shape, float("nan"), dtype=torch.float32, device=dev)
                   for k, v in m.items()} for m in phi_dev]
            h.set_phi_weight_grads(wg)
    if vmod is not None:
        h.set_value_modulation([{k: v.to(dev) for k, v in m.items()} for m in vmod], ln_eps)
    vwg = None
    if vmod_weight_grads:
        vwg = [{"d" + k: torch.full(v.shape, float("nan"), dtype=torch.float32, device=dev)
                for k, v in m.items()} for m in vmod]
        h.set_value_modulation_grads(vwg)
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
    if vwg is not None:
        res["vwg"] = [{k: v.cpu() for k, v in m.items()} for m in vwg]
    if features:
        B, H, N = t["V"].shape[:3]
        nfeat = (1 + F) * d_phi
        res["_features"] = h.read_workspace(hla.binding.HLA_WS_FEATURES, B * H * N * nfeat).reshape(B, H, N, nfeat)
    res["_path"] = h.active_path
    if handle is None:
        h.destroy()
    return res


def oracle_vmod(vmod, ln_eps):
    if vmod is None:
        return None
    keys = ("W1", "b1", "W2", "b2", "gamma", "beta")
    return tuple(orc.PhiVWeights(*(to_np(m[k]) for k in keys)) for m in vmod) + (ln_eps,)


def run_oracle(tensors, F, d_phi, eps, phi=None, cu_seqlens=None, backward=True,
               route="factorized", weight_grads=False, vmod=None, ln_eps=1e-5, vmod_weight_grads=False,
               causal=False, decay=1.0):
    """O (and dQ, dK, dV, 'wg') from the oracle; with feature maps and a backward also the
    feature gradients '_dqf', '_dkf' that the branch enumeration below starts from."""
    Q, K, V = (to_np(tensors[k]) for k in ("Q", "K", "V"))
    ophi = oracle_phi(phi)
    ovm = oracle_vmod(vmod, ln_eps)
    out = {"O": orc.hla_operator_forward(Q, K, V, F, d_phi, eps, phi=ophi, cu_seqlens=cu_seqlens,
                                         route=route, vmod=ovm, causal=causal, decay=decay)}
    if backward:
        res = orc.hla_operator_backward(Q, K, V, to_np(tensors["dO"]), F, d_phi, eps,
                                        phi=ophi, cu_seqlens=cu_seqlens, route=route,
                                        weight_grads=weight_grads, feature_grads=True, vmod=ovm,
                                        vmod_weight_grads=vmod_weight_grads, causal=causal, decay=decay)
        out.update(dQ=res[0], dK=res[1], dV=res[2])
        if weight_grads:
            out["wg"] = [dict(zip(WG_KEYS, m)) for m in res[3]]
        if vmod_weight_grads:
            out["vwg"] = [dict(zip(VWG_KEYS, m)) for m in res[-1]]
            res = res[:-1]
        out["_dqf"], out["_dkf"] = res[-1]
    return out


def run_oracle_per_head(tensors, F, d_phi, eps, phi, cu_seqlens=None, weight_grads=True):
    """Oracle for weights that carry a leading head dimension: the oracle's maps are shared by
    the heads it is given, so every head is run on its own with its own weights."""
    H = tensors["V"].shape[1]
    outs = []
    for h in range(H):
        th = {k: v[:, h:h + 1] for k, v in tensors.items()}
        ph = [{k: v[h] for k, v in m.items()} for m in phi]
        outs.append(run_oracle(th, F, d_phi, eps, phi=ph, cu_seqlens=cu_seqlens,
                               weight_grads=weight_grads))
    out = {k: np.concatenate([o[k] for o in outs], axis=1) for k in ("O", "dQ", "dK", "dV", "_dqf", "_dkf")}
    if weight_grads:
        out["wg"] = [{k: np.stack([o["wg"][m][k] for o in outs]) for k in WG_KEYS}
                     for m in range(len(phi))]
    return out


# ---- ReLU kinks: the oracle's branch choices ------------------------------------------------------
def _head_maps(phi, F, h, per_head):
    """Oracle weight tuples (phi_q, phi_k1..kF) of head h."""
    if per_head:
        phi = [{k: v[h] for k, v in m.items()} for m in phi]
    return [m.astuple() for m in oracle_phi(phi)]


def oracle_kinks(tensors, phi, F, d_phi, ref, band=RELU_BAND, per_head=False):
    """For dQ and dK: {(b, h, n): candidate rows [2^k, d]} for every token whose pre-ReLU values
    include k >= 1 within `band` of zero: all gradient rows the oracle computes by opening or
    closing those k features (orc.phi_backward_branches), from the oracle's own feature
    gradients ref['_dqf'], ref['_dkf']."""
    Q, K = to_np(tensors["Q"]), to_np(tensors["K"])
    B, H = Q.shape[:2]
    out = {"dQ": {}, "dK": {}}
    for b in range(B):
        for h in range(H):
            maps = _head_maps(phi, F, h, per_head)
            br = orc.phi_backward_branches([ref["_dqf"][b, h]], Q[b, h], maps[:1], band)
            out["dQ"].update({(b, h, n): c for n, c in br.items()})
            dk = [ref["_dkf"][b, h][:, f * d_phi:(f + 1) * d_phi] for f in range(F)]
            br = orc.phi_backward_branches(dk, K[b, h], maps[1:], band)
            out["dK"].update({(b, h, n): c for n, c in br.items()})
    return out


def _log_allclose(k, g, r, tol):
    """Elementwise view next to the per-tensor measure: share of entries outside
    |g - r| <= tol * |r| + tol * rms(r).  Logged, not asserted."""
    rms = float(np.sqrt(np.mean(r * r))) if r.size else 0.0
    bad = np.abs(g - r) > tol * np.abs(r) + tol * rms
    return f"{k}:{bad.mean():.1e}"


def assert_parity(gpu, ref, tol, what="", kinks=None, row_scale=None):
    """Per tensor: max |gpu - ref| / max |ref| <= tol.  kinks (from oracle_kinks): rows of dQ / dK
    listed there are compared with the closest of the oracle's branch choices instead of the
    single reference row.  row_scale: {tensor: (mask [B,H,N], scale)}: rows under the mask are
    measured against the absolute scale given instead of max |ref| (sequences too short for the
    gradient to be more than the remainder of two cancelling terms)."""
    errs, close, notes = {}, [], []
    for k, r in ref.items():
        if k == "wg" or k.startswith("_"):
            continue
        g = to_np(gpu[k])
        assert np.isfinite(g).all(), f"{what}: {k} has non-finite entries"
        diff = np.abs(g - r)
        if kinks is not None and kinks.get(k):
            n_other = 0
            for (b, h, n), cands in kinks[k].items():
                d_c = np.abs(cands - g[b, h, n][None, :]).max(axis=1)
                best = int(d_c.argmin())
                # the row is judged by its distance to the closest choice
                diff[b, h, n] = np.abs(cands[best] - g[b, h, n])
                n_other += int(np.abs(cands[best] - r[b, h, n]).max() > 1e-9 * max(np.abs(r).max(), 1e-300))
            notes.append(f"{k}: {len(kinks[k])} kink rows ({len(kinks[k]) / max(1, r[..., 0].size):.2%}), "
                         f"{n_other} on another branch than the oracle's own")
        scale = np.abs(r).max() if r.size else 0.0
        if row_scale is not None and k in row_scale:
            mask, s_abs = row_scale[k]
            short = diff[mask].max() / s_abs if mask.any() else 0.0
            rest = diff[~mask].max() / scale if (~mask).any() and scale > 0 else 0.0
            errs[k] = float(max(short, rest))
            notes.append(f"{k}: {int(mask.sum())} short-sequence rows on the absolute scale {s_abs:.3g}: {short:.2e}")
        elif scale == 0.0:
            errs[k] = 0.0 if not diff.size or diff.max() == 0.0 else float("inf")
        else:
            errs[k] = float(diff.max() / scale)
        close.append(_log_allclose(k, g, r, tol))
    msg = ", ".join(f"{k}={e:.2e}" for k, e in errs.items())
    print(f"[parity] {what}: {msg} (tol {tol:g}); outside elementwise allclose: {' '.join(close)}", flush=True)
    for n in notes:
        print(f"[parity]   {n}", flush=True)
    bad = {k: e for k, e in errs.items() if not e <= tol}
    assert not bad, f"{what}: max relative error above {tol:g}: {bad}"
    return errs


def assert_vmod_weight_grad_parity(gpu_vwg, ref_vwg, tol, what=""):
    """The six weight-gradient arrays of the two value-modulation maps against the oracle, each
    with the build's error measure (max |diff| / max |ref| per array).  These maps have no ReLU:
    nothing to enumerate."""
    worst = {}
    for m, (g, r) in enumerate(zip(gpu_vwg, ref_vwg)):
        for k in VWG_KEYS:
            got = to_np(g[k])
            assert np.isfinite(got).all(), f"{what}: map {m} {k} has non-finite entries"
            assert got.shape == r[k].shape
            worst[f"{k}[{m}]"] = max_rel_err(got, r[k])
    print(f"[parity] {what}: " + ", ".join(f"{k}={v:.2e}" for k, v in worst.items()) + f" (tol {tol:g})")
    bad = {k: v for k, v in worst.items() if not v <= tol}
    assert not bad, f"{what}: max relative error above {tol:g}: {bad}"
    return worst


def assert_weight_grad_parity(gpu_wg, ref_wg, tol, what="", branches=None):
    """Every weight-gradient array of every map against the oracle with the build's error
    measure (max |diff| / max |ref| per array).

    branches (from oracle_weight_grad_branches; bf16 paths): per (map[, head]) the oracle's
    (base, pairs, contribs, own).  The gradients are sums over all tokens, linear in the ReLU
    branch choices of the in-band (token, feature) pairs, so the library must agree with
    base + sum choice_p contrib_p for ONE assignment of choices in {0, 1}: the assignment is
    fitted by least squares over all four arrays of the map, rounded to {0, 1}, and the
    rounded and refined by single flips, and the residual of that single assignment is what is
    measured."""
    worst = {}
    for m, (g, r) in enumerate(zip(gpu_wg, ref_wg)):
        per_head = branches is not None and isinstance(branches[m], list)
        heads = len(branches[m]) if per_head else 1
        for hh in range(heads):
            sel = (lambda a: a[hh]) if per_head else (lambda a: a)
            got = {k: sel(to_np(g[k])) for k in WG_KEYS}
            own = {k: sel(r[k]) for k in WG_KEYS}
            for k in WG_KEYS:
                assert np.isfinite(got[k]).all(), f"{what}: map {m} {k} has non-finite entries"
                assert got[k].shape == own[k].shape, f"{what}: map {m} {k} shape {got[k].shape} vs {own[k].shape}"
            tag = f"[{m}]" + (f"h{hh}" if per_head else "")
            br = None if branches is None else (branches[m][hh] if per_head else branches[m])
            if br is None or not br[1]:
                for k in WG_KEYS:
                    worst[k + tag] = max_rel_err(got[k], own[k])
                continue
            base, pairs, contribs, own_choice = br
            scale = [max(np.abs(own[k]).max(), 1e-300) for k in WG_KEYS]
            resid = np.concatenate([((got[k] - base[i]) / scale[i]).ravel() for i, k in enumerate(WG_KEYS)])
            A = np.stack([np.concatenate([(c[i] / scale[i]).ravel() for i in range(4)]) for c in contribs], axis=1)
            coef = np.linalg.lstsq(A, resid, rcond=None)[0]
            choice = coef > 0.5
            bounds = np.cumsum([0] + [got[k].size for k in WG_KEYS])

            def per_array(c):
                fit = resid - A @ c.astype(np.float64)
                return [float(np.abs(fit[bounds[i]:bounds[i + 1]]).max()) for i in range(4)]

            # The least-squares fit is dominated by the largest array; a pair whose contribution
            # there is below the arithmetic's noise can come out on the wrong side of 1/2 and
            # still matter for a six-entry bias gradient.  Refine the rounded assignment by
            # single flips that lower the worst array error until none does.
            errs = per_array(choice)
            for _ in range(4):
                improved = False
                for pi in range(len(pairs)):
                    choice[pi] = not choice[pi]
                    e2 = per_array(choice)
                    if max(e2) < max(errs):
                        errs, improved = e2, True
                    else:
                        choice[pi] = not choice[pi]
                if not improved:
                    break
            for i, k in enumerate(WG_KEYS):
                worst[k + tag] = errs[i]
            slack = [float(sum(np.abs(c[i]) for c in contribs).max() / scale[i]) for i in range(4)]
            flips = int((choice != np.asarray(own_choice)).sum())
            print(f"[parity]   {what} map {m}{' head %d' % hh if per_head else ''}: {len(pairs)} in-band pairs, "
                  f"{flips} taken on the other branch than the oracle's own; a bound that ignored the choices "
                  f"would add {', '.join(f'{k} {s:.1e}' for k, s in zip(WG_KEYS, slack))} of max|ref|", flush=True)
    msg = ", ".join(f"{k}={e:.2e}" for k, e in worst.items())
    print(f"[parity] {what}: {msg} (tol {tol:g})", flush=True)
    bad = {k: e for k, e in worst.items() if not e <= tol}
    assert not bad, f"{what}: weight gradients above {tol:g}: {bad}"
    return worst


def oracle_weight_grad_branches(tensors, phi, F, d_phi, ref, cu_seqlens=None, band=RELU_BAND,
                                per_head=False):
    """orc.phi_weight_grad_branches for every map over all rows that share its weights (every
    batch row, head and sequence; one head at a time when the weights are per head): a list over
    maps of (base, pairs, contribs, own), or of per-head lists of them."""
    Q, K = to_np(tensors["Q"]), to_np(tensors["K"])
    B, H, N, d = Q.shape
    if cu_seqlens is not None:  # tokens outside every sequence do not exist for the operator
        assert cu_seqlens[0] == 0 and cu_seqlens[-1] == N
    out = []
    for m in range(1 + F):
        X = Q if m == 0 else K
        dfe = ref["_dqf"] if m == 0 else ref["_dkf"][..., (m - 1) * d_phi:m * d_phi]
        if per_head:
            res = []
            for h in range(H):
                w = _head_maps(phi, F, h, True)[m]
                res.append(orc.phi_weight_grad_branches(dfe[:, h].reshape(-1, d_phi), X[:, h].reshape(-1, d), *w, band))
            out.append(res)
        else:
            w = _head_maps(phi, F, 0, False)[m]
            out.append(orc.phi_weight_grad_branches(dfe.reshape(-1, d_phi), X.reshape(-1, d), *w, band))
    return out


def short_sequence_rows(tensors, ref, cu_seqlens, max_len=2):
    """row_scale argument of assert_parity for dQ and dK: rows of packed sequences of at most
    max_len tokens.  Their outputs barely depend on Q and K (one token: not at all, up to eps),
    so the gradient is what is left of two cancelling terms of size |dO| |v| (times the gain of
    the feature map's backward, taken as max |dX| / max |d feature| over the other rows of the
    oracle's result) and is measured on that scale."""
    B, H, N = tensors["V"].shape[:3]
    mask = np.zeros((B, H, N), bool)
    for lo, hi in zip(cu_seqlens[:-1], cu_seqlens[1:]):
        if 0 < hi - lo <= max_len:
            mask[:, :, lo:hi] = True
    base = float(tensors["dO"].float().abs().max() * tensors["V"].float().abs().max())
    out = {}
    for k, fk in (("dQ", "_dqf"), ("dK", "_dkf")):
        if fk in ref and (~mask).any():
            gain = np.abs(ref[k][~mask]).max() / max(np.abs(ref[fk][~mask]).max(), 1e-300)
        else:
            gain = 1.0
        out[k] = (mask, base * max(gain, 1.0))
    return out


def causal_first_token_rows(tensors, ref, cu_seqlens=None):
    """row_scale argument of assert_parity for dQ of the causal variant: the first token of every
    sequence sees itself only, so its output does not depend on its query (up to eps) and its dQ
    is what is left of two cancelling terms, exactly as for a one-token sequence (see
    short_sequence_rows): measured on the same absolute scale."""
    B, H, N = tensors["V"].shape[:3]
    mask = np.zeros((B, H, N), bool)
    starts = [0] if cu_seqlens is None else [lo for lo, hi in zip(cu_seqlens[:-1], cu_seqlens[1:]) if hi > lo]
    mask[:, :, starts] = True
    base = float(tensors["dO"].float().abs().max() * tensors["V"].float().abs().max())
    gain = 1.0
    if "_dqf" in ref and (~mask).any():
        gain = np.abs(ref["dQ"][~mask]).max() / max(np.abs(ref["_dqf"][~mask]).max(), 1e-300)
    return {"dQ": (mask, base * max(gain, 1.0))}

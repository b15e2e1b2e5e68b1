"""GPU parity of the causal variant (Sec. 4.4: token i attends to tokens j <= i) through the C ABI,
forward and backward: full comparison with the oracle's masked N x N matrix at sizes that span
several chunks of the scan with ragged tails, sampled rows at the video-DiT size, packed sequences
without leaks, both forms, through the feature maps, with decay factors, with the value
modulation on top, on the matrix-core kernels (bf16, 2e-2) and on the fp32 kernels (1e-4), and
the error codes."""
import numpy as np
import pytest
import torch

import paper_2602_12128_amd as hla
from oracle import hla_oracle as orc
from paper_2602_12128_amd import workloads as wl
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu


def _causal_gpu(t, F, dphi, phi=None, cu=None, decay=1.0):
    dev = torch.device("cuda:0")
    B, H, N, d = t["V"].shape
    nseq = B if cu is None else len(cu) - 1
    h = hla.HLA(head_dim=d, feature_dim=dphi, degree=F, eps=1e-6, io_dtype=hla.HLA_BF16,
                phi_mode=hla.HLA_PHI_NONE if phi is None else hla.HLA_PHI_MLP, max_heads=H,
                max_tokens=B * N, max_seqs=max(nseq, 1), causal=True, decay=decay)
    assert h.active_path == hla.HLA_PATH_MFMA
    if phi is not None:
        h.set_phi_weights([{k: v.to(dev) for k, v in m.items()} for m in phi])
    td = {k: v.to(dev) for k, v in t.items()}
    O = torch.full_like(td["V"], float("nan"))
    h.forward(td["Q"], td["K"], td["V"], O, cu_seqlens=cu)
    torch.cuda.synchronize()
    return h, O.cpu()


def _causal_oracle(t, F, dphi, phi=None, cu=None, decay=1.0):
    Q, K, V = (pu.to_np(t[k]) for k in ("Q", "K", "V"))
    return orc.hla_operator_forward(Q, K, V, F, dphi, 1e-6, phi=pu.oracle_phi(phi), cu_seqlens=cu,
                                    route="bruteforce", causal=True, decay=decay)


@pytest.mark.parametrize("F,dphi,d,B,H,N,kind", [
    (3, 6, 128, 1, 2, 1000, "halfnormal"),   # four chunks, ragged last one
    (3, 6, 64, 2, 3, 777, "lognormal"),
    (2, 12, 128, 1, 2, 600, "halfnormal"),
    (2, 12, 64, 1, 1, 256, "lognormal"),     # exactly one chunk
    (3, 6, 128, 1, 1, 33, "halfnormal"),     # less than two tiles
    (3, 6, 128, 2, 2, 1, "halfnormal"),      # one token: it sees itself only
])
def test_causal_feature_level_bf16(F, dphi, d, B, H, N, kind):
    t = wl.make_feature_inputs(1200 + N, B, H, N, d, F, dphi, torch.bfloat16, kind=kind)
    h, got = _causal_gpu(t, F, dphi)
    h.destroy()
    ref = _causal_oracle(t, F, dphi)
    pu.assert_parity({"O": got}, {"O": ref}, 2e-2, f"causal features F={F} d={d} N={N}")
    if N > 1:  # and it is not the non-causal result
        plain = pu.run_oracle(t, F, dphi, 1e-6, backward=False)["O"]
        assert np.abs(ref - plain).max() > 1e-2 * np.abs(plain).max()


def test_causal_through_feature_maps_packed_no_leak():
    cu = [0, 100, 100, 1500, 1501, 2600]
    t, phi = wl.make_raw_inputs(1210, 1, 2, cu[-1], 128, 3, 6, torch.bfloat16)
    h, got = _causal_gpu(t, 3, 6, phi=phi, cu=cu)
    ref = _causal_oracle(t, 3, 6, phi=phi, cu=cu)
    pu.assert_parity({"O": got}, {"O": ref}, 2e-2, "causal packed through the maps")
    # later tokens never reach earlier ones, inside a sequence or across sequences: perturbing
    # tokens from 2000 on leaves every output before 2000 bit-identical
    t2 = {k: v.clone() for k, v in t.items()}
    for k in ("Q", "K", "V"):
        t2[k][:, :, 2000:] = (t2[k][:, :, 2000:].float() * 1.5 + 0.01).to(torch.bfloat16)
    dev = torch.device("cuda:0")
    td = {k: v.to(dev) for k, v in t2.items()}
    O2 = torch.empty_like(td["V"])
    h.forward(td["Q"], td["K"], td["V"], O2, cu_seqlens=cu)
    torch.cuda.synchronize()
    assert torch.equal(got[:, :, :2000], O2.cpu()[:, :, :2000])
    assert not torch.equal(got[:, :, 2000:], O2.cpu()[:, :, 2000:])
    h.destroy()


def test_causal_video_size_sampled_rows():
    # the 480p video shape (Sec. 5.1) with the causal mask: every output is produced, sampled query
    # rows of three heads are recomputed from the masked definition over all their keys
    w = wl.make_workload(3, need_backward=False)
    h, got = _causal_gpu(w.tensors, w.F, w.d_phi, phi=w.phi)
    h.destroy()
    assert torch.isfinite(got.float()).all()
    ophi = pu.oracle_phi(w.phi)
    rng = np.random.default_rng(7)
    rows = np.sort(np.concatenate([[0, 1, 31, 32, 255, 256, 257, w.N - 1], rng.choice(w.N, 56, replace=False)]))
    worst = 0.0
    for hh in (0, 5, 11):
        K = pu.to_np(w.tensors["K"][0, hh])
        kfs = [orc.phi_forward(K, *ophi[1 + f].astuple())[0] for f in range(w.F)]
        qf = orc.phi_forward(pu.to_np(w.tensors["Q"][0, hh]), *ophi[0].astuple())[0]
        ref = orc.hla_causal_bruteforce(qf, kfs, pu.to_np(w.tensors["V"][0, hh]), w.eps, rows=rows)
        g = pu.to_np(got[0, hh][rows])
        worst = max(worst, float(np.abs(g - ref).max() / np.abs(ref).max()))
    print(f"[parity] causal 480p sampled rows: worst rel err {worst:.2e} (tol 0.02)", flush=True)
    assert worst <= 2e-2


@pytest.mark.parametrize("F,dphi,d,B,H,N,lam", [
    (3, 6, 128, 1, 2, 1000, 0.995),   # slow decay: earlier chunks still count
    (3, 6, 64, 2, 2, 777, 0.9),       # a chunk's worth of distance is gone (0.9^256 = 2e-12)
    (2, 12, 128, 1, 2, 600, 0.98),
    (3, 6, 128, 1, 1, 300, 0.3),      # fast decay: almost only the token itself and its neighbours
    (3, 6, 128, 1, 1, 33, 0.97),
])
def test_causal_decay_feature_level_bf16(F, dphi, d, B, H, N, lam):
    """Decay factors in the causal mask (Sec. 4.4; entries decay^(i-j)) against the oracle's masked
    matrix."""
    t = wl.make_feature_inputs(1300 + N, B, H, N, d, F, dphi, torch.bfloat16, kind="halfnormal")
    h, got = _causal_gpu(t, F, dphi, decay=lam)
    h.destroy()
    ref = _causal_oracle(t, F, dphi, decay=lam)
    pu.assert_parity({"O": got}, {"O": ref}, 2e-2, f"causal decay {lam} F={F} d={d} N={N}")
    nodecay = _causal_oracle(t, F, dphi)
    assert np.abs(ref - nodecay).max() > 1e-2 * np.abs(nodecay).max()  # the factor does something


def test_causal_decay_packed_through_the_maps_and_argument_checks():
    cu = [0, 300, 300, 1324, 1325, 2600]
    t, phi = wl.make_raw_inputs(1310, 1, 2, cu[-1], 128, 3, 6, torch.bfloat16)
    h, got = _causal_gpu(t, 3, 6, phi=phi, cu=cu, decay=0.99)
    h.destroy()
    ref = _causal_oracle(t, 3, 6, phi=phi, cu=cu, decay=0.99)
    pu.assert_parity({"O": got}, {"O": ref}, 2e-2, "causal decay packed through the maps")
    # decay 0 and 1 both mean none: bit-identical outputs
    t2 = wl.make_feature_inputs(1311, 1, 1, 500, 64, 3, 6, torch.bfloat16)
    outs = []
    for lam in (0.0, 1.0):
        h, o = _causal_gpu(t2, 3, 6, decay=lam)
        h.destroy()
        outs.append(o)
    assert torch.equal(outs[0], outs[1])
    for kw in (dict(causal=True, decay=1.5), dict(causal=True, decay=-0.1), dict(causal=False, decay=0.5)):
        with pytest.raises(hla.HLAError) as e:
            hla.HLA(head_dim=128, feature_dim=6, degree=3, io_dtype=hla.HLA_BF16, phi_mode=hla.HLA_PHI_NONE,
                    max_heads=1, max_tokens=8, max_seqs=1, **kw)
        assert e.value.code == 1


def _causal_gpu_backward(t, F, dphi, phi=None, cu=None, decay=1.0):
    dev = torch.device("cuda:0")
    B, H, N, d = t["V"].shape
    nseq = B if cu is None else len(cu) - 1
    h = hla.HLA(head_dim=d, feature_dim=dphi, degree=F, eps=1e-6, io_dtype=hla.HLA_BF16,
                phi_mode=hla.HLA_PHI_NONE if phi is None else hla.HLA_PHI_MLP, max_heads=H,
                max_tokens=B * N, max_seqs=max(nseq, 1), causal=True, decay=decay)
    if phi is not None:
        h.set_phi_weights([{k: v.to(dev) for k, v in m.items()} for m in phi])
    td = {k: v.to(dev) for k, v in t.items()}
    out = {"O": torch.full_like(td["V"], float("nan"))}
    h.forward(td["Q"], td["K"], td["V"], out["O"], cu_seqlens=cu)
    for n, src in (("dQ", "Q"), ("dK", "K"), ("dV", "V")):
        out[n] = torch.full_like(td[src], float("nan"))
    h.backward(td["Q"], td["K"], td["V"], out["O"], td["dO"], out["dQ"], out["dK"], out["dV"], cu_seqlens=cu)
    torch.cuda.synchronize()
    h.destroy()
    return {k: v.cpu() for k, v in out.items()}


def _causal_oracle_backward(t, F, dphi, phi=None, cu=None, decay=1.0):
    Q, K, V, dO = (pu.to_np(t[k]) for k in ("Q", "K", "V", "dO"))
    ophi = pu.oracle_phi(phi)
    O = orc.hla_operator_forward(Q, K, V, F, dphi, 1e-6, phi=ophi, cu_seqlens=cu, route="bruteforce",
                                 causal=True, decay=decay)
    res = orc.hla_operator_backward(Q, K, V, dO, F, dphi, 1e-6, phi=ophi, cu_seqlens=cu, route="bruteforce",
                                    causal=True, decay=decay, feature_grads=True)
    out = {"O": O, "dQ": res[0], "dK": res[1], "dV": res[2]}
    out["_dqf"], out["_dkf"] = res[-1]
    return out


@pytest.mark.parametrize("F,dphi,d,B,H,N,lam,kind", [
    (3, 6, 128, 1, 2, 1000, 1.0, "halfnormal"),   # four chunks, ragged last one
    (3, 6, 64, 2, 2, 777, 0.99, "lognormal"),
    (2, 12, 128, 1, 2, 600, 1.0, "halfnormal"),
    (2, 12, 64, 1, 1, 256, 0.9, "lognormal"),      # exactly one chunk
    (3, 6, 128, 1, 1, 33, 0.97, "halfnormal"),
    (3, 6, 128, 2, 2, 1, 1.0, "halfnormal"),
])
def test_causal_backward_feature_level_bf16(F, dphi, d, B, H, N, lam, kind):
    """Backward of the causal variant (with and without decay) against the oracle's masked-matrix
    route: gradients w.r.t. the features and V."""
    t = wl.make_feature_inputs(1400 + N, B, H, N, d, F, dphi, torch.bfloat16, kind=kind)
    gpu = _causal_gpu_backward(t, F, dphi, decay=lam)
    ref = _causal_oracle_backward(t, F, dphi, decay=lam)
    what = f"causal backward features F={F} d={d} N={N} decay={lam}"
    if N == 1:
        # a token that sees itself only has o = v eta / (eta + eps): its feature gradients are
        # O(eps), far below what bf16 arithmetic resolves; O and dV are compared, the rest is finite
        pu.assert_parity({k: gpu[k] for k in ("O", "dV")}, {k: ref[k] for k in ("O", "dV")}, 2e-2, what)
        assert torch.isfinite(gpu["dQ"].float()).all() and torch.isfinite(gpu["dK"].float()).all()
        return
    pu.assert_parity(gpu, ref, 2e-2, what)


def test_causal_backward_through_feature_maps_packed():
    cu = [0, 300, 300, 1324, 1325, 2600]
    t, phi = wl.make_raw_inputs(1410, 1, 2, cu[-1], 128, 3, 6, torch.bfloat16)
    gpu = _causal_gpu_backward(t, 3, 6, phi=phi, cu=cu, decay=0.995)
    ref = _causal_oracle_backward(t, 3, 6, phi=phi, cu=cu, decay=0.995)
    keep = np.ones(cu[-1], bool)
    keep[1324] = False  # the single-token sequence: O(eps) feature gradients
    kinks = pu.oracle_kinks(t, phi, 3, 6, ref)
    kinks = {k: {key: c for key, c in v.items() if key[2] != 1324} for k, v in kinks.items()}
    sel = lambda dct: {k: (v[:, :, keep] if not k.startswith("_") else v) for k, v in dct.items()}
    # kinks are indexed by the original token positions: compare in full but mask the lone token
    g2 = {k: v.clone() for k, v in gpu.items()}
    r2 = {k: v.copy() for k, v in ref.items()}
    for k in ("dQ", "dK", "dV", "O"):
        g2[k][:, :, 1324] = 0
        r2[k][:, :, 1324] = 0
    pu.assert_parity(g2, r2, 2e-2, "causal backward packed through the maps", kinks=kinks)


def test_causal_backward_twice_after_one_forward_is_bit_identical():
    """The first backward after a forward reuses the forward's chunk states, a second one has to
    compute them again: the same bits either way."""
    dev = torch.device("cuda:0")
    t = wl.make_feature_inputs(1420, 1, 2, 900, 128, 3, 6, torch.bfloat16)
    h = hla.HLA(head_dim=128, feature_dim=6, degree=3, eps=1e-6, io_dtype=hla.HLA_BF16,
                phi_mode=hla.HLA_PHI_NONE, max_heads=2, max_tokens=900, max_seqs=1, causal=True, decay=0.98)
    td = {k: v.to(dev) for k, v in t.items()}
    O = torch.empty_like(td["V"])
    h.forward(td["Q"], td["K"], td["V"], O)
    runs = []
    for _ in range(2):
        g = [torch.full_like(td[k], float("nan")) for k in "QKV"]
        h.backward(td["Q"], td["K"], td["V"], O, td["dO"], *g)
        torch.cuda.synchronize()
        runs.append([x.cpu() for x in g])
    h.destroy()
    for a, b in zip(*runs):
        assert torch.equal(a, b)


def test_causal_video_size_forward_backward_two_heads():
    """The 480p video shape as `bench.py --causal --decay` times it: two whole heads, forward and
    backward, against the oracle's state recursions (the route that is linear in N)."""
    w = wl.make_workload(3)
    lam = 0.999
    gpu = _causal_gpu_backward(w.tensors, w.F, w.d_phi, phi=w.phi, decay=lam)
    for k in ("O", "dQ", "dK", "dV"):
        assert torch.isfinite(gpu[k].float()).all(), k
    heads = [2, 9]
    sub = {k: v[:, heads].contiguous() for k, v in w.tensors.items()}
    Q, K, V, dO = (pu.to_np(sub[k]) for k in ("Q", "K", "V", "dO"))
    ophi = pu.oracle_phi(w.phi)
    ref = {"O": orc.hla_operator_forward(Q, K, V, w.F, w.d_phi, w.eps, phi=ophi, causal=True, decay=lam)}
    res = orc.hla_operator_backward(Q, K, V, dO, w.F, w.d_phi, w.eps, phi=ophi, causal=True, decay=lam,
                                    feature_grads=True)
    ref.update(dQ=res[0], dK=res[1], dV=res[2])
    ref["_dqf"], ref["_dkf"] = res[-1]
    got = {k: gpu[k][:, heads] for k in ("O", "dQ", "dK", "dV")}
    pu.assert_parity(got, ref, 2e-2, f"causal 480p heads {heads}, decay {lam}",
                     kinks=pu.oracle_kinks(sub, w.phi, w.F, w.d_phi, ref))


def test_causal_backward_with_feature_map_weight_gradients():
    """The feature maps' weight gradients (optional outputs of the backward) on a causal handle:
    they are formed from the causal feature gradients."""
    dev = torch.device("cuda:0")
    B, H, N, d, F, dphi, lam = 1, 2, 700, 128, 3, 6, 0.99
    t, phi = wl.make_raw_inputs(1430, B, H, N, d, F, dphi, torch.bfloat16)
    h = hla.HLA(head_dim=d, feature_dim=dphi, degree=F, eps=1e-6, io_dtype=hla.HLA_BF16, phi_mode=hla.HLA_PHI_MLP,
                max_heads=H, max_tokens=B * N, max_seqs=B, causal=True, decay=lam)
    phi_dev = [{k: v.to(dev) for k, v in m.items()} for m in phi]
    h.set_phi_weights(phi_dev)
    wg = [{"d" + k: torch.full(v.shape, float("nan"), dtype=torch.float32, device=dev) for k, v in m.items()}
          for m in phi_dev]
    h.set_phi_weight_grads(wg)
    td = {k: v.to(dev) for k, v in t.items()}
    O = torch.empty_like(td["V"])
    g = [torch.empty_like(td[k]) for k in "QKV"]
    h.forward(td["Q"], td["K"], td["V"], O)
    h.backward(td["Q"], td["K"], td["V"], O, td["dO"], *g)
    torch.cuda.synchronize()
    h.destroy()
    Q, K, V, dO = (pu.to_np(t[k]) for k in ("Q", "K", "V", "dO"))
    res = orc.hla_operator_backward(Q, K, V, dO, F, dphi, 1e-6, phi=pu.oracle_phi(phi), route="bruteforce",
                                    causal=True, decay=lam, weight_grads=True, feature_grads=True)
    ref = {"wg": [dict(zip(pu.WG_KEYS, m)) for m in res[3]]}
    ref["_dqf"], ref["_dkf"] = res[-1]
    br = pu.oracle_weight_grad_branches(t, phi, F, dphi, ref)
    pu.assert_weight_grad_parity([{k: v.cpu() for k, v in m.items()} for m in wg], ref["wg"], 2e-2,
                                 "causal weight gradients", branches=br)


def _vmod(seed, d):
    return wl.draw_vmod_weights(torch.Generator("cpu").manual_seed(seed), d, torch.bfloat16)


@pytest.mark.parametrize("F,dphi,d,B,H,N,lam", [(3, 6, 128, 1, 2, 700, 0.99), (2, 12, 64, 2, 2, 333, 1.0)])
def test_causal_with_value_modulation_forward_backward(F, dphi, d, B, H, N, lam):
    """Sec. 4.5 on top of Sec. 4.4: the modulation acts on the causal output T; the backward takes
    dO through the modulation first and hands dT to the causal operator."""
    t, phi = wl.make_raw_inputs(1440 + N, B, H, N, d, F, dphi, torch.bfloat16)
    vm = _vmod(1441 + N, d)
    gpu = pu.run_gpu(t, F, dphi, 1e-6, phi=phi, path=hla.HLA_PATH_MFMA, vmod=vm, vmod_weight_grads=True,
                     causal=True, decay=lam)
    ref = pu.run_oracle(t, F, dphi, 1e-6, phi=phi, vmod=vm, vmod_weight_grads=True, route="bruteforce",
                        causal=True, decay=lam)
    what = f"causal + value modulation F={F} d={d} N={N} decay={lam}"
    pu.assert_parity(gpu, {k: v for k, v in ref.items() if k != "vwg"}, 2e-2, what,
                     kinks=pu.oracle_kinks(t, phi, F, dphi, ref), row_scale=pu.causal_first_token_rows(t, ref))
    pu.assert_vmod_weight_grad_parity(gpu["vwg"], ref["vwg"], 2e-2, what)
    # neither the unmodulated causal result nor the modulated non-causal one
    plain = pu.run_oracle(t, F, dphi, 1e-6, phi=phi, backward=False, route="bruteforce", causal=True, decay=lam)
    other = pu.run_oracle(t, F, dphi, 1e-6, phi=phi, vmod=vm, backward=False)
    for o in (plain, other):
        assert np.abs(ref["O"] - o["O"]).max() > 1e-2 * np.abs(ref["O"]).max()


def test_causal_with_value_modulation_packed_feature_level():
    cu = [0, 300, 300, 1324, 2600]
    t = wl.make_feature_inputs(1450, 1, 2, cu[-1], 128, 3, 6, torch.bfloat16)
    vm = _vmod(1451, 128)
    gpu = pu.run_gpu(t, 3, 6, 1e-6, cu_seqlens=cu, vmod=vm, causal=True, decay=0.995)
    ref = pu.run_oracle(t, 3, 6, 1e-6, cu_seqlens=cu, vmod=vm, route="bruteforce", causal=True, decay=0.995)
    pu.assert_parity(gpu, ref, 2e-2, "causal + value modulation, packed features")


# ---- the fp32 kernels: the same scan, token tile by token tile, at the fp32 tolerance ------------
@pytest.mark.parametrize("F,dphi,d,B,H,N,lam,kind", [
    (3, 6, 32, 2, 2, 83, 1.0, "halfnormal"),      # ragged last tile of the scan
    (3, 6, 128, 1, 2, 300, 0.97, "lognormal"),
    (2, 12, 64, 1, 3, 1100, 0.995, "halfnormal"),  # crosses a chunk boundary of the token table
    (1, 16, 64, 2, 1, 64, 0.9, "halfnormal"),     # one factor: causal linear attention
    (4, 4, 128, 1, 1, 40, 1.0, "halfnormal"),     # 256 state rows: the scan steps by four tokens
    (3, 6, 64, 2, 2, 1, 1.0, "halfnormal"),       # one token
])
def test_causal_fp32_kernels_feature_level(F, dphi, d, B, H, N, lam, kind):
    t = wl.make_feature_inputs(1500 + N, B, H, N, d, F, dphi, torch.float32, kind=kind)
    gpu = pu.run_gpu(t, F, dphi, 1e-6, path=hla.HLA_PATH_GENERIC, causal=True, decay=lam)
    assert gpu["_path"] == hla.HLA_PATH_GENERIC
    ref = pu.run_oracle(t, F, dphi, 1e-6, route="bruteforce", causal=True, decay=lam)
    what = f"causal fp32 features F={F} dphi={dphi} d={d} N={N} decay={lam}"
    if N == 1:
        pu.assert_parity({k: gpu[k] for k in ("O", "dV")}, {k: ref[k] for k in ("O", "dV")}, 1e-4, what)
        return
    pu.assert_parity(gpu, ref, 1e-4, what, row_scale=pu.causal_first_token_rows(t, ref))
    seq = pu.run_oracle(t, F, dphi, 1e-6, route="factorized", causal=True, decay=lam)  # the state recursions
    pu.assert_parity(gpu, seq, 1e-4, what + " (sequential route)", row_scale=pu.causal_first_token_rows(t, seq))


def test_causal_fp32_kernels_through_the_maps_packed_with_weight_gradients():
    cu = [0, 37, 37, 38, 500, 1300]
    F, dphi, d, H, lam = 3, 6, 64, 2, 0.99
    t, phi = wl.make_raw_inputs(1520, 1, H, cu[-1], d, F, dphi, torch.float32)
    gpu = pu.run_gpu(t, F, dphi, 1e-6, phi=phi, cu_seqlens=cu, path=hla.HLA_PATH_GENERIC, weight_grads=True,
                     causal=True, decay=lam)
    ref = pu.run_oracle(t, F, dphi, 1e-6, phi=phi, cu_seqlens=cu, route="bruteforce", weight_grads=True,
                        causal=True, decay=lam)
    what = "causal fp32 packed through the maps"
    pu.assert_parity(gpu, ref, 1e-4, what, kinks=pu.oracle_kinks(t, phi, F, dphi, ref),
                     row_scale=pu.causal_first_token_rows(t, ref, cu))
    pu.assert_weight_grad_parity(gpu["wg"], ref["wg"], 1e-4, what,
                                 branches=pu.oracle_weight_grad_branches(t, phi, F, dphi, ref, cu_seqlens=cu))


def test_causal_fp32_kernels_with_value_modulation():
    F, dphi, d, B, H, N, lam = 3, 6, 32, 2, 2, 150, 0.98
    t, phi = wl.make_raw_inputs(1530, B, H, N, d, F, dphi, torch.float32)
    vm = wl.draw_vmod_weights(torch.Generator("cpu").manual_seed(1531), d, torch.float32)
    gpu = pu.run_gpu(t, F, dphi, 1e-6, phi=phi, path=hla.HLA_PATH_GENERIC, vmod=vm, vmod_weight_grads=True,
                     causal=True, decay=lam)
    ref = pu.run_oracle(t, F, dphi, 1e-6, phi=phi, vmod=vm, vmod_weight_grads=True, route="bruteforce",
                        causal=True, decay=lam)
    what = "causal fp32 with the value modulation"
    pu.assert_parity(gpu, {k: v for k, v in ref.items() if k != "vwg"}, 1e-4, what,
                     kinks=pu.oracle_kinks(t, phi, F, dphi, ref), row_scale=pu.causal_first_token_rows(t, ref))
    pu.assert_vmod_weight_grad_parity(gpu["vwg"], ref["vwg"], 1e-4, what)


def test_causal_fp32_kernels_against_the_matrix_core_kernels_bf16():
    """Two independent implementations of the scan on the GPU: bf16 inputs through the fp32
    vector-ALU kernels and through the matrix-core kernels agree with each other as both do with the
    oracle."""
    F, dphi, d, B, H, N, lam = 3, 6, 128, 1, 2, 700, 0.99
    t, phi = wl.make_raw_inputs(1540, B, H, N, d, F, dphi, torch.bfloat16)
    a = pu.run_gpu(t, F, dphi, 1e-6, phi=phi, path=hla.HLA_PATH_GENERIC, causal=True, decay=lam)
    b = pu.run_gpu(t, F, dphi, 1e-6, phi=phi, path=hla.HLA_PATH_MFMA, causal=True, decay=lam)
    assert a["_path"] == hla.HLA_PATH_GENERIC and b["_path"] == hla.HLA_PATH_MFMA
    ref = pu.run_oracle(t, F, dphi, 1e-6, phi=phi, route="bruteforce", causal=True, decay=lam)
    kinks = pu.oracle_kinks(t, phi, F, dphi, ref)
    for name, got in (("fp32 kernels", a), ("matrix cores", b)):
        pu.assert_parity(got, ref, 2e-2, f"causal bf16 I/O, {name}", kinks=kinks,
                         row_scale=pu.causal_first_token_rows(t, ref))


def test_causal_packed_video_sizes_one_head_of_two_sequences():
    """The packed configuration (four sequences of 8190 to 32760 tokens in one row) on a causal
    handle with decay, as `bench.py --config 5 --causal` runs it: every sequence starts its own
    scan.  One head of the first two sequences is compared in full (forward and backward) with the
    oracle's state recursions run on each sequence alone; sampled rows of the last sequence with
    the masked definition."""
    w = wl.make_workload(5)
    cu, lam, hh = w.cu_seqlens, 0.9995, 7
    gpu = _causal_gpu_backward(w.tensors, w.F, w.d_phi, phi=w.phi, cu=cu, decay=lam)
    for k in ("O", "dQ", "dK", "dV"):
        assert torch.isfinite(gpu[k].float()).all(), k
    ophi = pu.oracle_phi(w.phi)
    for sq in (0, 1):
        lo, hi = cu[sq], cu[sq + 1]
        sub = {k: v[:, hh:hh + 1, lo:hi].contiguous() for k, v in w.tensors.items()}
        Q, K, V, dO = (pu.to_np(sub[k]) for k in ("Q", "K", "V", "dO"))
        ref = {"O": orc.hla_operator_forward(Q, K, V, w.F, w.d_phi, w.eps, phi=ophi, causal=True, decay=lam)}
        res = orc.hla_operator_backward(Q, K, V, dO, w.F, w.d_phi, w.eps, phi=ophi, causal=True, decay=lam,
                                        feature_grads=True)
        ref.update(dQ=res[0], dK=res[1], dV=res[2])
        ref["_dqf"], ref["_dkf"] = res[-1]
        got = {k: gpu[k][:, hh:hh + 1, lo:hi] for k in ("O", "dQ", "dK", "dV")}
        pu.assert_parity(got, ref, 2e-2, f"causal packed config, sequence {sq} head {hh}",
                         kinks=pu.oracle_kinks(sub, w.phi, w.F, w.d_phi, ref),
                         row_scale=pu.causal_first_token_rows(sub, ref))
    lo, hi = cu[3], cu[4]
    rng = np.random.default_rng(8)
    rows = np.sort(np.concatenate([[0, 1, 255, 256, hi - lo - 1], rng.choice(hi - lo, 27, replace=False)]))
    K = pu.to_np(w.tensors["K"][0, hh, lo:hi])
    kfs = [orc.phi_forward(K, *ophi[1 + f].astuple())[0] for f in range(w.F)]
    qf = orc.phi_forward(pu.to_np(w.tensors["Q"][0, hh, lo:hi]), *ophi[0].astuple())[0]
    ref = orc.hla_causal_bruteforce(qf, kfs, pu.to_np(w.tensors["V"][0, hh, lo:hi]), w.eps, rows=rows, decay=lam)
    g = pu.to_np(gpu["O"][0, hh, lo:hi][rows])
    err = float(np.abs(g - ref).max() / np.abs(ref).max())
    print(f"[parity] causal packed config, sampled rows of the last sequence: {err:.2e} (tol 0.02)", flush=True)
    assert err <= 2e-2


def test_causal_steps_after_the_first_reuse_the_forward_scan_bit_identically():
    """Once a handle has run a backward, its forwards write the backward's image of the running
    state in the same scan launch: the second and third step on a handle give the bits a fresh
    handle gives, also when the inputs change in between and when a forward is repeated without a
    backward."""
    dev = torch.device("cuda:0")
    kw = dict(head_dim=128, feature_dim=6, degree=3, eps=1e-6, io_dtype=hla.HLA_BF16, phi_mode=hla.HLA_PHI_NONE,
              max_heads=2, max_tokens=900, max_seqs=1, causal=True, decay=0.99)
    ta = wl.make_feature_inputs(1460, 1, 2, 900, 128, 3, 6, torch.bfloat16)
    tb = wl.make_feature_inputs(1461, 1, 2, 700, 128, 3, 6, torch.bfloat16, kind="lognormal")

    def step(h, t):
        td = {k: v.to(dev) for k, v in t.items()}
        out = [torch.full_like(td["V"], float("nan"))] + [torch.full_like(td[k], float("nan")) for k in "QKV"]
        h.forward(td["Q"], td["K"], td["V"], out[0])
        h.backward(td["Q"], td["K"], td["V"], out[0], td["dO"], *out[1:])
        torch.cuda.synchronize()
        return [x.cpu() for x in out]

    fresh = {}
    for name, t in (("a", ta), ("b", tb)):
        h = hla.HLA(**kw)
        fresh[name] = step(h, t)
        h.destroy()
    h = hla.HLA(**kw)
    first = step(h, ta)       # scan without the backward's image, the backward makes its own
    second = step(h, ta)      # the forward's scan writes it
    third = step(h, tb)       # other inputs, another length
    td = {k: v.to(dev) for k, v in ta.items()}
    O = torch.empty_like(td["V"])
    h.forward(td["Q"], td["K"], td["V"], O)   # a forward that no backward follows
    fourth = step(h, ta)
    h.destroy()
    for got, want in ((first, fresh["a"]), (second, fresh["a"]), (third, fresh["b"]), (fourth, fresh["a"])):
        for x, y in zip(got, want):
            assert torch.equal(x, y)
    ref = _causal_oracle_backward(ta, 3, 6, decay=0.99)
    pu.assert_parity(dict(zip(("O", "dQ", "dK", "dV"), second)), ref, 2e-2, "causal, second step on a handle",
                     row_scale=pu.causal_first_token_rows(ta, ref))


def test_causal_dense_batch_of_longer_sequences_and_later_steps():
    """A dense batch of two sequences of 20 chunks each (more than one batch of the scans' loads, the
    last one ragged), with decay, the two-factor form: forward and backward against the oracle's
    state recursions, and the second step on the handle (forward scan writing both images) gives
    the bits of the first."""
    dev = torch.device("cuda:0")
    F, dphi, d, B, H, N, lam = 2, 12, 64, 2, 2, 4900, 0.9993
    t = wl.make_feature_inputs(1470, B, H, N, d, F, dphi, torch.bfloat16)
    h = hla.HLA(head_dim=d, feature_dim=dphi, degree=F, eps=1e-6, io_dtype=hla.HLA_BF16, phi_mode=hla.HLA_PHI_NONE,
                max_heads=H, max_tokens=B * N, max_seqs=B, causal=True, decay=lam)
    td = {k: v.to(dev) for k, v in t.items()}

    def step():
        out = [torch.full_like(td["V"], float("nan"))] + [torch.full_like(td[k], float("nan")) for k in "QKV"]
        h.forward(td["Q"], td["K"], td["V"], out[0])
        h.backward(td["Q"], td["K"], td["V"], out[0], td["dO"], *out[1:])
        torch.cuda.synchronize()
        return [x.cpu() for x in out]

    first, second = step(), step()
    h.destroy()
    for x, y in zip(first, second):
        assert torch.equal(x, y)
    Q, K, V, dO = (pu.to_np(t[k]) for k in ("Q", "K", "V", "dO"))
    ref = {"O": orc.hla_operator_forward(Q, K, V, F, dphi, 1e-6, causal=True, decay=lam)}
    res = orc.hla_operator_backward(Q, K, V, dO, F, dphi, 1e-6, causal=True, decay=lam)
    ref.update(dQ=res[0], dK=res[1], dV=res[2])
    pu.assert_parity(dict(zip(("O", "dQ", "dK", "dV"), first)), ref, 2e-2, "causal, dense batch of 4900-token sequences",
                     row_scale=pu.causal_first_token_rows(t, ref))

"""GPU parity of the feature-map weight gradients (optional outputs of hla_backward) against the
CPU oracle through the C ABI: both kernel paths, shared and per-head weights, packed sequences,
ragged sizes, and the registration rules."""
import numpy as np
import pytest
import torch

import paper_2602_12128_amd as hla
from paper_2602_12128_amd import workloads as wl
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu


def _per_head_phi(seed, H, d, d_phi, nmaps, dtype):
    gen = torch.Generator("cpu").manual_seed(seed)
    heads = [wl.draw_phi_weights(gen, d, d_phi, nmaps, dtype) for _ in range(H)]
    return [{k: torch.stack([heads[h][m][k] for h in range(H)]).contiguous() for k in heads[0][m]}
            for m in range(nmaps)]


@pytest.mark.parametrize("F,dphi,d,B,H,N", [(3, 6, 32, 2, 2, 83), (2, 12, 64, 1, 3, 50),
                                             (3, 6, 128, 1, 2, 41), (1, 5, 32, 1, 1, 9)])
def test_weight_grads_fp32_generic_path(F, dphi, d, B, H, N):
    t, phi = wl.make_raw_inputs(700 + N, B, H, N, d, F, dphi, torch.float32)
    gpu = pu.run_gpu(t, F, dphi, 1e-6, phi=phi, path=hla.HLA_PATH_GENERIC, weight_grads=True)
    ref = pu.run_oracle(t, F, dphi, 1e-6, phi=phi, weight_grads=True)
    pu.assert_parity(gpu, ref, 1e-4, f"generic fp32 F={F} d={d} N={N}")
    pu.assert_weight_grad_parity(gpu["wg"], ref["wg"], 1e-4, f"generic fp32 F={F} d={d} N={N}")


@pytest.mark.parametrize("d,B,H,N", [(128, 1, 2, 700), (64, 2, 3, 333), (128, 2, 1, 95), (64, 1, 1, 33),
                                     (64, 1, 4, 4100),    # enough tiles for a full grid of partial sums at d = 64
                                     (128, 1, 2, 8200)])  # and at d = 128
def test_weight_grads_bf16_mfma_path(d, B, H, N):
    t, phi = wl.make_raw_inputs(720 + N, B, H, N, d, 3, 6, torch.bfloat16)
    gpu = pu.run_gpu(t, 3, 6, 1e-6, phi=phi, path=hla.HLA_PATH_MFMA, weight_grads=True)
    assert gpu["_path"] == hla.HLA_PATH_MFMA
    # a weight gradient sums over all tokens, so a token whose pre-ReLU value lies within the
    # feature maps' rounding error of zero cannot be left out of the comparison: the oracle lists
    # those (token, feature) pairs with what each adds when its ReLU is open, and the library's
    # arrays must match the oracle's for one assignment of open / closed to them
    ref = pu.run_oracle(t, 3, 6, 1e-6, phi=phi, weight_grads=True)
    br = pu.oracle_weight_grad_branches(t, phi, 3, 6, ref)
    pu.assert_weight_grad_parity(gpu["wg"], ref["wg"], 2e-2, f"mfma bf16 d={d} N={N}", branches=br)


@pytest.mark.parametrize("path,dtype,tol", [(hla.HLA_PATH_GENERIC, torch.float32, 1e-4),
                                            (hla.HLA_PATH_MFMA, torch.bfloat16, 2e-2)])
def test_per_head_weights_and_their_gradients(path, dtype, tol):
    B, H, N, d = 2, 3, 150, 64
    t, _ = wl.make_raw_inputs(740, B, H, N, d, 3, 6, dtype)
    phi = _per_head_phi(741, H, d, 6, 4, dtype)
    gpu = pu.run_gpu(t, 3, 6, 1e-6, phi=phi, path=path, weight_grads=True, per_head=True)
    ref = pu.run_oracle_per_head(t, 3, 6, 1e-6, phi)
    bf16 = dtype == torch.bfloat16
    pu.assert_parity(gpu, ref, tol, "per-head weights",
                     kinks=pu.oracle_kinks(t, phi, 3, 6, ref, per_head=True) if bf16 else None)
    br = pu.oracle_weight_grad_branches(t, phi, 3, 6, ref, per_head=True) if bf16 else None
    pu.assert_weight_grad_parity(gpu["wg"], ref["wg"], tol, "per-head weights", branches=br)


def test_weight_grads_packed_sequences_bf16():
    cu = [0, 100, 100, 457, 600]
    t, phi = wl.make_raw_inputs(760, 1, 2, 600, 128, 3, 6, torch.bfloat16)
    gpu = pu.run_gpu(t, 3, 6, 1e-6, phi=phi, cu_seqlens=cu, weight_grads=True)
    ref = pu.run_oracle(t, 3, 6, 1e-6, phi=phi, cu_seqlens=cu, weight_grads=True)
    br = pu.oracle_weight_grad_branches(t, phi, 3, 6, ref, cu_seqlens=cu)
    pu.assert_weight_grad_parity(gpu["wg"], ref["wg"], 2e-2, "packed bf16", branches=br)


def test_registration_rules_and_repeatability():
    dev = torch.device("cuda:0")
    t, phi = wl.make_raw_inputs(780, 1, 2, 200, 64, 3, 6, torch.bfloat16)
    td = {k: v.to(dev) for k, v in t.items()}
    phid = [{k: v.to(dev) for k, v in m.items()} for m in phi]
    h = pu.make_handle(t, 3, 6, 1e-6, phi, None)
    mk = lambda: [{"d" + k: torch.full(v.shape, float("nan"), dtype=torch.float32, device=dev)
                   for k, v in m.items()} for m in phid]
    wg = mk()
    with pytest.raises(hla.HLAError) as e:  # no weights registered yet
        h.set_phi_weight_grads(wg)
    assert e.value.code == 5
    h.set_phi_weights(phid)
    with pytest.raises(hla.HLAError) as e:  # wrong number of maps
        h.set_phi_weight_grads(wg[:2])
    assert e.value.code == 1
    h.set_phi_weight_grads(wg)
    O = torch.empty_like(td["V"])
    g = [torch.empty_like(td[k]) for k in "QKV"]
    h.forward(td["Q"], td["K"], td["V"], O)
    h.backward(td["Q"], td["K"], td["V"], O, td["dO"], *g)
    torch.cuda.synchronize()
    first = [{k: v.clone() for k, v in m.items()} for m in wg]
    assert all(torch.isfinite(v).all() for m in first for v in m.values())
    # overwritten, not accumulated, and bit-identical from run to run
    h.backward(td["Q"], td["K"], td["V"], O, td["dO"], *g)
    torch.cuda.synchronize()
    for a, b in zip(first, wg):
        for k in a:
            assert torch.equal(a[k], b[k]), k
    # cleared: the arrays are left alone
    h.set_phi_weight_grads(None)
    for m in wg:
        for v in m.values():
            v.fill_(7.0)
    h.backward(td["Q"], td["K"], td["V"], O, td["dO"], *g)
    torch.cuda.synchronize()
    assert all(bool((v == 7.0).all()) for m in wg for v in m.values())
    h.destroy()
    # feature-level handles have no maps to differentiate
    h2 = hla.HLA(head_dim=64, phi_mode=hla.HLA_PHI_NONE, max_heads=1, max_tokens=8)
    with pytest.raises(hla.HLAError) as e:
        h2.set_phi_weight_grads(wg)
    assert e.value.code == 5
    h2.destroy()


@pytest.mark.parametrize("F,dphi", [(3, 6), (2, 12)])
def test_fewer_heads_than_the_handle_allows_and_empty_input(F, dphi):
    dev = torch.device("cuda:0")
    Hmax, H, N, d = 4, 2, 70, 64
    nmaps, nfeat = 1 + F, (1 + F) * dphi
    t, _ = wl.make_raw_inputs(790, 1, H, N, d, F, dphi, torch.bfloat16)
    phi = _per_head_phi(791, Hmax, d, dphi, nmaps, torch.bfloat16)
    h = hla.HLA(head_dim=d, feature_dim=dphi, degree=F, io_dtype=hla.HLA_BF16, max_heads=Hmax,
                max_tokens=N, max_seqs=1)
    assert h.active_path == hla.HLA_PATH_MFMA
    phid = [{k: v.to(dev) for k, v in m.items()} for m in phi]
    h.set_phi_weights(phid, per_head=True)
    wg = [{"d" + k: torch.full(v.shape, 7.0, dtype=torch.float32, device=dev) for k, v in m.items()}
          for m in phid]
    h.set_phi_weight_grads(wg)
    td = {k: v.to(dev) for k, v in t.items()}
    O = torch.empty_like(td["V"])
    g = [torch.empty_like(td[k]) for k in "QKV"]
    h.forward(td["Q"], td["K"], td["V"], O)
    h.backward(td["Q"], td["K"], td["V"], O, td["dO"], *g)
    torch.cuda.synchronize()
    # heads the call did not cover keep what the arrays held; the others match the oracle
    phi_used = [{k: v[:H] for k, v in m.items()} for m in phi]
    ref = pu.run_oracle_per_head(t, F, dphi, 1e-6, phi_used)
    for m in range(nmaps):
        for k in pu.WG_KEYS:
            assert bool((wg[m][k][H:] == 7.0).all()), (m, k)
    br = pu.oracle_weight_grad_branches(t, phi_used, F, dphi, ref, per_head=True)
    pu.assert_weight_grad_parity([{k: v[:H].cpu() for k, v in m.items()} for m in wg], ref["wg"], 2e-2,
                                 "two of four heads", branches=br)
    # a backward over no tokens writes zeros for the heads it names
    e = {k: v[:, :, :0] for k, v in td.items()}
    Oe = torch.empty_like(e["V"])
    ge = [torch.empty_like(e[k]) for k in "QKV"]
    h.forward(e["Q"], e["K"], e["V"], Oe)
    h.backward(e["Q"], e["K"], e["V"], Oe, e["dO"], *ge)
    torch.cuda.synchronize()
    for m in range(nmaps):
        for k in pu.WG_KEYS:
            assert bool((wg[m][k][:H] == 0.0).all()) and bool((wg[m][k][H:] == 7.0).all()), (m, k)
    # switching to shared weights drops the per-head registration: nothing is written any more
    h.set_phi_weights([{k: v[0].contiguous() for k, v in m.items()} for m in phid])
    for m in wg:
        for v in m.values():
            v.fill_(3.0)
    h.forward(td["Q"], td["K"], td["V"], O)
    h.backward(td["Q"], td["K"], td["V"], O, td["dO"], *g)
    torch.cuda.synchronize()
    assert all(bool((v == 3.0).all()) for m in wg for v in m.values())
    h.destroy()

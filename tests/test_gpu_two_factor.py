"""The two-factor form (F = 2, d_phi = 12; App. A.1, Fig. 4) on the matrix-core path: 78 monomials
in a 96-row symmetric state, feature maps with twelve outputs, weight gradients.  Same oracle,
same tolerances and the same kinds of cases as the three-factor tests."""
import numpy as np
import pytest
import torch

import paper_2602_12128_amd as hla
from oracle import hla_oracle as orc
from paper_2602_12128_amd import workloads as wl
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu

F, DPHI, EPS, TOL = 2, 12, 1e-6, 2e-2


def _mfma(t, **kw):
    gpu = pu.run_gpu(t, F, DPHI, EPS, path=hla.HLA_PATH_MFMA, **kw)
    assert gpu["_path"] == hla.HLA_PATH_MFMA
    return gpu


@pytest.mark.parametrize("B,H,N,d,kind", [(1, 2, 333, 128, "lognormal"), (2, 3, 1000, 64, "halfnormal"),
                                          (1, 1, 31, 128, "halfnormal"), (1, 2, 4097, 64, "lognormal")])
def test_feature_level_forward_backward(B, H, N, d, kind):
    t = wl.make_feature_inputs(800 + N, B, H, N, d, F, DPHI, torch.bfloat16, kind=kind)
    gpu = _mfma(t)
    ref = pu.run_oracle(t, F, DPHI, EPS)
    pu.assert_parity(gpu, ref, TOL, f"two-factor features B{B} H{H} N{N} d{d}")


def test_matches_plain_definition_rows():
    # sampled rows of O against the N x N definition of the attention matrix (Eq. 5 with F = 2)
    t = wl.make_feature_inputs(811, 1, 2, 2500, 128, F, DPHI, torch.bfloat16)
    gpu = _mfma(t, backward=False)
    rows = np.random.default_rng(5).choice(2500, size=48, replace=False)
    for h in range(2):
        kf = pu.to_np(t["K"][0, h])
        ref = orc.hla_bruteforce_rows(pu.to_np(t["Q"][0, h][rows]), [kf[:, :DPHI], kf[:, DPHI:]],
                                      pu.to_np(t["V"][0, h]), EPS)
        got = pu.to_np(gpu["O"][0, h][rows])
        assert np.abs(got - ref).max() <= TOL * np.abs(ref).max()


def test_packed_sequences_with_empty_one_and_no_leak():
    cu = [0, 37, 37, 1200, 1201, 1500]
    t = wl.make_feature_inputs(812, 1, 2, cu[-1], 128, F, DPHI, torch.bfloat16)
    gpu = _mfma(t, cu_seqlens=cu)
    ref = pu.run_oracle(t, F, DPHI, EPS, cu_seqlens=cu)
    pu.assert_parity(gpu, ref, TOL, "two-factor packed")
    t2 = {k: v.clone() for k, v in t.items()}
    t2["K"][:, :, :37] = (t2["K"][:, :, :37].float() * 1.5).to(torch.bfloat16)
    t2["V"][:, :, :37] = (t2["V"][:, :, :37].float() - 1.0).to(torch.bfloat16)
    gpu2 = _mfma(t2, cu_seqlens=cu)
    for k in ("O", "dQ", "dK", "dV"):
        assert torch.equal(gpu[k][:, :, 37:], gpu2[k][:, :, 37:]), k
    assert not torch.equal(gpu["O"][:, :, :37], gpu2["O"][:, :, :37])


def test_bit_reproducible():
    t = wl.make_feature_inputs(813, 1, 3, 3000, 64, F, DPHI, torch.bfloat16)
    a, b = _mfma(t), _mfma(t)
    for k in ("O", "dQ", "dK", "dV"):
        assert torch.equal(a[k], b[k]), k


@pytest.mark.parametrize("B,H,N,d", [(1, 2, 700, 128), (2, 2, 300, 64), (1, 3, 1031, 128)])
def test_feature_maps_forward_backward(B, H, N, d):
    t, phi = wl.make_raw_inputs(820 + N, B, H, N, d, F, DPHI, torch.bfloat16)
    gpu = _mfma(t, phi=phi)
    ref = pu.run_oracle(t, F, DPHI, EPS, phi=phi)
    pu.assert_parity(gpu, ref, TOL, f"two-factor maps B{B} H{H} N{N} d{d}",
                     kinks=pu.oracle_kinks(t, phi, F, DPHI, ref))


@pytest.mark.parametrize("B,H,N,d,per_head", [(1, 2, 700, 128, False), (2, 3, 333, 64, False),
                                               (1, 2, 450, 128, True)])
def test_weight_gradients(B, H, N, d, per_head):
    t, phi = wl.make_raw_inputs(830 + N, B, H, N, d, F, DPHI, torch.bfloat16)
    if per_head:  # every head its own weights: arrays with a leading head dimension
        gen = torch.Generator("cpu").manual_seed(831)
        heads = [wl.draw_phi_weights(gen, d, DPHI, 1 + F, torch.bfloat16) for _ in range(H)]
        phi = [{k: torch.stack([heads[h][m][k] for h in range(H)]).contiguous() for k in heads[0][m]}
               for m in range(1 + F)]
    gpu = _mfma(t, phi=phi, weight_grads=True, per_head=per_head)
    if per_head:
        ref = pu.run_oracle_per_head(t, F, DPHI, EPS, phi)
    else:
        ref = pu.run_oracle(t, F, DPHI, EPS, phi=phi, weight_grads=True)
    pu.assert_parity(gpu, ref, TOL, f"two-factor outputs N{N} d{d}",
                     kinks=pu.oracle_kinks(t, phi, F, DPHI, ref, per_head=per_head))
    br = pu.oracle_weight_grad_branches(t, phi, F, DPHI, ref, per_head=per_head)
    pu.assert_weight_grad_parity(gpu["wg"], ref["wg"], TOL, f"two-factor weight grads N{N} d{d}", branches=br)


def test_video_size_forward_backward():
    # the two-factor workload at the 480p video shape, as bench.py --config 7 times it
    w = wl.make_workload(7)
    assert w.tensors["V"].shape == (1, 12, 32760, 128) and (w.F, w.d_phi) == (F, DPHI)
    gpu = pu.run_gpu(w.tensors, w.F, w.d_phi, w.eps, phi=w.phi)
    assert gpu["_path"] == hla.HLA_PATH_MFMA
    for k in ("O", "dQ", "dK", "dV"):
        assert torch.isfinite(gpu[k].float()).all(), k
    heads = [0, 7]
    sub = {k: v[:, heads].contiguous() for k, v in w.tensors.items()}
    ref = pu.run_oracle(sub, w.F, w.d_phi, w.eps, phi=w.phi)
    pu.assert_parity({k: gpu[k][:, heads] for k in ref if not k.startswith("_")}, ref, TOL,
                     "two-factor 480p heads 0,7", kinks=pu.oracle_kinks(sub, w.phi, w.F, w.d_phi, ref))
    ophi = pu.oracle_phi(w.phi)
    rows = np.random.default_rng(w.seed + 99).choice(w.N, size=64, replace=False)
    for hh in (3, 11):
        K = pu.to_np(w.tensors["K"][0, hh])
        kfs = [orc.phi_forward(K, *ophi[1 + f].astuple())[0] for f in range(F)]
        qf = orc.phi_forward(pu.to_np(w.tensors["Q"][0, hh][rows]), *ophi[0].astuple())[0]
        ref_rows = orc.hla_bruteforce_rows(qf, kfs, pu.to_np(w.tensors["V"][0, hh]), w.eps)
        got = pu.to_np(gpu["O"][0, hh][rows])
        assert np.abs(got - ref_rows).max() <= TOL * np.abs(pu.to_np(gpu["O"][0, hh])).max()

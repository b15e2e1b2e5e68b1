"""GPU parity of the generic (fp32 vector-ALU, literal d_phi^F state) path against the CPU
oracle, element by element, through the C ABI.  Sizes span several tiles and chunks with
ragged tails; edge cases cover empty input, packed sequences and error codes."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2602_12128_amd as hla
from paper_2602_12128_amd import workloads as wl
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu


def test_config1_tiny_forward_fp32_both_oracle_routes():
    w = wl.make_workload(1)
    assert w.tensors["V"].shape == (1, 2, 256, 32) and w.dtype == torch.float32
    gpu = pu.run_gpu(w.tensors, w.F, w.d_phi, w.eps, phi=w.phi, backward=False)
    for route in ("factorized", "bruteforce"):
        ref = pu.run_oracle(w.tensors, w.F, w.d_phi, w.eps, phi=w.phi, backward=False, route=route)
        pu.assert_parity(gpu, ref, 1e-4, f"config 1 vs oracle {route}")


@pytest.mark.parametrize("F,dphi,d,N,kind", [
    (3, 6, 32, 300, "halfnormal"),
    (3, 6, 128, 1100, "lognormal"),   # crosses the 1024-token chunk boundary
    (2, 12, 64, 257, "sparse"),
    (1, 16, 32, 65, "halfnormal"),
    (4, 4, 64, 130, "halfnormal"),
])
def test_feature_level_forward_backward_fp32(F, dphi, d, N, kind):
    t = wl.make_feature_inputs(100 + N, 2, 3, N, d, F, dphi, torch.float32, kind=kind)
    gpu = pu.run_gpu(t, F, dphi, 1e-6, path=hla.HLA_PATH_GENERIC)
    assert gpu["_path"] == hla.HLA_PATH_GENERIC
    ref = pu.run_oracle(t, F, dphi, 1e-6)
    pu.assert_parity(gpu, ref, 1e-4, f"generic fp32 F={F} dphi={dphi} d={d} N={N} {kind}")


def test_single_token_sequence():
    # N = 1: o = v * eta / (eta + eps); the feature gradients cancel down to O(eps), so they are
    # compared on the scale of their two cancelling terms (|dO| |v|), not of the tiny remainder.
    t = wl.make_feature_inputs(101, 2, 3, 1, 128, 3, 5, torch.float32)
    gpu = pu.run_gpu(t, 3, 5, 1e-6, path=hla.HLA_PATH_GENERIC)
    ref = pu.run_oracle(t, 3, 5, 1e-6)
    pu.assert_parity({k: gpu[k] for k in ("O", "dV")}, {k: ref[k] for k in ("O", "dV")}, 1e-4,
                     "generic single token")
    scale = float(t["dO"].abs().max() * t["V"].abs().max())
    for k in ("dQ", "dK"):
        assert np.abs(pu.to_np(gpu[k]) - ref[k]).max() <= 1e-4 * scale


@pytest.mark.parametrize("d,N,b2", [(32, 77, 2.0), (64, 200, 0.5), (128, 1030, 2.0)])
def test_feature_maps_forward_backward_fp32(d, N, b2):
    t, phi = wl.make_raw_inputs(200 + N, 1, 2, N, d, 3, 6, torch.float32, b2_mean=b2)
    gpu = pu.run_gpu(t, 3, 6, 1e-6, phi=phi, path=hla.HLA_PATH_GENERIC)
    ref = pu.run_oracle(t, 3, 6, 1e-6, phi=phi)
    pu.assert_parity(gpu, ref, 1e-4, f"generic fp32 phi d={d} N={N} b2={b2}")


def test_bf16_io_on_generic_path():
    t, phi = wl.make_raw_inputs(7, 2, 2, 530, 64, 3, 6, torch.bfloat16)
    gpu = pu.run_gpu(t, 3, 6, 1e-6, phi=phi, path=hla.HLA_PATH_GENERIC)
    ref = pu.run_oracle(t, 3, 6, 1e-6, phi=phi)
    pu.assert_parity(gpu, ref, 2e-2, "generic bf16 phi")
    t = wl.make_feature_inputs(8, 1, 2, 333, 128, 2, 12, torch.bfloat16, kind="lognormal")
    gpu = pu.run_gpu(t, 2, 12, 1e-6, path=hla.HLA_PATH_GENERIC)
    ref = pu.run_oracle(t, 2, 12, 1e-6)
    pu.assert_parity(gpu, ref, 2e-2, "generic bf16 features F=2")


def test_packed_sequences_with_empty_one_and_no_leak():
    cu = [0, 37, 37, 1200, 1201, 1500]
    N = cu[-1]
    t = wl.make_feature_inputs(9, 1, 2, N, 32, 3, 6, torch.float32)
    gpu = pu.run_gpu(t, 3, 6, 1e-6, cu_seqlens=cu, path=hla.HLA_PATH_GENERIC)
    ref = pu.run_oracle(t, 3, 6, 1e-6, cu_seqlens=cu)
    pu.assert_parity(gpu, ref, 1e-4, "generic packed")
    # perturb sequence 0's keys and values: every other sequence must be bit-identical
    t2 = {k: v.clone() for k, v in t.items()}
    t2["K"][:, :, :37] += 0.5
    t2["V"][:, :, :37] -= 1.0
    gpu2 = pu.run_gpu(t2, 3, 6, 1e-6, cu_seqlens=cu, path=hla.HLA_PATH_GENERIC)
    for k in ("O", "dQ", "dK", "dV"):
        assert torch.equal(gpu[k][:, :, 37:], gpu2[k][:, :, 37:]), k
    assert not torch.equal(gpu["O"][:, :, :37], gpu2["O"][:, :, :37])


def test_strided_views_and_repeatability():
    # tensors stored [B, N, H, w] and viewed as [B, H, N, w]
    B, H, N, d, F, dphi = 2, 3, 150, 64, 3, 6
    t = wl.make_feature_inputs(10, B, H, N, d, F, dphi, torch.float32)
    ts = {k: v.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for k, v in t.items()}
    assert not ts["V"].is_contiguous()
    dev = torch.device("cuda:0")
    td = {k: v.to(dev).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for k, v in t.items()}
    h = pu.make_handle(t, F, dphi, 1e-6, None, None, hla.HLA_PATH_GENERIC)
    outs = []
    for rep in range(2):
        O = torch.empty(B, N, H, d, device=dev).permute(0, 2, 1, 3)
        dQ = torch.empty(B, N, H, dphi, device=dev).permute(0, 2, 1, 3)
        dK = torch.empty(B, N, H, F * dphi, device=dev).permute(0, 2, 1, 3)
        dV = torch.empty(B, N, H, d, device=dev).permute(0, 2, 1, 3)
        h.forward(td["Q"], td["K"], td["V"], O)
        h.backward(td["Q"], td["K"], td["V"], O, td["dO"], dQ, dK, dV)
        torch.cuda.synchronize()
        outs.append({"O": O.cpu(), "dQ": dQ.cpu(), "dK": dK.cpu(), "dV": dV.cpu()})
    h.destroy()
    ref = pu.run_oracle(t, F, dphi, 1e-6)
    pu.assert_parity(outs[0], ref, 1e-4, "generic strided")
    for k in outs[0]:
        assert torch.equal(outs[0][k], outs[1][k]), f"{k} not bit-reproducible"


def test_empty_inputs_and_error_codes():
    dev = torch.device("cuda:0")
    h = hla.HLA(head_dim=32, feature_dim=6, degree=3, io_dtype=hla.HLA_F32,
                phi_mode=hla.HLA_PHI_NONE, kernel_path=hla.HLA_PATH_GENERIC, max_heads=2,
                max_tokens=64, max_seqs=2)
    z = lambda w: torch.zeros(1, 2, 0, w, device=dev)
    h.forward(z(6), z(18), z(32), z(32))  # N = 0: nothing to do, no error
    h.backward(z(6), z(18), z(32), z(32), z(32), z(6), z(18), z(32))
    t = {k: v.to(dev) for k, v in wl.make_feature_inputs(1, 1, 2, 16, 32, 3, 6, torch.float32).items()}
    O = torch.empty_like(t["V"])
    g = [torch.empty_like(t[k]) for k in ("Q", "K", "V")]
    with pytest.raises(hla.HLAError) as e:  # backward before forward
        h.backward(t["Q"], t["K"], t["V"], O, t["dO"], *g)
    assert e.value.code == 5
    with pytest.raises(hla.HLAError) as e:  # more tokens than the handle was sized for
        big = {k: torch.zeros(1, 2, 65, v.shape[-1], device=dev) for k, v in t.items()}
        h.forward(big["Q"], big["K"], big["V"], torch.empty_like(big["V"]))
    assert e.value.code == 1
    with pytest.raises(hla.HLAError) as e:  # cu_seqlens not ending at N
        h.forward(t["Q"], t["K"], t["V"], O, cu_seqlens=[0, 8, 15])
    assert e.value.code == 1
    with pytest.raises(hla.HLAError) as e:  # decreasing cu_seqlens
        h.forward(t["Q"], t["K"], t["V"], O, cu_seqlens=[0, 9, 8, 16][:3] + [16])
    assert e.value.code == 1
    with pytest.raises(hla.HLAError) as e:  # weights make no sense without feature maps
        h.set_phi_weights([{k: torch.zeros(1, device=dev) for k in ("W1", "b1", "W2", "b2")}] * 4)
    assert e.value.code == 5
    h.forward(t["Q"], t["K"], t["V"], O)  # the handle still works after the errors
    torch.cuda.synchronize()
    assert torch.isfinite(O).all()
    h.destroy()
    hm = hla.HLA(head_dim=32, feature_dim=6, degree=3, io_dtype=hla.HLA_F32,
                 phi_mode=hla.HLA_PHI_MLP, kernel_path=hla.HLA_PATH_GENERIC, max_heads=2,
                 max_tokens=64, max_seqs=1)
    with pytest.raises(hla.HLAError) as e:  # feature maps never registered
        hm.forward(torch.zeros(1, 2, 16, 32, device=dev), torch.zeros(1, 2, 16, 32, device=dev),
                   t["V"], O)
    assert e.value.code == 5
    hm.destroy()


def test_all_features_clipped_gives_zero_output():
    # eta = 0 for a query whose features are all zero: 0 / (0 + eps) = 0 exactly
    t = wl.make_feature_inputs(11, 1, 1, 40, 32, 3, 6, torch.float32)
    t["Q"][0, 0, 5] = 0.0
    gpu = pu.run_gpu(t, 3, 6, 1e-6, path=hla.HLA_PATH_GENERIC)
    assert torch.all(gpu["O"][0, 0, 5] == 0.0)
    ref = pu.run_oracle(t, 3, 6, 1e-6)
    pu.assert_parity(gpu, ref, 1e-4, "generic zero-feature query")

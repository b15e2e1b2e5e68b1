"""GPU parity of the value modulation (Sec. 4.5: O = T + phi_v1(T) * phi_v2(V), phi_v of App. A.1
with a LayerNorm on its output) through the C ABI: forward and backward on both kernel paths,
feature-level and through the feature maps, packed sequences, strided views, switching it off."""
import numpy as np
import pytest
import torch

import paper_2602_12128_amd as hla
from paper_2602_12128_amd import workloads as wl
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu


def _vmod(seed, d, dtype):
    return wl.draw_vmod_weights(torch.Generator("cpu").manual_seed(seed), d, dtype)


@pytest.mark.parametrize("F,dphi,d,B,H,N", [(3, 6, 32, 2, 2, 83), (2, 12, 64, 1, 3, 150), (3, 6, 128, 1, 2, 70)])
def test_value_modulation_fp32_generic_path(F, dphi, d, B, H, N):
    t, phi = wl.make_raw_inputs(1100 + N, B, H, N, d, F, dphi, torch.float32)
    vm = _vmod(1101 + N, d, torch.float32)
    gpu = pu.run_gpu(t, F, dphi, 1e-6, phi=phi, path=hla.HLA_PATH_GENERIC, vmod=vm)
    ref = pu.run_oracle(t, F, dphi, 1e-6, phi=phi, vmod=vm)
    pu.assert_parity(gpu, ref, 1e-4, f"value modulation fp32 F={F} d={d} N={N}")
    plain = pu.run_oracle(t, F, dphi, 1e-6, phi=phi, backward=False)
    assert np.abs(ref["O"] - plain["O"]).max() > 0.1 * np.abs(plain["O"]).max()  # it does something


@pytest.mark.parametrize("F,dphi,d,B,H,N", [(3, 6, 128, 1, 2, 700), (2, 12, 64, 2, 3, 333), (3, 6, 128, 2, 1, 2049)])
def test_value_modulation_bf16_mfma_path(F, dphi, d, B, H, N):
    t, phi = wl.make_raw_inputs(1120 + N, B, H, N, d, F, dphi, torch.bfloat16)
    vm = _vmod(1121 + N, d, torch.bfloat16)
    gpu = pu.run_gpu(t, F, dphi, 1e-6, phi=phi, path=hla.HLA_PATH_MFMA, vmod=vm)
    assert gpu["_path"] == hla.HLA_PATH_MFMA
    ref = pu.run_oracle(t, F, dphi, 1e-6, phi=phi, vmod=vm)
    pu.assert_parity(gpu, ref, 2e-2, f"value modulation bf16 F={F} d={d} N={N}",
                     kinks=pu.oracle_kinks(t, phi, F, dphi, ref))


def test_value_modulation_feature_level_packed_bf16():
    cu = [0, 100, 100, 1500, 1501, 2600]
    t = wl.make_feature_inputs(1140, 1, 2, cu[-1], 128, 3, 6, torch.bfloat16)
    vm = _vmod(1141, 128, torch.bfloat16)
    gpu = pu.run_gpu(t, 3, 6, 1e-6, cu_seqlens=cu, vmod=vm)
    ref = pu.run_oracle(t, 3, 6, 1e-6, cu_seqlens=cu, vmod=vm)
    keep = np.ones(cu[-1], bool)
    keep[1500] = False  # the single-token sequence: O(eps) feature gradients, compared apart elsewhere
    pu.assert_parity({k: v[:, :, keep] for k, v in gpu.items() if k != "_path"},
                     {k: v[:, :, keep] for k, v in ref.items()}, 2e-2, "value modulation packed")


def test_switching_the_modulation_off_and_on():
    dev = torch.device("cuda:0")
    t = wl.make_feature_inputs(1150, 1, 2, 500, 64, 3, 6, torch.bfloat16)
    vm = _vmod(1151, 64, torch.bfloat16)
    td = {k: v.to(dev) for k, v in t.items()}
    h = pu.make_handle(t, 3, 6, 1e-6, None, None)
    O = [torch.empty_like(td["V"]) for _ in range(3)]
    g = [torch.empty_like(td[k]) for k in "QKV"]
    h.forward(td["Q"], td["K"], td["V"], O[0])
    h.set_value_modulation([{k: v.to(dev) for k, v in m.items()} for m in vm])
    with pytest.raises(hla.HLAError) as e:  # the saved forward was made without the modulation
        h.backward(td["Q"], td["K"], td["V"], O[0], td["dO"], *g)
    assert e.value.code == 5
    h.forward(td["Q"], td["K"], td["V"], O[1])
    h.backward(td["Q"], td["K"], td["V"], O[1], td["dO"], *g)
    h.set_value_modulation(None)
    h.forward(td["Q"], td["K"], td["V"], O[2])
    torch.cuda.synchronize()
    assert torch.equal(O[0], O[2]) and not torch.equal(O[0], O[1])
    with pytest.raises(hla.HLAError) as e:
        h.set_value_modulation([{k: v.to(dev) for k, v in m.items()} for m in vm], ln_eps=-1.0)
    assert e.value.code == 1
    h.destroy()


@pytest.mark.parametrize("dtype,path,F,dphi,d,B,H,N,tol", [
    (torch.float32, hla.HLA_PATH_GENERIC, 3, 6, 32, 2, 2, 83, 1e-4),
    (torch.float32, hla.HLA_PATH_GENERIC, 2, 12, 64, 1, 3, 150, 1e-4),
    (torch.bfloat16, hla.HLA_PATH_MFMA, 3, 6, 128, 1, 2, 700, 2e-2),
    (torch.bfloat16, hla.HLA_PATH_MFMA, 2, 12, 64, 2, 3, 333, 2e-2),
    # mostly padding in the last tile: rows that are not tokens must not reach the sums over tokens
    (torch.bfloat16, hla.HLA_PATH_MFMA, 3, 6, 128, 1, 2, 40, 2e-2),
    (torch.bfloat16, hla.HLA_PATH_MFMA, 3, 6, 64, 2, 1, 33, 2e-2),
])
def test_modulation_weight_gradients(dtype, path, F, dphi, d, B, H, N, tol):
    """Gradients of the two maps' own weights (summed over all tokens of all heads) next to the
    input gradients, which registering them must not change."""
    t, phi = wl.make_raw_inputs(1160 + N, B, H, N, d, F, dphi, dtype)
    vm = _vmod(1161 + N, d, dtype)
    gpu = pu.run_gpu(t, F, dphi, 1e-6, phi=phi, path=path, vmod=vm, vmod_weight_grads=True)
    ref = pu.run_oracle(t, F, dphi, 1e-6, phi=phi, vmod=vm, vmod_weight_grads=True)
    pu.assert_vmod_weight_grad_parity(gpu["vwg"], ref["vwg"], tol, f"modulation weight grads {dtype} d={d} N={N}")
    plain = pu.run_gpu(t, F, dphi, 1e-6, phi=phi, path=path, vmod=vm)
    for k in ("O", "dQ", "dK", "dV"):
        assert torch.equal(gpu[k], plain[k]), k


def test_modulation_weight_gradients_registration_rules():
    dev = torch.device("cuda:0")
    t = wl.make_feature_inputs(1170, 1, 2, 100, 64, 3, 6, torch.bfloat16)
    vm = _vmod(1171, 64, torch.bfloat16)
    td = {k: v.to(dev) for k, v in t.items()}
    h = pu.make_handle(t, 3, 6, 1e-6, None, None)
    grads = [{"d" + k: torch.full(v.shape, float("nan"), dtype=torch.float32, device=dev) for k, v in m.items()}
             for m in vm]
    with pytest.raises(hla.HLAError) as e:  # the modulation is off
        h.set_value_modulation_grads(grads)
    assert e.value.code == 5
    h.set_value_modulation([{k: v.to(dev) for k, v in m.items()} for m in vm])
    h.set_value_modulation_grads(grads)
    O = torch.empty_like(td["V"])
    g = [torch.empty_like(td[k]) for k in "QKV"]
    h.forward(td["Q"], td["K"], td["V"], O)
    h.backward(td["Q"], td["K"], td["V"], O, td["dO"], *g)
    torch.cuda.synchronize()
    assert all(torch.isfinite(a).all() for m in grads for a in m.values())
    first = [{k: v.clone() for k, v in m.items()} for m in grads]
    h.backward(td["Q"], td["K"], td["V"], O, td["dO"], *g)  # overwritten, not accumulated; deterministic
    torch.cuda.synchronize()
    assert all(torch.equal(a[k], b[k]) for a, b in zip(first, grads) for k in a)
    h.set_value_modulation(None)  # clears the registration
    for m in grads:
        for a in m.values():
            a.fill_(7.0)
    h.forward(td["Q"], td["K"], td["V"], O)
    h.backward(td["Q"], td["K"], td["V"], O, td["dO"], *g)
    torch.cuda.synchronize()
    assert all((a == 7.0).all() for m in grads for a in m.values())
    h.destroy()


def test_value_modulation_video_size_two_heads():
    """The 480p video shape as `bench.py --value-modulation --weight-grads` times it: two whole heads
    of O, dQ, dK, dV against the oracle; the modulation's weight gradients (sums over all heads)
    against the oracle run on every head would take minutes, so they are checked for these two
    heads alone in a second call on the sliced tensors."""
    w = wl.make_workload(3)
    vm = _vmod(1180, w.d, torch.bfloat16)
    gpu = pu.run_gpu(w.tensors, w.F, w.d_phi, w.eps, phi=w.phi, vmod=vm)
    assert gpu["_path"] == hla.HLA_PATH_MFMA
    heads = [1, 10]
    sub = {k: v[:, heads].contiguous() for k, v in w.tensors.items()}
    ref = pu.run_oracle(sub, w.F, w.d_phi, w.eps, phi=w.phi, vmod=vm, vmod_weight_grads=True)
    got = {k: gpu[k][:, heads] for k in ("O", "dQ", "dK", "dV")}
    pu.assert_parity(got, {k: v for k, v in ref.items() if k != "vwg"}, 2e-2, f"value modulation 480p heads {heads}",
                     kinks=pu.oracle_kinks(sub, w.phi, w.F, w.d_phi, ref))
    gsub = pu.run_gpu(sub, w.F, w.d_phi, w.eps, phi=w.phi, vmod=vm, vmod_weight_grads=True)
    # (the chunking of the state sums depends on the number of heads in the call, so the two calls
    # agree to rounding, not bit for bit)
    for k in ("O", "dQ", "dK", "dV"):
        assert pu.max_rel_err(pu.to_np(gsub[k]), pu.to_np(gpu[k][:, heads])) < 1e-2, k
    pu.assert_vmod_weight_grad_parity(gsub["vwg"], ref["vwg"], 2e-2, "modulation weight grads 480p two heads")

"""Parity at the five benchmark configurations, in the launch configuration bench.py times
(AUTO path, full sizes).  Small configurations are compared in full; at the video-DiT sizes the
GPU runs the full problem and the oracle recomputes (a) every output of a subset of heads with
its factorized route and (b) sampled query rows of other heads by brute force over all keys."""
import numpy as np
import pytest
import torch

import paper_2602_12128_amd as hla
from oracle import hla_oracle as orc
from paper_2602_12128_amd import workloads as wl
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu



def _head_slice(tensors, heads):
    return {k: v[:, heads].contiguous() for k, v in tensors.items()}


def _check_heads(w, gpu, heads, tol, what):
    sub = _head_slice(w.tensors, heads)
    ref = pu.run_oracle(sub, w.F, w.d_phi, w.eps, phi=w.phi, cu_seqlens=w.cu_seqlens,
                        backward=w.backward)
    got = {k: gpu[k][:, heads] for k in ref if not k.startswith("_")}
    # tokens with a pre-ReLU value within the feature maps' rounding error of zero: their dQ / dK
    # rows must equal one of the branch choices the oracle enumerates
    kinks = pu.oracle_kinks(sub, w.phi, w.F, w.d_phi, ref) if w.backward else None
    return pu.assert_parity(got, ref, tol, what, kinks=kinks)


def _check_bruteforce_rows(w, gpu, heads, rows_per_head, tol, what):
    """Forward outputs of sampled query rows against the plain N x N definition."""
    rng = np.random.default_rng(w.seed + 99)
    ophi = pu.oracle_phi(w.phi)
    units = [(0, w.N)] if w.cu_seqlens is None else list(zip(w.cu_seqlens[:-1], w.cu_seqlens[1:]))
    worst = 0.0
    for hh in heads:
        for (lo, hi) in units:
            if hi == lo:
                continue
            K = pu.to_np(w.tensors["K"][0, hh, lo:hi])
            V = pu.to_np(w.tensors["V"][0, hh, lo:hi])
            kfs = [orc.phi_forward(K, *ophi[1 + f].astuple())[0] for f in range(w.F)]
            rows = rng.choice(hi - lo, size=min(rows_per_head, hi - lo), replace=False)
            Q = pu.to_np(w.tensors["Q"][0, hh, lo:hi][rows])
            qf = orc.phi_forward(Q, *ophi[0].astuple())[0]
            ref = orc.hla_bruteforce_rows(qf, kfs, V, w.eps)
            got = pu.to_np(gpu["O"][0, hh, lo:hi][rows])
            scale = np.abs(pu.to_np(gpu["O"][0, hh, lo:hi])).max()
            worst = max(worst, float(np.abs(got - ref).max() / scale))
    print(f"[parity] {what}: brute-force rows worst rel err {worst:.2e} (tol {tol:g})", flush=True)
    assert worst <= tol


def test_config2_mid_forward_backward_bf16_full():
    w = wl.make_workload(2)
    gpu = pu.run_gpu(w.tensors, w.F, w.d_phi, w.eps, phi=w.phi)
    assert gpu["_path"] == hla.HLA_PATH_MFMA
    ref = pu.run_oracle(w.tensors, w.F, w.d_phi, w.eps, phi=w.phi)
    kinks = pu.oracle_kinks(w.tensors, w.phi, w.F, w.d_phi, ref)
    pu.assert_parity(gpu, ref, 2e-2, "config 2 full", kinks=kinks)


@pytest.mark.parametrize("h0", [0, 4, 8])
def test_config3_dit480p_forward_backward_bf16(h0):
    # every head against the factorized oracle, four per test case (the oracle's memory, and a case
    # stays well under two minutes)
    w = wl.make_workload(3)
    assert w.tensors["V"].shape == (1, 12, 32760, 128)
    gpu = pu.run_gpu(w.tensors, w.F, w.d_phi, w.eps, phi=w.phi)
    assert gpu["_path"] == hla.HLA_PATH_MFMA
    for k in ("O", "dQ", "dK", "dV"):
        assert torch.isfinite(gpu[k].float()).all(), k
    heads = list(range(h0, h0 + 4))
    _check_heads(w, gpu, heads, 2e-2, f"config 3 heads {heads} (factorized oracle)")


def test_config3_dit480p_bruteforce_rows():
    w = wl.make_workload(3)
    gpu = pu.run_gpu(w.tensors, w.F, w.d_phi, w.eps, phi=w.phi, backward=False)
    _check_bruteforce_rows(w, gpu, [3, 11], 64, 2e-2, "config 3 heads 3,11")


def test_second_resolution_12600_tokens_forward_backward_bf16():
    # the lower of the paper's two video resolutions (Sec. 5.1: 81x320x480 -> 12600 tokens), as
    # bench.py --config 6 times it: every head against the factorized oracle
    w = wl.make_workload(6)
    assert w.tensors["V"].shape == (1, 12, 12600, 128)
    gpu = pu.run_gpu(w.tensors, w.F, w.d_phi, w.eps, phi=w.phi)
    assert gpu["_path"] == hla.HLA_PATH_MFMA
    for h0 in range(0, 12, 6):
        heads = list(range(h0, h0 + 6))
        _check_heads(w, gpu, heads, 2e-2, f"12600-token resolution heads {heads}")
    _check_bruteforce_rows(w, gpu, [2, 9], 64, 2e-2, "12600-token resolution heads 2,9")


def test_config4_dit720p_forward_bf16():
    w = wl.make_workload(4)
    assert w.tensors["V"].shape == (1, 40, 75600, 128) and not w.backward
    gpu = pu.run_gpu(w.tensors, w.F, w.d_phi, w.eps, phi=w.phi, backward=False)
    assert torch.isfinite(gpu["O"].float()).all()
    _check_heads(w, gpu, [0, 13, 26, 39], 2e-2, "config 4 heads 0,13,26,39 (factorized oracle)")
    _check_bruteforce_rows(w, gpu, [17], 64, 2e-2, "config 4 head 17")


@pytest.mark.parametrize("hh", [0, 5, 11])
def test_config5_packed_forward_backward_bf16(hh):
    w = wl.make_workload(5)
    assert w.cu_seqlens == [0, 8190, 24570, 57330, 90090]
    gpu = pu.run_gpu(w.tensors, w.F, w.d_phi, w.eps, phi=w.phi, cu_seqlens=w.cu_seqlens)
    _check_heads(w, gpu, [hh], 2e-2, f"config 5 head {hh} (factorized oracle, all four sequences)")


def test_config5_packed_bruteforce_rows_and_no_leak():
    w = wl.make_workload(5)
    gpu = pu.run_gpu(w.tensors, w.F, w.d_phi, w.eps, phi=w.phi, cu_seqlens=w.cu_seqlens)
    _check_bruteforce_rows(w, gpu, [0, 11], 32, 2e-2, "config 5 heads 0,11")
    # state must not leak across sequences: perturbing sequence 0 leaves 1..3 bit-identical
    t2 = {k: v.clone() for k, v in w.tensors.items()}
    t2["K"][:, :, :8190] = (t2["K"][:, :, :8190].float() * 1.5).to(t2["K"].dtype)
    t2["V"][:, :, :8190] = (t2["V"][:, :, :8190].float() + 0.25).to(t2["V"].dtype)
    gpu2 = pu.run_gpu(t2, w.F, w.d_phi, w.eps, phi=w.phi, cu_seqlens=w.cu_seqlens)
    for k in ("O", "dQ", "dK", "dV"):
        assert torch.equal(gpu[k][:, :, 8190:], gpu2[k][:, :, 8190:]), k
    assert not torch.equal(gpu["O"][:, :, :8190], gpu2["O"][:, :, :8190])

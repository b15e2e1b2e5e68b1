"""GPU parity of the MFMA (bf16 matrix-core) path against the CPU oracle through the C ABI, on
inputs that span several tiles, chunks and ragged tails, plus packed sequences."""
import numpy as np
import pytest
import torch

import paper_2602_12128_amd as hla
from paper_2602_12128_amd import workloads as wl
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu

BWD = True


@pytest.mark.parametrize("d,N,kind", [
    (128, 64, "halfnormal"),
    (128, 1000, "lognormal"),
    (64, 777, "halfnormal"),
    (128, 2500, "sparse"),
    (64, 33, "lognormal"),
    (128, 1, "halfnormal"),
])
def test_feature_level_bf16(d, N, kind):
    t = wl.make_feature_inputs(300 + N, 2, 3, N, d, 3, 6, torch.bfloat16, kind=kind)
    bwd = BWD and N > 1
    gpu = pu.run_gpu(t, 3, 6, 1e-6, path=hla.HLA_PATH_MFMA, backward=bwd)
    assert gpu["_path"] == hla.HLA_PATH_MFMA
    ref = pu.run_oracle(t, 3, 6, 1e-6, backward=bwd)
    pu.assert_parity(gpu, ref, 2e-2, f"mfma features d={d} N={N} {kind}")


@pytest.mark.parametrize("d,N,b2", [(128, 700, 2.0), (64, 1300, 0.5), (128, 95, 1.0)])
def test_feature_maps_bf16(d, N, b2):
    t, phi = wl.make_raw_inputs(400 + N, 1, 2, N, d, 3, 6, torch.bfloat16, b2_mean=b2)
    gpu = pu.run_gpu(t, 3, 6, 1e-6, phi=phi, path=hla.HLA_PATH_MFMA, backward=BWD)
    ref = pu.run_oracle(t, 3, 6, 1e-6, phi=phi, backward=BWD)
    # bf16 hidden activations put about 2e-3 of noise on the pre-ReLU values: rows within 1e-2 of
    # the kink may legitimately take the other branch and are left out of the gradient comparison
    masks = pu.relu_kink_masks(t, phi, 3, 1e-2)
    if b2 < 1.0:
        # many queries have all features near zero here: their tiny denominators amplify the
        # feature maps' bf16 rounding in dQ (an input-conditioning effect, not a kernel one), so
        # dQ gets a wider bound in this stress case; the benchmark recipe (b2 = 2) does not.
        dq = {"dQ": gpu["dQ"]}
        pu.assert_parity(dq, {"dQ": ref.pop("dQ")}, 8e-2, f"mfma phi d={d} N={N} b2={b2} (dQ)", row_masks=masks)
    pu.assert_parity(gpu, ref, 2e-2, f"mfma phi d={d} N={N} b2={b2}", row_masks=masks)


def test_packed_sequences_no_leak_bf16():
    cu = [0, 100, 100, 1500, 1501, 2600]
    t = wl.make_feature_inputs(12, 1, 2, cu[-1], 128, 3, 6, torch.bfloat16)
    gpu = pu.run_gpu(t, 3, 6, 1e-6, cu_seqlens=cu, path=hla.HLA_PATH_MFMA, backward=BWD)
    ref = pu.run_oracle(t, 3, 6, 1e-6, cu_seqlens=cu, backward=BWD)
    # the single-token sequence [1500,1501) has O(eps) feature gradients: compare it apart
    keep = np.ones(cu[-1], bool)
    keep[1500] = False
    pu.assert_parity({k: v[:, :, keep] for k, v in gpu.items() if k != "_path"},
                     {k: v[:, :, keep] for k, v in ref.items()}, 2e-2, "mfma packed")
    np.testing.assert_allclose(pu.to_np(gpu["O"])[:, :, 1500], ref["O"][:, :, 1500], rtol=2e-2, atol=1e-3)
    t2 = {k: v.clone() for k, v in t.items()}
    t2["K"][:, :, :100] += 0.5
    t2["V"][:, :, :100] -= 1.0
    gpu2 = pu.run_gpu(t2, 3, 6, 1e-6, cu_seqlens=cu, path=hla.HLA_PATH_MFMA, backward=BWD)
    for k in gpu:
        if k != "_path":
            assert torch.equal(gpu[k][:, :, 100:], gpu2[k][:, :, 100:]), k
    assert not torch.equal(gpu["O"][:, :, :100], gpu2["O"][:, :, :100])


def test_mfma_matches_generic_path_and_is_repeatable():
    t = wl.make_feature_inputs(13, 2, 2, 900, 128, 3, 6, torch.bfloat16, kind="lognormal")
    a = pu.run_gpu(t, 3, 6, 1e-6, path=hla.HLA_PATH_MFMA, backward=BWD)
    b = pu.run_gpu(t, 3, 6, 1e-6, path=hla.HLA_PATH_MFMA, backward=BWD)
    c = pu.run_gpu(t, 3, 6, 1e-6, path=hla.HLA_PATH_GENERIC, backward=BWD)
    for k in a:
        if k == "_path":
            continue
        assert torch.equal(a[k], b[k]), f"{k} not bit-reproducible"
        assert pu.max_rel_err(pu.to_np(a[k]), pu.to_np(c[k])) < 2e-2, k


def test_unsupported_shapes_fall_back_or_report():
    # AUTO falls back to the generic kernels when the MFMA path has none; forcing MFMA reports it
    h = hla.HLA(head_dim=32, feature_dim=6, degree=3, io_dtype=hla.HLA_BF16,
                phi_mode=hla.HLA_PHI_NONE, max_heads=1, max_tokens=8, max_seqs=1)
    assert h.active_path == hla.HLA_PATH_GENERIC
    h.destroy()
    with pytest.raises(hla.HLAError) as e:
        hla.HLA(head_dim=128, feature_dim=8, degree=2, io_dtype=hla.HLA_BF16,
                phi_mode=hla.HLA_PHI_NONE, kernel_path=hla.HLA_PATH_MFMA, max_heads=1,
                max_tokens=8, max_seqs=1)
    assert e.value.code == 2


def test_forward_backward_can_be_captured_in_a_graph():
    # After a first eager step (tables uploaded, kernel attributes set) the two calls allocate
    # nothing, copy nothing and never synchronise, so a stream capture of them replays to the
    # eager result; replays are interleaved with eager steps and checked every time.
    dev = torch.device("cuda:0")
    t, phi = wl.make_raw_inputs(900, 1, 2, 777, 128, 3, 6, torch.bfloat16)
    td = {k: v.to(dev) for k, v in t.items()}
    h = pu.make_handle(t, 3, 6, 1e-6, phi, None, path=hla.HLA_PATH_MFMA)
    h.set_phi_weights([{k: v.to(dev) for k, v in m.items()} for m in phi])
    outs = [torch.empty_like(td[k]) for k in ("V", "Q", "K", "V")]

    def step():
        h.forward(td["Q"], td["K"], td["V"], outs[0])
        h.backward(td["Q"], td["K"], td["V"], outs[0], td["dO"], outs[1], outs[2], outs[3])

    step()
    torch.cuda.synchronize()
    ref = [x.clone() for x in outs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for x in outs:
            x.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(ref, outs):
            assert torch.equal(a, b), f"replay {rep}"
        step()  # eager work between the replays
        torch.cuda.synchronize()
        for a, b in zip(ref, outs):
            assert torch.equal(a, b), f"eager after replay {rep}"
    h.destroy()


@pytest.mark.parametrize("F,dphi", [(3, 6), (2, 12)])
def test_handle_reuse_sees_fresh_partial_states(F, dphi):
    # A handle keeps its workspace (chunk partials, reduced states, features) between calls; a call
    # must read only what it wrote itself, never what an earlier call left at the same addresses.
    # Two different inputs through one handle, several times over: every result must equal, bit
    # for bit, what a fresh handle computes for that input.
    B, H, N, d = 2, 6, 9000, 128   # 12 units of several chunks each, workgroups on every XCD
    ta = wl.make_feature_inputs(901, B, H, N, d, F, dphi, torch.bfloat16)
    tb = wl.make_feature_inputs(902, B, H, N, d, F, dphi, torch.bfloat16, kind="lognormal")
    fresh = {id(t): pu.run_gpu(t, F, dphi, 1e-6, path=hla.HLA_PATH_MFMA) for t in (ta, tb)}
    h = pu.make_handle(ta, F, dphi, 1e-6, None, None, hla.HLA_PATH_MFMA)
    for t in (ta, tb, tb, ta, tb, ta):
        got = pu.run_gpu(t, F, dphi, 1e-6, handle=h)
        for k in ("O", "dQ", "dK", "dV"):
            assert torch.equal(got[k], fresh[id(t)][k]), k
    h.destroy()
    ref = pu.run_oracle({k: v[:, :2] for k, v in tb.items()}, F, dphi, 1e-6)
    pu.assert_parity({k: fresh[id(tb)][k][:, :2] for k in ref}, ref, 2e-2, f"reuse F={F}")

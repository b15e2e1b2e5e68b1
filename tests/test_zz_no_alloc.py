"""hla_forward_static, the forward for callers that cannot allocate device memory: through the C
ABI, against hla_forward (same kernels: same bits) and against the oracle, on two calls in a row
(the second smaller, so it meets what the first left in the shared static workspace), then other
configurations through the same array, and the size and mode limits."""
import pytest
import torch

import paper_2602_12128_amd as hla
from paper_2602_12128_amd import workloads as wl
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu


def _static_forward(t, F, dphi, io_dtype=hla.HLA_BF16, path=hla.HLA_PATH_AUTO):
    dev = torch.device("cuda:0")
    td = {k: v.to(dev) for k, v in t.items()}
    O = torch.full_like(td["V"], float("nan"))
    hla.hla_forward_static(td["Q"], td["K"], td["V"], O, feature_dim=dphi, degree=F, eps=1e-6,
                           io_dtype=io_dtype, kernel_path=path)
    torch.cuda.synchronize()
    return O.cpu()


def test_static_forward_matches_handle_forward_and_oracle():
    cases = [
        (3, 6, 2, 3, 3000, 128, torch.bfloat16),   # first call
        (3, 6, 1, 2, 700, 128, torch.bfloat16),    # smaller, right after it
        (2, 12, 2, 2, 1500, 64, torch.bfloat16),   # another form and head dim: the array is re-laid out
        (3, 6, 1, 2, 700, 128, torch.bfloat16),    # and back
        (3, 5, 1, 2, 300, 32, torch.float32),      # fp32 kernels
    ]
    for i, (F, dphi, B, H, N, d, dtype) in enumerate(cases):
        t = wl.make_feature_inputs(950 + i, B, H, N, d, F, dphi, dtype, kind="lognormal" if i % 2 else "halfnormal")
        io = hla.HLA_F32 if dtype == torch.float32 else hla.HLA_BF16
        print(f"[static] case {i}: F={F} d_phi={dphi} B={B} H={H} N={N} d={d} {dtype}", flush=True)
        got = _static_forward(t, F, dphi, io_dtype=io)
        want = pu.run_gpu(t, F, dphi, 1e-6, backward=False)
        assert torch.equal(got, want["O"]), f"case {i}: differs from hla_forward"
        ref = pu.run_oracle(t, F, dphi, 1e-6, backward=False)
        pu.assert_parity({"O": got}, ref, pu.TOL[dtype], f"static forward case {i}")


def test_static_forward_limits():
    dev = torch.device("cuda:0")
    # a layout that does not fit the static array is refused and leaves the output alone
    B, H, N, d = 1, 8, 60000, 128
    Q = torch.zeros(B, H, N, 6, dtype=torch.bfloat16, device=dev)
    K = torch.zeros(B, H, N, 18, dtype=torch.bfloat16, device=dev)
    V = torch.zeros(B, H, N, d, dtype=torch.bfloat16, device=dev)
    O = torch.full_like(V, 3.0)
    with pytest.raises(hla.HLAError) as e:
        hla.hla_forward_static(Q, K, V, O)
    assert e.value.code == 6
    torch.cuda.synchronize()
    assert bool((O == 3.0).all())
    # feature maps need registered weights, i.e. a handle
    lib = hla.load_library()
    from paper_2602_12128_amd import binding as b
    import ctypes
    cfg = b.hla_config(128, 6, 3, 1e-6, b.HLA_BF16, b.HLA_PHI_MLP, 0, 1, 1, 1)
    v = b._view(V)
    assert lib.hla_forward_static(ctypes.byref(cfg), B, H, N, v, v, v, v, None) == 2
    assert lib.hla_forward_static(None, B, H, N, v, v, v, v, None) == 1
    # the array still serves a call that fits
    t = wl.make_feature_inputs(960, 1, 2, 500, 128, 3, 6, torch.bfloat16)
    got = _static_forward(t, 3, 6)
    want = pu.run_gpu(t, 3, 6, 1e-6, backward=False)
    assert torch.equal(got, want["O"])
    # empty input: nothing to do
    z = lambda w: torch.zeros(1, 2, 0, w, dtype=torch.bfloat16, device=dev)
    hla.hla_forward_static(z(6), z(18), z(128), z(128))

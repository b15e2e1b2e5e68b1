"""Seeded sweep over awkward shapes of the MFMA path (ragged tails, single tokens, many short
sequences, batch rows, sequence lengths around the tile / step / chunk sizes), forward and backward
with feature maps and weight gradients, against the CPU oracle."""
import numpy as np
import pytest
import torch

import paper_2602_12128_amd as hla
from paper_2602_12128_amd import workloads as wl
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu


def _cu(lens):
    cu = [0]
    for n in lens:
        cu.append(cu[-1] + n)
    return cu


CASES = [
    # d, B, H, N or packed lengths
    (128, 3, 1, 31, None),
    (128, 1, 5, 129, None),
    (64, 4, 2, 65, None),
    (64, 1, 1, 2049, None),
    (128, 1, 2, None, [1, 2, 33, 64, 127, 300]),
    (64, 1, 3, None, [5, 0, 0, 70, 1]),
    (128, 1, 1, None, [2000, 37]),
    (128, 2, 13, 257, None),
]


@pytest.mark.parametrize("F,dphi", [(3, 6), (2, 12)])
@pytest.mark.parametrize("d,B,H,N,lens", CASES)
def test_shape_sweep_bf16(d, B, H, N, lens, F, dphi):
    cu = None if lens is None else _cu(lens)
    n_tok = N if lens is None else cu[-1]
    seed = 1000 + 7 * d + 13 * B + 17 * H + n_tok + F
    t, phi = wl.make_raw_inputs(seed, B, H, n_tok, d, F, dphi, torch.bfloat16)
    gpu = pu.run_gpu(t, F, dphi, 1e-6, phi=phi, cu_seqlens=cu, path=hla.HLA_PATH_MFMA, weight_grads=True)
    assert gpu["_path"] == hla.HLA_PATH_MFMA
    ref = pu.run_oracle(t, F, dphi, 1e-6, phi=phi, cu_seqlens=cu, weight_grads=True)
    what = f"sweep F={F} d={d} B={B} H={H} " + (f"N={N}" if lens is None else f"lens={lens}")
    kinks = pu.oracle_kinks(t, phi, F, dphi, ref)
    # sequences of one or two tokens have outputs that barely depend on Q and K: their dQ, dK are
    # what two cancelling terms leave behind, and are measured on those terms' scale
    short = lens is not None and min(x for x in lens if x > 0) <= 2
    pu.assert_parity(gpu, ref, 2e-2, what, kinks=kinks,
                     row_scale=pu.short_sequence_rows(t, ref, cu) if short else None)
    br = pu.oracle_weight_grad_branches(t, phi, F, dphi, ref, cu_seqlens=cu)
    pu.assert_weight_grad_parity(gpu["wg"], ref["wg"], 2e-2, what, branches=br)

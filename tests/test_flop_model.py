"""The FLOP model used by the bench reproduces the per-layer numbers the paper prints."""
import os

from paper_2602_12128_amd import flops

GOLD = os.path.join(os.path.dirname(__file__), "golden", "table3_attention_layer_tflops.txt")


def test_reproduces_paper_complexity_table():
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for kind, tokens, printed in rows:
        got = flops.attention_layer_tflops(int(tokens), "quadratic" if kind == "quadratic" else "hla")
        assert abs(got - float(printed)) <= 0.005 + 1e-9, (kind, tokens, got, printed)


def test_core_share_and_path_totals():
    # the operator core is 4 D d per token-head: 0.0435 TFLOP of the 0.77 TFLOP layer at 32760 tokens
    core = 4 * 216 * 128 * 32760 * 12 / 1e12
    assert abs(core - 0.0435) < 1e-4
    assert flops.core_forward_flops(128, 6, 3) == 4 * 216 * 128 + 3 * 216 + 2 * (36 + 216)
    assert flops.path_bytes(128, 6, 3, True, True) == 12 * 128 * 2
    assert flops.path_bytes(128, 6, 3, False, False) == (6 + 18 + 256) * 2

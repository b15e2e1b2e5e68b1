"""Nominal FLOP and algorithmic-byte model of the HLA hot path (2 flops per multiply-add, the
paper's counting), per token-head, plus the per-layer totals that reproduce the paper's
complexity table.  Host-side bookkeeping for the bench; no arithmetic of the method."""
from __future__ import annotations


def core_forward_flops(d: int, d_phi: int, F: int) -> int:
    """Outer products, state (context + normaliser) and query contraction (Theorem 4.2)."""
    D = d_phi ** F
    outer = 2 * sum(d_phi ** f for f in range(2, F + 1))      # T_k and T_q built slot by slot
    return 4 * D * d + 3 * D + outer


def core_backward_flops(d: int, d_phi: int, F: int) -> int:
    """dT_q = C g, dC = T_q (x) g, dT_k = dC v, dv = dC^T T_k: four contractions of size D x d."""
    return 8 * d_phi ** F * d


def phi_forward_flops(d: int, d_phi: int, F: int) -> int:
    """1+F feature maps (App. A.1): Linear d->d, Linear d->d_phi."""
    return (1 + F) * (2 * d * d + 2 * d * d_phi)


def phi_backward_flops(d: int, d_phi: int, F: int) -> int:
    """Input gradients only: recompute the first layer, back through both layers."""
    return (1 + F) * (2 * d * d + 2 * d * d_phi + 2 * d * d)


def path_flops(d: int, d_phi: int, F: int, backward: bool, phi: bool) -> int:
    f = core_forward_flops(d, d_phi, F)
    if phi:
        f += phi_forward_flops(d, d_phi, F)
    if backward:
        f += core_backward_flops(d, d_phi, F)
        if phi:
            f += phi_backward_flops(d, d_phi, F)
    return f


def path_bytes(d: int, d_phi: int, F: int, backward: bool, phi: bool, elem: int = 2) -> int:
    """Bytes that must cross HBM per token-head if nothing but the operator's own inputs and
    outputs moved (features never stored): forward reads Q,K,V and writes O; backward reads
    Q,K,V,O,dO and writes dQ,dK,dV."""
    qk = 2 * d if phi else (1 + F) * d_phi
    fwd = (qk + 2 * d) * elem
    bwd = (qk + 3 * d + qk + d) * elem
    return fwd + (bwd if backward else 0)


def symmetric_rows(d_phi: int, F: int) -> int:
    """Rows of the padded symmetric state the matrix-core kernels contract over: 64 for three
    factors of six features (56 monomials), 96 for two factors of twelve (78 monomials)."""
    return {(3, 6): 64, (2, 12): 96}[(F, d_phi)]


def executed_kernel_flops(name: str, d: int, d_phi: int, F: int) -> int:
    """Matrix-core flops the MFMA path ISSUES per token-head in one launch of `name` (every
    v_mfma_f32_32x32x16 counts its full 32*32*16*2 flops: padded rows of the symmetric state and the
    26 unused output rows of the second feature-map layer included), against the nominal model's
    literal d_phi^F contraction.  0 for kernels without matrix work."""
    MP = symmetric_rows(d_phi, F)
    maps = 1 + F
    return {
        "mfma_phi_forward": maps * (2 * d * d + 64 * d),             # first layer; second layer in 32 output rows
        "mfma_state": 2048 * (MP // 32) * (d // 32 + 1),            # S^T [V | 1] per 64-token step
        "mfma_query": 2 * d * MP,
        "mfma_bwd_query": 4 * d * MP,                               # X = Csym dO^T and dCsym += Qm^T dO
        "mfma_bwd_key": 4 * d * MP,                                 # dS = dCsym V^T and dV = dCsym^T S^T
        "mfma_phi_backward": maps * (2 * d * d + 32 * d + 2 * d * d),  # recompute, dg (one k-step), dx
    }.get(name, 0)


def executed_path_flops(d: int, d_phi: int, F: int, backward: bool, phi: bool) -> int:
    names = ["mfma_state", "mfma_query"] + (["mfma_phi_forward"] if phi else [])
    if backward:
        names += ["mfma_bwd_query", "mfma_bwd_key"] + (["mfma_phi_backward"] if phi else [])
    return sum(executed_kernel_flops(n, d, d_phi, F) for n in names)


def attention_layer_tflops(tokens: int, kind: str, width: int = 1536, heads: int = 12,
                           d_phi: int = 6, F: int = 3) -> float:
    """FLOPs of one attention layer as the paper's complexity table counts them: q/k/v/o
    projections (8 N W^2) plus either the quadratic scores and values (4 N^2 W) or, for HLA,
    the feature maps of q and k, the two value-modulation maps (two d->d layers each) and the
    HLA core (4 D d per token-head)."""
    d = width // heads
    proj = 8 * tokens * width * width
    if kind == "quadratic":
        return (proj + 4 * tokens * tokens * width) / 1e12
    th = tokens * heads
    phi_qk = phi_forward_flops(d, d_phi, F)
    phi_v = 2 * (2 * d * d + 2 * d * d)
    core = 4 * d_phi ** F * d
    return (proj + th * (phi_qk + phi_v + core)) / 1e12


# Per-kernel model for the roofline line of the bench: algorithmic HBM bytes and nominal flops
# per token-head handled by one launch (d = head dim, nf = (1+F)*d_phi fp32 feature row, e = I/O
# element size).  Bound: what limits the kernel on MI355X by this model.
def kernel_model(name: str, d: int, d_phi: int, F: int, e: int = 2):
    D = d_phi ** F
    qf, kf = 4 * d_phi, 4 * F * d_phi
    lin = 2 * d * d + 2 * d * d_phi            # one feature map forward
    lin_b = 4 * d * d + 2 * d * d_phi          # one feature map backward (recompute + input grad)
    m = {
        "mfma_phi_forward": (2 * d * e + qf + kf, (1 + F) * lin, "mfma"),     # query map and key maps, one launch
        "mfma_state": (d * e + kf, 2 * D * d + D, "hbm"),
        "mfma_query": (qf + d * e + 4, 2 * D * d + 2 * D, "hbm"),
        "mfma_bwd_query": (d * e + qf + 4 + qf, 4 * D * d, "hbm"),   # dO, features, den in; feature grads out
        "mfma_bwd_key": (d * e + kf + d * e + kf, 4 * D * d, "hbm"),
        "mfma_phi_backward": (4 * d * e + 2 * (qf + kf), (1 + F) * lin_b, "mfma"),
        # value modulation (Sec. 4.5): two maps of two d x d layers; the backward recomputes them
        # and goes back through both (on the matrix cores for bf16 I/O, else fp32 vector ALU)
        "vmod_forward": (3 * d * e, 8 * d * d, "mfma" if e == 2 else "alu"),
        "vmod_backward": (5 * d * e, 16 * d * d, "mfma" if e == 2 else "alu"),
        "generic_phi_forward": (2 * d * e + qf + kf, phi_forward_flops(d, d_phi, F), "alu"),
        "generic_phi_backward": (2 * d * e + 2 * (qf + kf) + 2 * d * e, phi_backward_flops(d, d_phi, F), "alu"),
    }
    return m.get(name)


PEAKS = {"hbm": (8000.0, "GB/s"), "mfma": (2500.0, "TFLOP/s"), "alu": (157.3, "TFLOP/s")}  # alu: fp32 vector

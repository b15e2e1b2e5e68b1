"""Seeded synthetic inputs for the HLA operator: the five benchmark configurations and a few
generic generators for tests.

This module holds NO arithmetic of the method (no feature maps, no attention): it only draws
random tensors with the shapes and value distributions of the paper's video-DiT workloads
(Sec. 5.1: Wan2.1-1.3B, width 1536 = 12 heads x 128; 32760 tokens for 81x480x832 video), so the
CPU oracle and the GPU library can be fed exactly the same numbers.  The paper's real inputs
(video latents, trained feature-map weights) are not available; these stand in for them.

All draws come from one `torch.Generator('cpu')` per configuration, in the fixed order
Q, K, V, dO, then the feature-map weights map by map (W1, b1, W2, b2).  Tensors are drawn in
fp32 and rounded once to the I/O dtype; both sides read the rounded values.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import torch


@dataclass
class Workload:
    name: str
    B: int
    H: int
    N: int                      # tokens per batch row (sum of sequence lengths when packed)
    d: int
    F: int = 3                  # Hadamard degree (paper's main variant: 3 factors)
    d_phi: int = 6              # feature dim (App. A.1: 6 for 3 factors, 12 for 2 factors)
    eps: float = 1e-6
    dtype: torch.dtype = torch.bfloat16
    backward: bool = True
    cu_seqlens: Optional[List[int]] = None
    seed: int = 0
    value_recipe: str = "gauss"  # "gauss" | "unit_norm" | "unit_norm_lowrank"
    grid: Optional[tuple] = None  # latent grid (t, h, w) the token count comes from
    tensors: Dict[str, torch.Tensor] = field(default_factory=dict)
    phi: List[Dict[str, torch.Tensor]] = field(default_factory=list)

    @property
    def token_heads(self) -> int:
        return self.B * self.H * self.N


def _spec(idx: int) -> Workload:
    if idx == 1:
        return Workload("c1_tiny_fwd_fp32", 1, 2, 256, 32, dtype=torch.float32, backward=False,
                        seed=0)
    if idx == 2:
        return Workload("c2_mid_fwdbwd_bf16", 2, 12, 4096, 64, seed=1)
    if idx == 3:
        return Workload("c3_dit480p_fwdbwd_bf16", 1, 12, 32760, 128, seed=2,
                        value_recipe="unit_norm", grid=(21, 30, 52))
    if idx == 4:
        return Workload("c4_dit720p_fwd_bf16", 1, 40, 75600, 128, backward=False, seed=3,
                        value_recipe="unit_norm_lowrank", grid=(21, 45, 80))
    if idx == 5:
        lens = [8190, 16380, 32760, 32760]
        cu = [0]
        for n in lens:
            cu.append(cu[-1] + n)
        return Workload("c5_packed_fwdbwd_bf16", 1, 12, cu[-1], 128, seed=4, cu_seqlens=cu)
    # variants of configuration 3 that the paper also evaluates (not headline configurations)
    if idx == 6:  # the lower resolution of Sec. 5.1: 81x320x480 video -> 12600 tokens
        return Workload("r2_dit320p_fwdbwd_bf16", 1, 12, 12600, 128, seed=5,
                        value_recipe="unit_norm", grid=(21, 20, 30))
    if idx == 7:  # two Hadamard factors with 12 features (App. A.1)
        return Workload("c3_dit480p_2factor_fwdbwd_bf16", 1, 12, 32760, 128, F=2, d_phi=12, seed=6,
                        value_recipe="unit_norm", grid=(21, 30, 52))
    raise ValueError(f"no such configuration: {idx}")


def _draw(gen, shape):
    return torch.randn(shape, generator=gen, dtype=torch.float32)


def _unit_norm(x: torch.Tensor) -> torch.Tensor:
    """Divide each d-vector by its RMS, then by sqrt(d): unit L2 norm per token-head."""
    d = x.shape[-1]
    rms = x.pow(2).mean(dim=-1, keepdim=True).sqrt()
    return x / rms / math.sqrt(d)


def draw_phi_weights(gen, d: int, d_phi: int, n_maps: int, dtype,
                     b2_mean: float = 2.0) -> List[Dict[str, torch.Tensor]]:
    """Stand-ins for trained feature-map weights.  W1 ~ N(0,1) keeps pre-activations O(1) for
    unit-norm inputs; W2 ~ N(0, 1/(0.425 d)) gives the second layer unit output variance
    (0.425 ~ E[GELU(h)^2] for h ~ N(0,1)); the second bias is centred at `b2_mean` so that with
    the default +2 practically no token has all features clipped by the ReLU."""
    maps = []
    for _ in range(n_maps):
        W1 = _draw(gen, (d, d))
        b1 = 0.25 * _draw(gen, (d,))
        W2 = _draw(gen, (d, d_phi)) / math.sqrt(0.425 * d)
        b2 = b2_mean + 0.25 * _draw(gen, (d_phi,))
        maps.append({k: t.to(dtype).contiguous()
                     for k, t in (("W1", W1), ("b1", b1), ("W2", W2), ("b2", b2))})
    return maps


def draw_vmod_weights(gen, d: int, dtype, in_scale=(32.0, 1.0), out_scale: float = 0.05):
    """Stand-ins for the trained value-modulation maps phi_v1, phi_v2 (Sec. 4.5; App. A.1: two
    d x d layers and a LayerNorm each).  phi_v1 reads the attention output, which for synthetic
    inputs is an average of many nearly independent value vectors and therefore tiny: its first
    layer is scaled up (in_scale[0]) so that its pre-activations are O(1) like phi_v2's.  gamma
    and beta are scaled by out_scale so that the product of the two maps is comparable to the
    attention output it is added to (otherwise the sum would hide that output below the bf16
    resolution of the result)."""
    maps = []
    for k in range(2):
        W1 = in_scale[k] * _draw(gen, (d, d))
        b1 = 0.25 * _draw(gen, (d,))
        W2 = _draw(gen, (d, d)) / math.sqrt(0.425 * d)
        b2 = 0.25 * _draw(gen, (d,))
        gamma = math.sqrt(out_scale) * (1.0 + 0.1 * _draw(gen, (d,)))
        beta = math.sqrt(out_scale) * 0.1 * _draw(gen, (d,))
        maps.append({n: t.to(dtype).contiguous() for n, t in
                     (("W1", W1), ("b1", b1), ("W2", W2), ("b2", b2), ("gamma", gamma), ("beta", beta))})
    return maps


def make_workload(idx: int, *, need_backward: Optional[bool] = None) -> Workload:
    """Build configuration `idx` (1..5, or a variant 6..7) with all tensors on the CPU in the I/O dtype."""
    w = _spec(idx)
    if need_backward is not None:
        w.backward = w.backward and need_backward
    gen = torch.Generator("cpu").manual_seed(w.seed)
    shape = (w.B, w.H, w.N, w.d)
    raw = {}
    for name in ("Q", "K", "V"):
        x = _draw(gen, shape)
        if w.value_recipe == "gauss":
            x = x / math.sqrt(w.d)
        elif w.value_recipe == "unit_norm":
            x = _unit_norm(x)
        elif w.value_recipe == "unit_norm_lowrank":
            rank = 16
            basis = _draw(gen, (w.B, w.H, rank, w.d))
            coef = _draw(gen, (w.B, w.H, w.N, rank)) / math.sqrt(rank)
            x = _unit_norm(x + 0.5 * torch.matmul(coef, basis))
        raw[name] = x
    dO = _draw(gen, shape) if _spec(idx).backward else None
    w.tensors = {k: v.to(w.dtype).contiguous() for k, v in raw.items()}
    if dO is not None and w.backward:
        w.tensors["dO"] = dO.to(w.dtype).contiguous()
    w.phi = draw_phi_weights(gen, w.d, w.d_phi, 1 + w.F, w.dtype)
    return w


def make_feature_inputs(seed: int, B: int, H: int, N: int, d: int, F: int, d_phi: int, dtype,
                        kind: str = "halfnormal"):
    """Inputs for the feature-level interface (Q [..,d_phi], K [..,F*d_phi] already >= 0).
    kind: 'halfnormal' = |N(0,1)|; 'lognormal' = exp(N(0,1)) (peaky attention rows);
    'sparse' = |N(0,1)| with about half the entries set to zero."""
    gen = torch.Generator("cpu").manual_seed(seed)
    q = _draw(gen, (B, H, N, d_phi))
    k = _draw(gen, (B, H, N, F * d_phi))
    if kind == "halfnormal":
        q, k = q.abs(), k.abs()
    elif kind == "lognormal":
        q, k = q.exp(), k.exp()
    elif kind == "sparse":
        mq = _draw(gen, q.shape) > 0
        mk = _draw(gen, k.shape) > 0
        q, k = q.abs() * mq, k.abs() * mk
    else:
        raise ValueError(kind)
    v = _draw(gen, (B, H, N, d))
    do = _draw(gen, (B, H, N, d))
    return {n: t.to(dtype).contiguous() for n, t in (("Q", q), ("K", k), ("V", v), ("dO", do))}


def make_raw_inputs(seed: int, B: int, H: int, N: int, d: int, F: int, d_phi: int, dtype,
                    b2_mean: float = 2.0):
    """Raw Q,K,V ~ N(0,1)/sqrt(d), dO ~ N(0,1), plus feature-map weights, for any shape."""
    gen = torch.Generator("cpu").manual_seed(seed)
    t = {n: (_draw(gen, (B, H, N, d)) / math.sqrt(d)) for n in ("Q", "K", "V")}
    t["dO"] = _draw(gen, (B, H, N, d))
    t = {n: x.to(dtype).contiguous() for n, x in t.items()}
    phi = draw_phi_weights(gen, d, d_phi, 1 + F, dtype, b2_mean=b2_mean)
    return t, phi

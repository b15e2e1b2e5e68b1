"""CPU oracle for non-causal Hadamard Linear Attention (HLA), fp64, numpy.

TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must compute; it is
deliberately plain and slow.  It shares no code with the HIP path and must never be imported by
the product package: only tests, the smoke check and the bench's cpu_baseline leg call it.

Every function works on ONE attention unit (one sequence of one head) with 2-D float64 arrays;
`hla_operator_forward/backward` loop such units over batch, heads and packed sequences.

Notation follows the paper: N tokens, head dim d, feature dim d_phi, Hadamard degree F,
D = d_phi**F.  qf = phi_q(Q) is [N, d_phi]; kfs = [phi_k1(K), ..., phi_kF(K)], each [N, d_phi];
v is [N, d].

Pins (tests/test_oracle_*.py): brute force == factorized; F=1 == textbook linear attention;
d_phi=1, identical-key, one-hot and N=1 closed forms; row normalisation; convexity; permutation
invariance; homogeneity (rational-function form); the sequential state update; Lemma 4.1; GELU
against tabulated normal-CDF values; both backward routes, and the feature-map weight gradients,
against central finite differences; the enumeration of ReLU branch choices against the masked
(smooth) map; the value modulation of Sec. 4.5 against scalar loops (LayerNorm, the map), the
identity special case and finite differences (tests/test_oracle_value_modulation.py); the
causal variant of Sec. 4.4 through its two routes, its first and last rows and causality itself
(tests/test_oracle_causal.py).  No function here is "parity unpinned".
"""
from __future__ import annotations

import math
import string
from typing import List, Optional, Sequence, Tuple

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


# --------------------------------------------------------------------------------------------
# Feature maps phi (App. A.1; Alg. 1 Step 4): Linear(d->d) -> GELU -> Linear(d->d_phi) -> ReLU
# --------------------------------------------------------------------------------------------
def gelu_erf(h: np.ndarray) -> np.ndarray:
    """Exact GELU: h * Phi(h), Phi the standard normal CDF = (1 + erf(h/sqrt 2)) / 2."""
    h = np.asarray(h, dtype=F64)
    return h * 0.5 * (1.0 + _erf(h / math.sqrt(2.0)))


def gelu_erf_grad(h: np.ndarray) -> np.ndarray:
    """d/dh [h Phi(h)] = Phi(h) + h * pdf(h), pdf the standard normal density."""
    h = np.asarray(h, dtype=F64)
    cdf = 0.5 * (1.0 + _erf(h / math.sqrt(2.0)))
    pdf = np.exp(-0.5 * h * h) / math.sqrt(2.0 * math.pi)
    return cdf + h * pdf


def phi_forward(x, W1, b1, W2, b2):
    """phi(x) = max(GELU(x W1 + b1) W2 + b2, 0)  (App. A.1: two linear layers, GELU between,
    ReLU after; weights act from the right, W1 is [d, d], W2 is [d, d_phi]).

    Returns (features [N, d_phi], pre-activation h [N, d], pre-ReLU u [N, d_phi])."""
    x = np.asarray(x, dtype=F64)
    h = x @ np.asarray(W1, F64) + np.asarray(b1, F64)
    g = gelu_erf(h)
    u = g @ np.asarray(W2, F64) + np.asarray(b2, F64)
    return np.maximum(u, 0.0), h, u


def phi_backward(dfeat, x, W1, b1, W2, b2, relu_open=None):
    """Gradient of a scalar loss w.r.t. x given its gradient w.r.t. phi(x) (chain rule through
    ReLU, the second linear layer, GELU and the first linear layer of App. A.1).

    The ReLU makes this gradient discontinuous where a pre-activation u crosses zero.  relu_open
    (bool [N, d_phi]) replaces the decision u > 0 by a given branch choice: the map is then
    differentiated as relu_open * u(x).  It exists for phi_backward_branches below, which
    enumerates the choices an implementation in lower precision may legitimately take for
    pre-activations that are zero to within its rounding error; the choices always come from this
    oracle's own pre-activations, never from an implementation under test."""
    _, h, u = phi_forward(x, W1, b1, W2, b2)
    du = np.asarray(dfeat, F64) * ((u > 0.0) if relu_open is None else np.asarray(relu_open, bool))
    dg = du @ np.asarray(W2, F64).T
    dh = dg * gelu_erf_grad(h)
    return dh @ np.asarray(W1, F64).T


def phi_weight_grads(dfeat, x, W1, b1, W2, b2, relu_open=None):
    """Gradient of a scalar loss w.r.t. the weights of one feature map given its gradient w.r.t.
    phi(x) for the N rows of x (same chain rule as phi_backward, App. A.1 layers; the paper trains
    these layers, Sec. 5 stage 1, and leaves the formulas to autograd):
      du = dfeat * [u > 0];  dW2 = g^T du;  db2 = sum_n du;  dg = du W2^T;
      dh = dg * GELU'(h);    dW1 = x^T dh;  db1 = sum_n dh.
    relu_open: as in phi_backward.  Returns (dW1 [d,d], db1 [d], dW2 [d,d_phi], db2 [d_phi])."""
    x = np.asarray(x, F64)
    _, h, u = phi_forward(x, W1, b1, W2, b2)
    g = gelu_erf(h)
    du = np.asarray(dfeat, F64) * ((u > 0.0) if relu_open is None else np.asarray(relu_open, bool))
    dg = du @ np.asarray(W2, F64).T
    dh = dg * gelu_erf_grad(h)
    return x.T @ dh, dh.sum(axis=0), g.T @ du, du.sum(axis=0)


def phi_backward_branches(dfeats, x, maps, band: float, max_inband: int = 12):
    """Every input-gradient row a correct implementation may produce for the rows of x whose ReLU
    decisions are not settled at resolution `band` (App. A.1: the ReLU ends each map).

    x [N, d] feeds len(maps) feature maps (maps[m] = (W1, b1, W2, b2)); dfeats[m] [N, d_phi] is
    the loss gradient w.r.t. map m's features; the gradient w.r.t. x sums the maps (as dK sums
    the key maps).  A feature (m, a) of row n is "in band" when |u_m[n, a]| < band.  For every
    row with k >= 1 in-band features the result holds the 2^k gradient rows obtained by opening
    or closing each of them, all other features following u > 0.  Candidate 0 closes all of them.
    Returns {row: array [2^k, d]}.  More than max_inband in-band features in one row raise."""
    x = np.asarray(x, F64)
    us = [phi_forward(x, *m)[2] for m in maps]
    inband = [np.abs(u) < band for u in us]
    rows = np.nonzero(np.any(np.concatenate(inband, axis=1), axis=1))[0]
    out = {}
    for n in rows:
        slots = [(m, a) for m in range(len(maps)) for a in np.nonzero(inband[m][n])[0]]
        if len(slots) > max_inband:
            raise ValueError(f"row {n}: {len(slots)} pre-activations within {band} of zero")
        cands = np.zeros((1 << len(slots), x.shape[1]), F64)
        for bits in range(1 << len(slots)):
            opens = [(u[n] > 0.0) & ~ib[n] for u, ib in zip(us, inband)]
            for i, (m, a) in enumerate(slots):
                opens[m][a] = bool((bits >> i) & 1)
            for m in range(len(maps)):
                cands[bits] += phi_backward(np.asarray(dfeats[m], F64)[n:n + 1], x[n:n + 1], *maps[m],
                                            relu_open=opens[m][None, :])[0]
        out[int(n)] = cands
    return out


def phi_weight_grad_branches(dfeat, x, W1, b1, W2, b2, band: float):
    """The weight gradients of one feature map as a function of the ReLU branch choices that are
    not settled at resolution `band` (companion of phi_backward_branches; the gradients are sums
    over all rows, so the choices of all rows enter every entry, linearly):
        grads(choice) = base + sum over in-band pairs p of choice[p] * contrib[p],   choice[p] in {0, 1}
    with base = phi_weight_grads taking every in-band feature as closed and the others by u > 0, and
    contrib[p] = phi_weight_grads of the single pair p = (row n, feature a) taken as open.
    Returns (base, pairs, contribs, own): base and each contribs[i] are (dW1, db1, dW2, db2);
    pairs[i] = (n, a); own[i] = the oracle's own decision u[n, a] > 0."""
    x = np.asarray(x, F64)
    dfeat = np.asarray(dfeat, F64)
    u = phi_forward(x, W1, b1, W2, b2)[2]
    inband = np.abs(u) < band
    base = phi_weight_grads(dfeat, x, W1, b1, W2, b2, relu_open=(u > 0.0) & ~inband)
    pairs = [(int(n), int(a)) for n, a in zip(*np.nonzero(inband))]
    contribs = []
    for n, a in pairs:
        one = np.zeros((1, u.shape[1]), bool)
        one[0, a] = True
        contribs.append(phi_weight_grads(dfeat[n:n + 1], x[n:n + 1], W1, b1, W2, b2, relu_open=one))
    own = [bool(u[n, a] > 0.0) for n, a in pairs]
    return base, pairs, contribs, own


# --------------------------------------------------------------------------------------------
# Outer-product feature tensors (Sec. 4.2, definition of T_q and T_k before Theorem 4.2)
# --------------------------------------------------------------------------------------------
def outer_features(feats: Sequence[np.ndarray]) -> np.ndarray:
    """Per token n: feats[0][n] (x) feats[1][n] (x) ... flattened to length d_phi**F, slot f of
    the outer product belonging to feats[f] (first slot slowest, as the listings' einsum
    'bhsd,bhse,bhsf->bhsdef' followed by a flatten)."""
    n = feats[0].shape[0]
    t = np.asarray(feats[0], F64)
    for f in feats[1:]:
        t = (t[:, :, None] * np.asarray(f, F64)[:, None, :]).reshape(n, -1)
    return t


# --------------------------------------------------------------------------------------------
# Forward
# --------------------------------------------------------------------------------------------
def hla_bruteforce(qf, kfs, v, eps: float):
    """The plain definition (Eq. 'hla' + row normalisation of Sec. 4.2), O(N^2):
    A_ij = prod_f <qf_i, kf_f,j>,  eta_i = sum_j A_ij,  o_i = sum_j A_ij v_j / (eta_i + eps)."""
    qf = np.asarray(qf, F64)
    v = np.asarray(v, F64)
    A = np.ones((qf.shape[0], v.shape[0]), dtype=F64)
    for kf in kfs:
        A = A * (qf @ np.asarray(kf, F64).T)
    eta = A.sum(axis=1)
    o = (A @ v) / (eta + eps)[:, None]
    return o, A, eta


def hla_state(kfs, v):
    """Key-side state of Theorem 4.2: context C = T_k (x)_1 V  [D, d] and the key-feature sum
    z = sum_j T_k,j  [D] that the normaliser eta contracts against."""
    Tk = outer_features(kfs)
    v = np.asarray(v, F64)
    return Tk.T @ v, Tk.sum(axis=0)


def hla_factorized(qf, kfs, v, eps: float):
    """The paper's linear-time scheme (Theorem 4.2, normaliser eta of Sec. 4.2; same steps as
    the listings for 2 and 3 factors, any F): C, z from the keys; T_q from the queries;
    num_i = T_q,i . C, eta_i = T_q,i . z, o_i = num_i / (eta_i + eps)."""
    C, z = hla_state(kfs, v)
    Tq = outer_features([qf] * len(kfs))
    eta = Tq @ z
    o = (Tq @ C) / (eta + eps)[:, None]
    return o, C, z, eta


def hla_sequential_state(kfs, v):
    """Token-by-token update C^i = C^{i-1} + T_k,i (Kronecker) v_i (Sec. 4.4, sequential
    updates); returns the final (C^N, z^N).  Python loop: small inputs only."""
    kfs = [np.asarray(k, F64) for k in kfs]
    v = np.asarray(v, F64)
    D = kfs[0].shape[1] ** len(kfs)
    C = np.zeros((D, v.shape[1]), F64)
    z = np.zeros(D, F64)
    for i in range(v.shape[0]):
        t = outer_features([k[i:i + 1] for k in kfs])[0]
        C += np.outer(t, v[i])
        z += t
    return C, z


# --------------------------------------------------------------------------------------------
# Causal variant (Sec. 4.4): token i attends to tokens j <= i only
# --------------------------------------------------------------------------------------------
def hla_causal_bruteforce(qf, kfs, v, eps: float, rows=None, decay: float = 1.0):
    """Eq. 'hla' with the {0,1} causal mask of Sec. 4.4 on the N x N matrix: A_ij as before for
    j <= i, zero for j > i; eta_i = sum_{j<=i} A_ij; o_i = sum_{j<=i} A_ij v_j / (eta_i + eps).
    rows: optional indices of the query rows to evaluate (against all their keys).
    decay: Sec. 4.4 lets the mask carry decay factors but gives no formula; the reading taken is
    one scalar lambda in (0, 1] and mask entries lambda^(i - j) for j <= i (a token's
    contribution fades geometrically with its distance), 1 = the plain {0,1} mask."""
    qf = np.asarray(qf, F64)
    v = np.asarray(v, F64)
    idx = np.arange(qf.shape[0]) if rows is None else np.asarray(rows)
    A = np.ones((len(idx), v.shape[0]), dtype=F64)
    for kf in kfs:
        A = A * (qf[idx] @ np.asarray(kf, F64).T)
    dist = idx[:, None] - np.arange(v.shape[0])[None, :]
    A = A * np.where(dist >= 0, float(decay) ** np.maximum(dist, 0), 0.0)
    eta = A.sum(axis=1)
    return (A @ v) / (eta + eps)[:, None]


def hla_causal_sequential(qf, kfs, v, eps: float, decay: float = 1.0):
    """The sequential updates of Sec. 4.4: the context tensor is the state, C^i = C^{i-1} +
    T_k,i (Kronecker) v_i (and z^i = z^{i-1} + T_k,i for the normaliser), and token i's output is
    the contraction of T_q,i with C^i, divided by T_q,i . z^i + eps.  With a decay factor the old
    state is multiplied by it before the new token is added: C^i = decay C^{i-1} + T_k,i (x) v_i.
    Python loop: small inputs."""
    qf = np.asarray(qf, F64)
    kfs = [np.asarray(k, F64) for k in kfs]
    v = np.asarray(v, F64)
    F = len(kfs)
    D = kfs[0].shape[1] ** F
    C = np.zeros((D, v.shape[1]), F64)
    z = np.zeros(D, F64)
    out = np.zeros_like(v)
    for i in range(v.shape[0]):
        tk = outer_features([k[i:i + 1] for k in kfs])[0]
        C = decay * C + np.outer(tk, v[i])
        z = decay * z + tk
        tq = outer_features([qf[i:i + 1]] * F)[0]
        out[i] = (tq @ C) / (tq @ z + eps)
    return out


# --------------------------------------------------------------------------------------------
# Backward (the paper leaves this to autograd; derived from the factorized form)
# --------------------------------------------------------------------------------------------
def _slot_gradient(dT: np.ndarray, feats: Sequence[np.ndarray], slot: int) -> np.ndarray:
    """Given dT [N, d_phi, ..., d_phi] (gradient w.r.t. the outer product of `feats`), return
    the gradient w.r.t. feats[slot] holding the other factors fixed:
    out[n, a] = sum over the other indices of dT[n, .., a at `slot`, ..] * prod_{f != slot} feats[f][n, .]"""
    F = len(feats)
    letters = string.ascii_lowercase[:F]
    operands = [dT]
    spec = ["n" + letters]
    for f in range(F):
        if f != slot:
            operands.append(np.asarray(feats[f], F64))
            spec.append("n" + letters[f])
    return np.einsum(",".join(spec) + "->n" + letters[slot], *operands)


def hla_backward_factorized(qf, kfs, v, do, eps: float):
    """Gradients of L = sum(O * dO) through the factorized form.  With den_i = eta_i + eps,
    g_i = dO_i / den_i, s_i = -<dO_i, o_i> / den_i:
      dT_q,i = C g_i + s_i z;   dC = sum_i T_q,i (x) g_i;   dz = sum_i s_i T_q,i;
      dT_k,j = dC v_j + dz;     dv_j = dC^T T_k,j;
    and every feature vector collects the gradient of each outer-product slot it fills.
    Returns (dqf [N,d_phi], [dkf_1..dkf_F], dv [N,d])."""
    qf = np.asarray(qf, F64)
    kfs = [np.asarray(k, F64) for k in kfs]
    v = np.asarray(v, F64)
    do = np.asarray(do, F64)
    F = len(kfs)
    n, dp = qf.shape
    o, C, z, eta = hla_factorized(qf, kfs, v, eps)
    den = eta + eps
    g = do / den[:, None]
    s = -(do * o).sum(axis=1) / den
    Tq = outer_features([qf] * F)
    Tk = outer_features(kfs)
    dTq = g @ C.T + s[:, None] * z[None, :]
    dC = Tq.T @ g
    dz = Tq.T @ s
    dTk = v @ dC.T + dz[None, :]
    dv = Tk @ dC
    shape = (n,) + (dp,) * F
    dTq = dTq.reshape(shape)
    dTk = dTk.reshape((v.shape[0],) + (dp,) * F)
    dqf = np.zeros_like(qf)
    for slot in range(F):
        dqf += _slot_gradient(dTq, [qf] * F, slot)
    dkfs = [_slot_gradient(dTk, kfs, slot) for slot in range(F)]
    return dqf, dkfs, dv


def hla_backward_bruteforce(qf, kfs, v, do, eps: float):
    """Same gradients through the explicit N x N matrix (independent route):
    dA_ij = <g_i, v_j> + s_i;  with P^f_ij = <qf_i, kf_f,j>,  dP^f = dA * prod_{f' != f} P^f';
    dqf = sum_f dP^f kf_f;  dkf_f = dP^f^T qf;  dv = A^T g."""
    qf = np.asarray(qf, F64)
    kfs = [np.asarray(k, F64) for k in kfs]
    v = np.asarray(v, F64)
    do = np.asarray(do, F64)
    o, A, eta = hla_bruteforce(qf, kfs, v, eps)
    den = eta + eps
    g = do / den[:, None]
    s = -(do * o).sum(axis=1) / den
    dA = g @ v.T + s[:, None]
    P = [qf @ k.T for k in kfs]
    dqf = np.zeros_like(qf)
    dkfs = []
    for f in range(len(kfs)):
        others = np.ones_like(A)
        for f2 in range(len(kfs)):
            if f2 != f:
                others = others * P[f2]
        dP = dA * others
        dqf += dP @ kfs[f]
        dkfs.append(dP.T @ qf)
    dv = A.T @ g
    return dqf, dkfs, dv


def hla_causal_backward_bruteforce(qf, kfs, v, do, eps: float, decay: float = 1.0):
    """Gradients of L = sum(O * dO) for the causal variant through the masked N x N matrix: with
    M_ij = decay^(i-j) for j <= i (0 otherwise) and A = M * prod_f P^f, the steps of
    hla_backward_bruteforce apply with every product carrying the mask:
    dP^f = (<g_i, v_j> + s_i) * M * prod_{f' != f} P^f'.  Returns (dqf, [dkf_f], dv)."""
    qf = np.asarray(qf, F64)
    kfs = [np.asarray(k, F64) for k in kfs]
    v = np.asarray(v, F64)
    do = np.asarray(do, F64)
    n = v.shape[0]
    dist = np.arange(n)[:, None] - np.arange(n)[None, :]
    M = np.where(dist >= 0, float(decay) ** np.maximum(dist, 0), 0.0)
    P = [qf @ k.T for k in kfs]
    A = M.copy()
    for Pf in P:
        A = A * Pf
    eta = A.sum(axis=1)
    den = eta + eps
    o = (A @ v) / den[:, None]
    g = do / den[:, None]
    s = -(do * o).sum(axis=1) / den
    dA = (g @ v.T + s[:, None]) * M
    dqf = np.zeros_like(qf)
    dkfs = []
    for f in range(len(kfs)):
        others = np.ones_like(A)
        for f2 in range(len(kfs)):
            if f2 != f:
                others = others * P[f2]
        dP = dA * others
        dqf += dP @ kfs[f]
        dkfs.append(dP.T @ qf)
    return dqf, dkfs, A.T @ g


def hla_causal_backward_sequential(qf, kfs, v, do, eps: float, decay: float = 1.0):
    """The same gradients through the state recursions (independent route): forward in time the
    states C^i, z^i of hla_causal_sequential give o_i and dT_q,i = C^i g_i + s_i z^i; backward in
    time the gradient states dC^j = decay dC^{j+1} + T_q,j (x) g_j and dz^j = decay dz^{j+1} +
    s_j T_q,j give dT_k,j = dC^j v_j + dz^j and dv_j = (dC^j)^T T_k,j.  Python loops: small inputs."""
    qf = np.asarray(qf, F64)
    kfs = [np.asarray(k, F64) for k in kfs]
    v = np.asarray(v, F64)
    do = np.asarray(do, F64)
    F = len(kfs)
    n, dp = qf.shape
    Tq = outer_features([qf] * F)
    Tk = outer_features(kfs)
    D = Tq.shape[1]
    C = np.zeros((D, v.shape[1]), F64)
    z = np.zeros(D, F64)
    g = np.zeros_like(v)
    s = np.zeros(n, F64)
    dTq = np.zeros((n, D), F64)
    for i in range(n):
        C = decay * C + np.outer(Tk[i], v[i])
        z = decay * z + Tk[i]
        den = Tq[i] @ z + eps
        o = (Tq[i] @ C) / den
        g[i] = do[i] / den
        s[i] = -(do[i] @ o) / den
        dTq[i] = C @ g[i] + s[i] * z
    dC = np.zeros((D, v.shape[1]), F64)
    dz = np.zeros(D, F64)
    dTk = np.zeros((n, D), F64)
    dv = np.zeros_like(v)
    for j in range(n - 1, -1, -1):
        dC = decay * dC + np.outer(Tq[j], g[j])
        dz = decay * dz + s[j] * Tq[j]
        dTk[j] = dC @ v[j] + dz
        dv[j] = Tk[j] @ dC
    shape = (n,) + (dp,) * F
    dqf = np.zeros_like(qf)
    for slot in range(F):
        dqf += _slot_gradient(dTq.reshape(shape), [qf] * F, slot)
    dkfs = [_slot_gradient(dTk.reshape(shape), kfs, slot) for slot in range(F)]
    return dqf, dkfs, dv


# --------------------------------------------------------------------------------------------
# Value modulation (Sec. 4.5): T <- T + phi_v1(T) * phi_v2(V), elementwise product
# --------------------------------------------------------------------------------------------
def layer_norm(u, gamma, beta, eps: float):
    """LayerNorm over the last axis: (u - mean) / sqrt(var + eps) * gamma + beta, var the biased
    (1/d) variance.  Returns (y, normalised u-hat, 1/sqrt(var + eps))."""
    u = np.asarray(u, F64)
    mu = u.mean(axis=-1, keepdims=True)
    var = ((u - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    uhat = (u - mu) * rstd
    return uhat * np.asarray(gamma, F64) + np.asarray(beta, F64), uhat, rstd


class PhiVWeights:
    """Weights of one value-modulation map phi_v (App. A.1): two linear layers d -> d -> d with
    a GELU in between, no ReLU, and a LayerNorm (gamma, beta).  The paper's figure of the
    network is missing from its text; the reading taken here puts the LayerNorm on the output
    of the second layer."""

    def __init__(self, W1, b1, W2, b2, gamma, beta):
        self.W1, self.b1, self.W2, self.b2, self.gamma, self.beta = (
            np.asarray(a, F64) for a in (W1, b1, W2, b2, gamma, beta))

    def astuple(self):
        return self.W1, self.b1, self.W2, self.b2, self.gamma, self.beta


def phi_v_forward(x, W1, b1, W2, b2, gamma, beta, ln_eps: float):
    """phi_v(x) = LayerNorm(GELU(x W1 + b1) W2 + b2) for rows x [N, d].
    Returns (m [N, d], h, u-hat, rstd) -- the last three are what the backward needs."""
    x = np.asarray(x, F64)
    h = x @ np.asarray(W1, F64) + np.asarray(b1, F64)
    u = gelu_erf(h) @ np.asarray(W2, F64) + np.asarray(b2, F64)
    m, uhat, rstd = layer_norm(u, gamma, beta, ln_eps)
    return m, h, uhat, rstd


def phi_v_backward(dm, x, W1, b1, W2, b2, gamma, beta, ln_eps: float):
    """Gradient w.r.t. x of a loss with gradient dm w.r.t. phi_v(x).  LayerNorm backward with
    g = dm * gamma: du = rstd * (g - mean(g) - u-hat * mean(g * u-hat)); then the two layers as in
    phi_backward (no ReLU)."""
    _, h, uhat, rstd = phi_v_forward(x, W1, b1, W2, b2, gamma, beta, ln_eps)
    g = np.asarray(dm, F64) * np.asarray(gamma, F64)
    du = rstd * (g - g.mean(axis=-1, keepdims=True) - uhat * (g * uhat).mean(axis=-1, keepdims=True))
    dh = (du @ np.asarray(W2, F64).T) * gelu_erf_grad(h)
    return dh @ np.asarray(W1, F64).T


def phi_v_weight_grads(dm, x, W1, b1, W2, b2, gamma, beta, ln_eps: float):
    """(dW1, db1, dW2, db2, dgamma, dbeta) of phi_v (App. A.1) for a loss with gradient dm w.r.t.
    phi_v(x), summed over the rows of x: dgamma = sum dm * u-hat, dbeta = sum dm, then du as in
    phi_v_backward, dW2 = GELU(h)^T du, db2 = sum du, dh = (du W2^T) * GELU'(h), dW1 = x^T dh,
    db1 = sum dh."""
    x = np.asarray(x, F64)
    dm = np.asarray(dm, F64)
    _, h, uhat, rstd = phi_v_forward(x, W1, b1, W2, b2, gamma, beta, ln_eps)
    g = dm * np.asarray(gamma, F64)
    du = rstd * (g - g.mean(axis=-1, keepdims=True) - uhat * (g * uhat).mean(axis=-1, keepdims=True))
    dh = (du @ np.asarray(W2, F64).T) * gelu_erf_grad(h)
    return (x.T @ dh, dh.sum(axis=0), gelu_erf(h).T @ du, du.sum(axis=0),
            (dm * uhat).sum(axis=0), dm.sum(axis=0))


def value_modulation_weight_grads(dout, t, v, pv1: PhiVWeights, pv2: PhiVWeights, ln_eps: float):
    """Weight gradients of the two maps of value_modulation_forward for rows [N, d]: phi_v1 sees
    the upstream gradient dOut * phi_v2(V), phi_v2 sees dOut * phi_v1(T).  Two tuples as
    phi_v_weight_grads returns them."""
    dout = np.asarray(dout, F64)
    m1 = phi_v_forward(t, *pv1.astuple(), ln_eps)[0]
    m2 = phi_v_forward(v, *pv2.astuple(), ln_eps)[0]
    return (phi_v_weight_grads(dout * m2, t, *pv1.astuple(), ln_eps),
            phi_v_weight_grads(dout * m1, v, *pv2.astuple(), ln_eps))


def value_modulation_forward(t, v, pv1: PhiVWeights, pv2: PhiVWeights, ln_eps: float):
    """Sec. 4.5: T + phi_v1(T) * phi_v2(V) (elementwise), T = A V the normalised attention output,
    rows [N, d]."""
    t = np.asarray(t, F64)
    m1 = phi_v_forward(t, *pv1.astuple(), ln_eps)[0]
    m2 = phi_v_forward(v, *pv2.astuple(), ln_eps)[0]
    return t + m1 * m2


def value_modulation_backward(dout, t, v, pv1: PhiVWeights, pv2: PhiVWeights, ln_eps: float):
    """(dT, dV) of value_modulation_forward: dT = dOut + phi_v1'(T)^T (dOut * phi_v2(V)),
    dV = phi_v2'(V)^T (dOut * phi_v1(T))."""
    dout = np.asarray(dout, F64)
    m1 = phi_v_forward(t, *pv1.astuple(), ln_eps)[0]
    m2 = phi_v_forward(v, *pv2.astuple(), ln_eps)[0]
    dt = dout + phi_v_backward(dout * m2, t, *pv1.astuple(), ln_eps)
    dv = phi_v_backward(dout * m1, v, *pv2.astuple(), ln_eps)
    return dt, dv


# --------------------------------------------------------------------------------------------
# Whole operator over batch / heads / packed sequences (Alg. 1 Steps 4-5)
# --------------------------------------------------------------------------------------------
class PhiWeights:
    """Weights of one feature map: W1 [d,d], b1 [d], W2 [d,d_phi], b2 [d_phi]; shared by all
    heads (App. A.1 sizes the first layer by the head dimension)."""

    def __init__(self, W1, b1, W2, b2):
        self.W1 = np.asarray(W1, F64)
        self.b1 = np.asarray(b1, F64)
        self.W2 = np.asarray(W2, F64)
        self.b2 = np.asarray(b2, F64)

    def astuple(self):
        return self.W1, self.b1, self.W2, self.b2


def _units(B: int, N: int, cu_seqlens: Optional[Sequence[int]]):
    """(batch index, first token, one-past-last token) of every independent sequence."""
    if cu_seqlens is None:
        return [(b, 0, N) for b in range(B)]
    if B != 1:
        raise ValueError("packed input needs B == 1")
    cu = list(cu_seqlens)
    return [(0, cu[s], cu[s + 1]) for s in range(len(cu) - 1)]


def _features(Q, K, lo, hi, b, h, F, d_phi, phi: Optional[Sequence[PhiWeights]]):
    if phi is None:  # features handed in: Q is [.., d_phi], K is [.., F*d_phi] factor-major
        qf = np.asarray(Q[b, h, lo:hi], F64)
        kk = np.asarray(K[b, h, lo:hi], F64)
        kfs = [kk[:, f * d_phi:(f + 1) * d_phi] for f in range(F)]
    else:
        qf = phi_forward(Q[b, h, lo:hi], *phi[0].astuple())[0]
        kfs = [phi_forward(K[b, h, lo:hi], *phi[1 + f].astuple())[0] for f in range(F)]
    return qf, kfs


def hla_operator_forward(Q, K, V, F: int, d_phi: int, eps: float,
                         phi: Optional[Sequence[PhiWeights]] = None,
                         cu_seqlens: Optional[Sequence[int]] = None,
                         route: str = "factorized", vmod=None, causal: bool = False,
                         decay: float = 1.0) -> np.ndarray:
    """O [B,H,N,d] for Q,K,V [B,H,N,*].  `phi` = [phi_q, phi_k1..phi_kF] or None when Q and K
    already hold features.  Sequences (batch entries, or the packed ranges of cu_seqlens) never
    share state.  vmod = (phi_v1, phi_v2, ln_eps) applies the value modulation of Sec. 4.5 to the
    attention output, token by token (maps shared by all heads).  causal: the masked variant of
    Sec. 4.4 inside every sequence (route 'bruteforce' = masked N x N matrix, 'factorized' = the
    sequential state updates), `decay` its decay factor (see hla_causal_bruteforce)."""
    B, H, N = V.shape[:3]
    O = np.zeros(V.shape, F64)
    for (b, lo, hi) in _units(B, N, cu_seqlens):
        if hi == lo:
            continue
        for h in range(H):
            qf, kfs = _features(Q, K, lo, hi, b, h, F, d_phi, phi)
            v = np.asarray(V[b, h, lo:hi], F64)
            if causal:
                O[b, h, lo:hi] = (hla_causal_sequential if route == "factorized" else
                                  hla_causal_bruteforce)(qf, kfs, v, eps, decay=decay)
            elif route == "factorized":
                O[b, h, lo:hi] = hla_factorized(qf, kfs, v, eps)[0]
            elif route == "bruteforce":
                O[b, h, lo:hi] = hla_bruteforce(qf, kfs, v, eps)[0]
            else:
                raise ValueError(route)
            if vmod is not None:
                O[b, h, lo:hi] = value_modulation_forward(O[b, h, lo:hi], v, vmod[0], vmod[1], vmod[2])
    return O


def hla_operator_backward(Q, K, V, dO, F: int, d_phi: int, eps: float,
                          phi: Optional[Sequence[PhiWeights]] = None,
                          cu_seqlens: Optional[Sequence[int]] = None,
                          route: str = "factorized", weight_grads: bool = False,
                          feature_grads: bool = False, vmod=None, vmod_weight_grads: bool = False,
                          causal: bool = False, decay: float = 1.0):
    """(dQ, dK, dV) with the shapes of Q, K, V for L = sum(O * dO).  With feature maps, dK sums
    the contributions of the F key maps (they all read the same K).  With weight_grads (needs
    `phi`) a fourth result lists (dW1, db1, dW2, db2) for phi_q, phi_k1..phi_kF, each summed over
    every sequence, head and token that shares the map.  With feature_grads the last result is
    the gradient w.r.t. the features themselves, (dqf [B,H,N,d_phi], dkf [B,H,N,F*d_phi]), the
    intermediate that the feature maps' backward consumes.  vmod as in hla_operator_forward: dO
    is then the gradient w.r.t. the modulated output; it is first taken back through the
    modulation (to the attention output T and to V), T's share then goes through the operator.
    With vmod_weight_grads (needs `vmod`) the last result lists (dW1, db1, dW2, db2, dgamma,
    dbeta) for phi_v1 and phi_v2, summed over every sequence, head and token.
    causal / decay: the masked variant of Sec. 4.4 (route 'bruteforce' = masked matrix,
    'factorized' = the state recursions).  With vmod as well, T is the causal output: the
    modulation acts token by token on (T, V), so the chain rule is the same composition."""
    B, H, N = V.shape[:3]
    dQ = np.zeros(Q.shape, F64)
    dK = np.zeros(K.shape, F64)
    dV = np.zeros(V.shape, F64)
    wg = None
    dQf = np.zeros(Q.shape[:3] + (d_phi,), F64)
    dKf = np.zeros(K.shape[:3] + (F * d_phi,), F64)
    if weight_grads:
        if phi is None:
            raise ValueError("weight gradients need the feature maps")
        wg = [[np.zeros_like(a) for a in m.astuple()] for m in phi]
    vwg = None
    if vmod_weight_grads:
        if vmod is None:
            raise ValueError("the modulation's weight gradients need the modulation")
        vwg = [[np.zeros_like(a) for a in m.astuple()] for m in vmod[:2]]
    bwd = hla_backward_factorized if route == "factorized" else hla_backward_bruteforce
    if causal:
        cb = hla_causal_backward_sequential if route == "factorized" else hla_causal_backward_bruteforce
        bwd = lambda qf, kfs, v, do, eps: cb(qf, kfs, v, do, eps, decay=decay)
    for (b, lo, hi) in _units(B, N, cu_seqlens):
        if hi == lo:
            continue
        for h in range(H):
            qf, kfs = _features(Q, K, lo, hi, b, h, F, d_phi, phi)
            v = np.asarray(V[b, h, lo:hi], F64)
            do = np.asarray(dO[b, h, lo:hi], F64)
            dv_mod = 0.0
            if vmod is not None:
                if causal:
                    t = (hla_causal_sequential if route == "factorized" else
                         hla_causal_bruteforce)(qf, kfs, v, eps, decay=decay)
                else:
                    t = (hla_factorized if route == "factorized" else hla_bruteforce)(qf, kfs, v, eps)[0]
                if vwg is not None:
                    for m, part in enumerate(value_modulation_weight_grads(do, t, v, vmod[0], vmod[1], vmod[2])):
                        for a, da in zip(vwg[m], part):
                            a += da
                do, dv_mod = value_modulation_backward(do, t, v, vmod[0], vmod[1], vmod[2])
            dqf, dkfs, dv = bwd(qf, kfs, v, do, eps)
            dV[b, h, lo:hi] = dv + dv_mod
            dQf[b, h, lo:hi] = dqf
            dKf[b, h, lo:hi] = np.concatenate(dkfs, axis=1)
            if phi is None:
                dQ[b, h, lo:hi] = dqf
                dK[b, h, lo:hi] = np.concatenate(dkfs, axis=1)
            else:
                dQ[b, h, lo:hi] = phi_backward(dqf, Q[b, h, lo:hi], *phi[0].astuple())
                acc = np.zeros((hi - lo, K.shape[-1]), F64)
                for f in range(F):
                    acc += phi_backward(dkfs[f], K[b, h, lo:hi], *phi[1 + f].astuple())
                dK[b, h, lo:hi] = acc
                if wg is not None:
                    parts = [phi_weight_grads(dqf, Q[b, h, lo:hi], *phi[0].astuple())]
                    parts += [phi_weight_grads(dkfs[f], K[b, h, lo:hi], *phi[1 + f].astuple())
                              for f in range(F)]
                    for m, part in enumerate(parts):
                        for a, da in zip(wg[m], part):
                            a += da
    res = (dQ, dK, dV)
    if wg is not None:
        res += ([tuple(m) for m in wg],)
    if feature_grads:
        res += ((dQf, dKf),)
    if vwg is not None:
        res += ([tuple(m) for m in vwg],)
    return res


def hla_bruteforce_rows(qf_rows, kfs, v, eps: float) -> np.ndarray:
    """Brute-force outputs for a subset of query rows against ALL keys: O(rows * N).  Used to
    spot-check full-size problems against the plain definition."""
    return hla_bruteforce(qf_rows, kfs, v, eps)[0]

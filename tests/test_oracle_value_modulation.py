"""Pins for the oracle's value modulation (Sec. 4.5: T <- T + phi_v1(T) * phi_v2(V); phi_v of
App. A.1 with a LayerNorm on its output): LayerNorm against scalar loops and its invariances,
the identity special case, the closed form for a one-channel-pair check, and every gradient
against central finite differences, alone and through the whole operator."""
import math

import numpy as np
import pytest

from oracle import hla_oracle as orc


def _fd(fun, x, h=1e-6):
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + h
        fp = fun()
        x[i] = old - h
        fm = fun()
        x[i] = old
        g[i] = (fp - fm) / (2 * h)
    return g


def _pv(rng, d, scale=1.0):
    return orc.PhiVWeights(scale * rng.standard_normal((d, d)), 0.3 * rng.standard_normal(d),
                           rng.standard_normal((d, d)) / math.sqrt(d), 0.3 * rng.standard_normal(d),
                           1.0 + 0.2 * rng.standard_normal(d), 0.2 * rng.standard_normal(d))


def test_layer_norm_against_scalar_loops_and_invariances():
    rng = np.random.default_rng(70)
    n, d, eps = 4, 7, 1e-5
    u = rng.standard_normal((n, d)) * 3 + 1
    gamma, beta = rng.standard_normal(d), rng.standard_normal(d)
    y, uhat, rstd = orc.layer_norm(u, gamma, beta, eps)
    for i in range(n):
        mean = sum(u[i, c] for c in range(d)) / d
        var = sum((u[i, c] - mean) ** 2 for c in range(d)) / d      # biased, as the usual definition
        for c in range(d):
            want = (u[i, c] - mean) / math.sqrt(var + eps) * gamma[c] + beta[c]
            assert abs(y[i, c] - want) <= 1e-13 * max(1.0, abs(want))
    # with gamma = 1, beta = 0, eps = 0: zero mean, unit variance, invariant to shift and positive scale
    y0 = orc.layer_norm(u, np.ones(d), np.zeros(d), 0.0)[0]
    np.testing.assert_allclose(y0.mean(axis=1), 0.0, atol=1e-14)
    np.testing.assert_allclose((y0 ** 2).mean(axis=1), 1.0, rtol=1e-13)
    np.testing.assert_allclose(orc.layer_norm(3.7 * u + 11.0, np.ones(d), np.zeros(d), 0.0)[0], y0,
                               rtol=1e-11, atol=1e-12)


def test_zero_second_factor_is_the_identity_and_known_product():
    rng = np.random.default_rng(71)
    n, d, eps = 6, 5, 1e-5
    t, v = rng.standard_normal((n, d)), rng.standard_normal((n, d))
    pv1 = _pv(rng, d)
    zero = orc.PhiVWeights(rng.standard_normal((d, d)), rng.standard_normal(d), np.zeros((d, d)),
                           np.zeros(d), np.ones(d), np.zeros(d))   # constant input to the LayerNorm -> beta = 0
    np.testing.assert_array_equal(orc.value_modulation_forward(t, v, pv1, zero, eps), t)
    # a map whose LayerNorm input is constant returns beta exactly: the product is then elementwise known
    const = orc.PhiVWeights(np.zeros((d, d)), np.zeros(d), np.zeros((d, d)), np.full(d, 2.5), np.ones(d),
                            np.arange(d, dtype=float))
    const2 = orc.PhiVWeights(np.zeros((d, d)), np.zeros(d), np.zeros((d, d)), np.full(d, -1.0), np.ones(d),
                             np.full(d, 0.5))
    out = orc.value_modulation_forward(t, v, const, const2, eps)
    np.testing.assert_allclose(out, t + np.arange(d) * 0.5, rtol=0, atol=1e-15)


def test_phi_v_against_scalar_loops():
    rng = np.random.default_rng(72)
    n, d, eps = 3, 4, 1e-5
    x = rng.standard_normal((n, d))
    pv = _pv(rng, d)
    m = orc.phi_v_forward(x, *pv.astuple(), eps)[0]
    for i in range(n):
        h = [sum(x[i, a] * pv.W1[a, j] for a in range(d)) + pv.b1[j] for j in range(d)]
        g = [hj * 0.5 * (1.0 + math.erf(hj / math.sqrt(2.0))) for hj in h]
        u = [sum(g[j] * pv.W2[j, c] for j in range(d)) + pv.b2[c] for c in range(d)]
        mean = sum(u) / d
        var = sum((uc - mean) ** 2 for uc in u) / d
        for c in range(d):
            want = (u[c] - mean) / math.sqrt(var + eps) * pv.gamma[c] + pv.beta[c]
            assert abs(m[i, c] - want) <= 1e-12 * max(1.0, abs(want))


def test_modulation_backward_against_finite_differences():
    rng = np.random.default_rng(73)
    n, d, eps = 5, 6, 1e-5
    t, v, dout = (rng.standard_normal((n, d)) for _ in range(3))
    pv1, pv2 = _pv(rng, d), _pv(rng, d)
    f = lambda: float((orc.value_modulation_forward(t, v, pv1, pv2, eps) * dout).sum())
    dt, dv = orc.value_modulation_backward(dout, t, v, pv1, pv2, eps)
    np.testing.assert_allclose(dt, _fd(f, t), rtol=2e-6, atol=1e-8)
    np.testing.assert_allclose(dv, _fd(f, v), rtol=2e-6, atol=1e-8)
    # the map alone
    w = rng.standard_normal((n, d))
    fm = lambda: float((orc.phi_v_forward(t, *pv1.astuple(), eps)[0] * w).sum())
    np.testing.assert_allclose(orc.phi_v_backward(w, t, *pv1.astuple(), eps), _fd(fm, t), rtol=2e-6, atol=1e-8)


@pytest.mark.parametrize("packed", [False, True])
def test_operator_with_modulation_against_finite_differences(packed):
    rng = np.random.default_rng(74)
    B, H, N, d, F, dp = (1, 2, 7, 4, 3, 3) if packed else (2, 1, 5, 4, 2, 3)
    cu = [0, 3, 7] if packed else None
    Q, K, V, dO = (rng.standard_normal((B, H, N, d)) for _ in range(4))
    phi = [orc.PhiWeights(rng.standard_normal((d, d)), 0.3 * rng.standard_normal(d),
                          rng.standard_normal((d, dp)), rng.standard_normal(dp) + 1.5)
           for _ in range(1 + F)]
    vmod = (_pv(rng, d, 3.0), _pv(rng, d), 1e-5)
    eps = 1e-4
    f = lambda: float((orc.hla_operator_forward(Q, K, V, F, dp, eps, phi=phi, cu_seqlens=cu,
                                                route="bruteforce", vmod=vmod) * dO).sum())
    for route in ("factorized", "bruteforce"):
        dQ, dK, dV = orc.hla_operator_backward(Q, K, V, dO, F, dp, eps, phi=phi, cu_seqlens=cu,
                                               route=route, vmod=vmod)
        np.testing.assert_allclose(dQ, _fd(f, Q), rtol=5e-6, atol=5e-8)
        np.testing.assert_allclose(dK, _fd(f, K), rtol=5e-6, atol=5e-8)
        np.testing.assert_allclose(dV, _fd(f, V), rtol=5e-6, atol=5e-8)
    # the modulated output differs from the plain one and reduces to it when phi_v2 vanishes
    plain = orc.hla_operator_forward(Q, K, V, F, dp, eps, phi=phi, cu_seqlens=cu)
    mod = orc.hla_operator_forward(Q, K, V, F, dp, eps, phi=phi, cu_seqlens=cu, vmod=vmod)
    assert np.abs(mod - plain).max() > 1e-3
    zero = orc.PhiVWeights(np.zeros((d, d)), np.zeros(d), np.zeros((d, d)), np.zeros(d), np.ones(d), np.zeros(d))
    np.testing.assert_array_equal(
        orc.hla_operator_forward(Q, K, V, F, dp, eps, phi=phi, cu_seqlens=cu, vmod=(vmod[0], zero, 1e-5)), plain)


def test_modulation_weight_gradients_against_finite_differences():
    """Every weight array of both maps, perturbed entry by entry through the forward alone."""
    rng = np.random.default_rng(75)
    n, d, eps = 6, 5, 1e-5
    t, v, dout = (rng.standard_normal((n, d)) for _ in range(3))
    pv1, pv2 = _pv(rng, d, 2.0), _pv(rng, d)
    f = lambda: float((orc.value_modulation_forward(t, v, pv1, pv2, eps) * dout).sum())
    got = orc.value_modulation_weight_grads(dout, t, v, pv1, pv2, eps)
    for pv, grads in zip((pv1, pv2), got):
        assert len(grads) == 6
        for arr, ga in zip(pv.astuple(), grads):
            assert ga.shape == arr.shape
            np.testing.assert_allclose(ga, _fd(f, arr), rtol=5e-6, atol=2e-8)
    # closed forms that need no derivative of the network: d/dbeta_1 = sum_t dOut * phi_v2(V),
    # d/dgamma_1 = sum_t dOut * phi_v2(V) * u-hat_1
    m2 = orc.phi_v_forward(v, *pv2.astuple(), eps)[0]
    uhat1 = orc.phi_v_forward(t, *pv1.astuple(), eps)[2]
    np.testing.assert_allclose(got[0][5], (dout * m2).sum(axis=0), rtol=1e-13)
    np.testing.assert_allclose(got[0][4], (dout * m2 * uhat1).sum(axis=0), rtol=1e-13)
    # the second layer's bias cannot move a LayerNorm's output by a common shift: db2 sums to zero
    assert abs(got[0][3].sum()) < 1e-12 * np.abs(got[0][3]).sum() + 1e-15


def test_operator_modulation_weight_gradients_sum_over_heads_and_sequences():
    rng = np.random.default_rng(76)
    B, H, N, d, F, dp = 1, 2, 7, 4, 3, 3
    cu = [0, 3, 7]
    Q, K, V, dO = (rng.standard_normal((B, H, N, d)) for _ in range(4))
    phi = [orc.PhiWeights(rng.standard_normal((d, d)), 0.3 * rng.standard_normal(d),
                          rng.standard_normal((d, dp)), rng.standard_normal(dp) + 1.5)
           for _ in range(1 + F)]
    vmod = (_pv(rng, d, 3.0), _pv(rng, d), 1e-5)
    eps = 1e-4
    f = lambda: float((orc.hla_operator_forward(Q, K, V, F, dp, eps, phi=phi, cu_seqlens=cu,
                                                route="bruteforce", vmod=vmod) * dO).sum())
    res = orc.hla_operator_backward(Q, K, V, dO, F, dp, eps, phi=phi, cu_seqlens=cu, vmod=vmod,
                                    vmod_weight_grads=True)
    for pv, grads in zip(vmod[:2], res[-1]):
        for arr, ga in zip(pv.astuple(), grads):
            np.testing.assert_allclose(ga, _fd(f, arr), rtol=1e-5, atol=1e-7)
    with pytest.raises(ValueError):
        orc.hla_operator_backward(Q, K, V, dO, F, dp, eps, phi=phi, vmod_weight_grads=True)

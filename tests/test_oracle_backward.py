"""Pins for the oracle's backward: central finite differences of the forward (which is itself
pinned in test_oracle_forward.py), agreement of the two independent gradient routes, and
structural facts (scale invariance => <dq, q> = 0; linearity in V)."""
import numpy as np
import pytest

from oracle import hla_oracle as orc


def _loss_feats(q, ks, v, do, eps):
    return float((orc.hla_bruteforce(q, ks, v, eps)[0] * do).sum())


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


@pytest.mark.parametrize("F,dp", [(1, 5), (2, 4), (3, 3), (3, 6)])
def test_feature_level_backward_against_finite_differences(F, dp):
    rng = np.random.default_rng(30 + F * 10 + dp)
    n, d, eps = 7, 3, 1e-3
    q = np.abs(rng.standard_normal((n, dp))) + 0.2
    ks = [np.abs(rng.standard_normal((n, dp))) + 0.2 for _ in range(F)]
    v = rng.standard_normal((n, d))
    do = rng.standard_normal((n, d))
    for route in (orc.hla_backward_factorized, orc.hla_backward_bruteforce):
        dq, dks, dv = route(q, ks, v, do, eps)
        f = lambda: _loss_feats(q, ks, v, do, eps)
        np.testing.assert_allclose(dq, _fd(f, q), rtol=2e-7, atol=1e-8)
        for a in range(F):
            np.testing.assert_allclose(dks[a], _fd(f, ks[a]), rtol=2e-7, atol=1e-8)
        np.testing.assert_allclose(dv, _fd(f, v), rtol=2e-7, atol=1e-8)


@pytest.mark.parametrize("F,dp", [(2, 12), (3, 6)])
def test_backward_routes_agree(F, dp):
    rng = np.random.default_rng(40 + F)
    n, d = 50, 8
    q = np.abs(rng.standard_normal((n, dp)))
    ks = [np.abs(rng.standard_normal((n, dp))) for _ in range(F)]
    v = rng.standard_normal((n, d))
    do = rng.standard_normal((n, d))
    a = orc.hla_backward_factorized(q, ks, v, do, 1e-6)
    b = orc.hla_backward_bruteforce(q, ks, v, do, 1e-6)
    np.testing.assert_allclose(a[0], b[0], rtol=1e-9, atol=1e-12)
    for x, y in zip(a[1], b[1]):
        np.testing.assert_allclose(x, y, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(a[2], b[2], rtol=1e-9, atol=1e-12)


def test_scale_invariance_makes_query_gradient_orthogonal():
    # eps = 0: the output does not change when a query's features are rescaled, so the gradient
    # has no component along the features; the same holds for each key map scaled as a whole.
    rng = np.random.default_rng(50)
    n, dp, d, F = 20, 6, 5, 3
    q = np.abs(rng.standard_normal((n, dp)))
    ks = [np.abs(rng.standard_normal((n, dp))) for _ in range(F)]
    v = rng.standard_normal((n, d))
    do = rng.standard_normal((n, d))
    dq, dks, dv = orc.hla_backward_factorized(q, ks, v, do, 0.0)
    scale = np.abs(dq).max() * np.abs(q).max()
    assert np.abs((dq * q).sum(1)).max() <= 1e-12 * scale * dp
    for f in range(F):
        assert abs((dks[f] * ks[f]).sum()) <= 1e-10 * np.abs(dks[f]).sum() * np.abs(ks[f]).max()
    # linear in V: dV does not depend on V, and <dV, V> = L
    dv2 = orc.hla_backward_factorized(q, ks, 3.0 * v + 1.0, do, 0.0)[2]
    np.testing.assert_allclose(dv2, dv, rtol=1e-11, atol=1e-13)
    L = _loss_feats(q, ks, v, do, 0.0)
    assert abs((dv * v).sum() - L) <= 1e-11 * max(1.0, abs(L))


def test_phi_backward_against_finite_differences():
    rng = np.random.default_rng(51)
    n, d, dp = 5, 6, 4
    x = rng.standard_normal((n, d))
    W1, b1 = rng.standard_normal((d, d)), rng.standard_normal(d)
    W2, b2 = rng.standard_normal((d, dp)), rng.standard_normal(dp)
    w = rng.standard_normal((n, dp))
    f = lambda: float((orc.phi_forward(x, W1, b1, W2, b2)[0] * w).sum())
    dx = orc.phi_backward(w, x, W1, b1, W2, b2)
    np.testing.assert_allclose(dx, _fd(f, x), rtol=1e-6, atol=1e-8)
    # clipped features pass no gradient
    feat = orc.phi_forward(x, W1, b1, W2, b2)[0]
    assert (feat == 0).any()
    w0 = np.where(feat == 0, w, 0.0)
    assert np.all(orc.phi_backward(w0, x, W1, b1, W2, b2) == 0.0)


@pytest.mark.parametrize("packed", [False, True])
def test_operator_backward_with_feature_maps_against_finite_differences(packed):
    rng = np.random.default_rng(52)
    B, H, N, d, F, dp = (1, 2, 9, 4, 3, 3) if packed else (2, 1, 5, 4, 3, 3)
    cu = [0, 4, 9] if packed else None
    Q, K, V, dO = (rng.standard_normal((B, H, N, d)) for _ in range(4))
    phi = [orc.PhiWeights(rng.standard_normal((d, d)), 0.3 * rng.standard_normal(d),
                          rng.standard_normal((d, dp)), rng.standard_normal(dp) + 1.5)
           for _ in range(1 + F)]
    eps = 1e-4
    f = lambda: float((orc.hla_operator_forward(Q, K, V, F, dp, eps, phi=phi, cu_seqlens=cu,
                                                route="bruteforce") * dO).sum())
    for route in ("factorized", "bruteforce"):
        dQ, dK, dV = orc.hla_operator_backward(Q, K, V, dO, F, dp, eps, phi=phi, cu_seqlens=cu,
                                               route=route)
        np.testing.assert_allclose(dQ, _fd(f, Q), rtol=2e-6, atol=2e-8)
        np.testing.assert_allclose(dK, _fd(f, K), rtol=2e-6, atol=2e-8)
        np.testing.assert_allclose(dV, _fd(f, V), rtol=2e-6, atol=2e-8)


def test_operator_backward_feature_level_layout():
    # K gradients come back factor-major in the last dim, matching the input layout
    rng = np.random.default_rng(53)
    B, H, N, d, F, dp = 1, 2, 6, 3, 2, 3
    Q = np.abs(rng.standard_normal((B, H, N, dp))) + 0.1
    K = np.abs(rng.standard_normal((B, H, N, F * dp))) + 0.1
    V, dO = rng.standard_normal((B, H, N, d)), rng.standard_normal((B, H, N, d))
    f = lambda: float((orc.hla_operator_forward(Q, K, V, F, dp, 1e-5) * dO).sum())
    dQ, dK, dV = orc.hla_operator_backward(Q, K, V, dO, F, dp, 1e-5)
    np.testing.assert_allclose(dK, _fd(f, K), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(dQ, _fd(f, Q), rtol=1e-6, atol=1e-8)


def test_phi_weight_grads_against_finite_differences():
    # one feature map alone: L = sum(phi(x) * w), every weight entry perturbed in turn
    rng = np.random.default_rng(54)
    n, d, dp = 6, 5, 3
    x = rng.standard_normal((n, d))
    W1, b1 = rng.standard_normal((d, d)), rng.standard_normal(d)
    W2, b2 = rng.standard_normal((d, dp)), rng.standard_normal(dp) + 0.5
    w = rng.standard_normal((n, dp))
    f = lambda: float((orc.phi_forward(x, W1, b1, W2, b2)[0] * w).sum())
    dW1, db1, dW2, db2 = orc.phi_weight_grads(w, x, W1, b1, W2, b2)
    np.testing.assert_allclose(dW1, _fd(f, W1), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(db1, _fd(f, b1), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(dW2, _fd(f, W2), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(db2, _fd(f, b2), rtol=1e-6, atol=1e-8)
    # a transposed operand or a dropped GELU' would survive none of the above; the shapes pin
    # the orientation (W1 acts from the right: rows = input channels)
    assert dW1.shape == (d, d) and dW2.shape == (d, dp)
    # rows are independent: the gradient of the whole batch is the sum of per-row gradients
    parts = [orc.phi_weight_grads(w[i:i + 1], x[i:i + 1], W1, b1, W2, b2) for i in range(n)]
    for k, whole in enumerate((dW1, db1, dW2, db2)):
        np.testing.assert_allclose(sum(p[k] for p in parts), whole, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("packed", [False, True])
def test_operator_weight_grads_against_finite_differences(packed):
    # the whole operator: L = sum(O * dO) differentiated w.r.t. every weight of every map, with
    # the maps shared by all heads, batch rows and packed sequences
    rng = np.random.default_rng(55)
    B, H, N, d, F, dp = (1, 2, 7, 3, 3, 2) if packed else (2, 2, 4, 3, 3, 2)
    cu = [0, 3, 7] if packed else None
    Q, K, V, dO = (rng.standard_normal((B, H, N, d)) for _ in range(4))
    phi = [orc.PhiWeights(rng.standard_normal((d, d)), 0.3 * rng.standard_normal(d),
                          rng.standard_normal((d, dp)), rng.standard_normal(dp) + 1.5)
           for _ in range(1 + F)]
    eps = 1e-4
    f = lambda: float((orc.hla_operator_forward(Q, K, V, F, dp, eps, phi=phi, cu_seqlens=cu,
                                                route="bruteforce") * dO).sum())
    for route in ("factorized", "bruteforce"):
        res = orc.hla_operator_backward(Q, K, V, dO, F, dp, eps, phi=phi, cu_seqlens=cu,
                                        route=route, weight_grads=True)
        assert len(res) == 4 and len(res[3]) == 1 + F
        for m, grads in enumerate(res[3]):
            for arr, g in zip(phi[m].astuple(), grads):
                np.testing.assert_allclose(g, _fd(f, arr), rtol=5e-6, atol=5e-8)
        # input gradients are unchanged by asking for the weight gradients
        plain = orc.hla_operator_backward(Q, K, V, dO, F, dp, eps, phi=phi, cu_seqlens=cu,
                                          route=route)
        for a, b in zip(plain, res[:3]):
            np.testing.assert_array_equal(a, b)


def test_weight_grads_need_feature_maps():
    rng = np.random.default_rng(56)
    Q = np.abs(rng.standard_normal((1, 1, 3, 2)))
    K = np.abs(rng.standard_normal((1, 1, 3, 4)))
    V = rng.standard_normal((1, 1, 3, 2))
    with pytest.raises(ValueError):
        orc.hla_operator_backward(Q, K, V, V, 2, 2, 1e-6, weight_grads=True)


def test_relu_branch_choices():
    # With a branch choice given, the feature map is differentiated as mask * u(x): the gradients
    # must equal the finite differences of exactly that (smooth) function, and with the oracle's
    # own decisions nothing changes.
    rng = np.random.default_rng(57)
    n, d, dp = 6, 5, 4
    x = rng.standard_normal((n, d))
    W1, b1 = rng.standard_normal((d, d)), rng.standard_normal(d)
    W2, b2 = rng.standard_normal((d, dp)), rng.standard_normal(dp)
    w = rng.standard_normal((n, dp))
    own = orc.phi_forward(x, W1, b1, W2, b2)[2] > 0
    assert own.any() and not own.all()
    np.testing.assert_array_equal(orc.phi_backward(w, x, W1, b1, W2, b2, relu_open=own),
                                  orc.phi_backward(w, x, W1, b1, W2, b2))
    mask = rng.random((n, dp)) < 0.5  # decisions that differ from the oracle's own
    assert (mask != own).any()
    f = lambda: float((orc.phi_forward(x, W1, b1, W2, b2)[2] * mask * w).sum())
    np.testing.assert_allclose(orc.phi_backward(w, x, W1, b1, W2, b2, relu_open=mask), _fd(f, x),
                               rtol=1e-6, atol=1e-8)
    dW1, db1, dW2, db2 = orc.phi_weight_grads(w, x, W1, b1, W2, b2, relu_open=mask)
    np.testing.assert_allclose(dW1, _fd(f, W1), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(db1, _fd(f, b1), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(dW2, _fd(f, W2), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(db2, _fd(f, b2), rtol=1e-6, atol=1e-8)


def _branch_setup(seed, n=9, d=5, dp=3, nmaps=2):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, d))
    maps = [(rng.standard_normal((d, d)), rng.standard_normal(d), rng.standard_normal((d, dp)),
             0.3 * rng.standard_normal(dp)) for _ in range(nmaps)]
    dfeats = [rng.standard_normal((n, dp)) for _ in range(nmaps)]
    return x, maps, dfeats


def test_phi_backward_branches_enumerates_every_choice():
    x, maps, dfeats = _branch_setup(58)
    us = [orc.phi_forward(x, *m)[2] for m in maps]
    allu = np.abs(np.concatenate(us, axis=1))
    band = float(np.sort(allu.ravel())[7]) * 1.0001  # the seven smallest |u| are "in band"
    br = orc.phi_backward_branches(dfeats, x, maps, band)
    inband_rows = np.nonzero((allu < band).any(axis=1))[0]
    assert sorted(br) == [int(r) for r in inband_rows] and len(br) >= 2
    own = sum(orc.phi_backward(df, x, *m) for df, m in zip(dfeats, maps))
    for n, cands in br.items():
        slots = [(m, a) for m in range(len(maps)) for a in range(us[m].shape[1]) if abs(us[m][n, a]) < band]
        assert cands.shape == (2 ** len(slots), x.shape[1])
        # the oracle's own decisions are one of the choices, at the index their bits spell
        bits = sum((1 << i) for i, (m, a) in enumerate(slots) if us[m][n, a] > 0)
        np.testing.assert_allclose(cands[bits], own[n], rtol=1e-12, atol=1e-14)
        # every choice is the finite difference of the correspondingly masked (smooth) maps
        for b in range(cands.shape[0]):
            masks = [(u[n] > 0) & (np.abs(u[n]) >= band) for u in us]
            for i, (m, a) in enumerate(slots):
                masks[m][a] = bool((b >> i) & 1)
            xr = x[n:n + 1].copy()
            f = lambda: float(sum((orc.phi_forward(xr, *maps[m])[2][0] * masks[m] * dfeats[m][n]).sum()
                                  for m in range(len(maps))))
            np.testing.assert_allclose(cands[b], _fd(f, xr)[0], rtol=1e-6, atol=1e-8)
        # choices that differ in one open feature with a non-zero gradient are different rows
        if cands.shape[0] > 1:
            assert np.abs(cands[1] - cands[0]).max() > 0
    # nothing is in band at resolution zero; too many in-band features in a row are refused
    assert orc.phi_backward_branches(dfeats, x, maps, 0.0) == {}
    with pytest.raises(ValueError):
        orc.phi_backward_branches(dfeats, x, maps, 1e9, max_inband=3)


def test_phi_weight_grad_branches_are_linear_in_the_choices():
    x, maps, dfeats = _branch_setup(59, n=11)
    m, df = maps[0], dfeats[0]
    u = orc.phi_forward(x, *m)[2]
    band = float(np.sort(np.abs(u).ravel())[5]) * 1.0001
    base, pairs, contribs, own = orc.phi_weight_grad_branches(df, x, *m, band)
    assert len(pairs) == 6 == len(contribs) == len(own)
    assert all(abs(u[n, a]) < band for n, a in pairs)
    # the oracle's own decisions reproduce phi_weight_grads
    ref = orc.phi_weight_grads(df, x, *m)
    for k in range(4):
        tot = base[k] + sum(c[k] for c, o in zip(contribs, own) if o)
        np.testing.assert_allclose(tot, ref[k], rtol=1e-12, atol=1e-13)
    # an arbitrary choice equals phi_weight_grads under the corresponding mask
    rng = np.random.default_rng(60)
    choice = rng.random(len(pairs)) < 0.5
    mask = (u > 0) & (np.abs(u) >= band)
    for (n, a), c in zip(pairs, choice):
        mask[n, a] = c
    ref = orc.phi_weight_grads(df, x, *m, relu_open=mask)
    for k in range(4):
        tot = base[k] + sum(c[k] for c, ch in zip(contribs, choice) if ch)
        np.testing.assert_allclose(tot, ref[k], rtol=1e-12, atol=1e-13)
    assert orc.phi_weight_grad_branches(df, x, *m, 0.0)[1] == []


def test_operator_backward_returns_the_feature_gradients():
    # the intermediate handed out with feature_grads is what phi_backward consumes: pushing it
    # through the maps reproduces dQ and dK, and at the feature level it is dQ, dK themselves
    rng = np.random.default_rng(61)
    B, H, N, d, F, dp = 1, 2, 6, 4, 2, 3
    Q, K, V, dO = (rng.standard_normal((B, H, N, d)) for _ in range(4))
    phi = [orc.PhiWeights(rng.standard_normal((d, d)), 0.3 * rng.standard_normal(d),
                          rng.standard_normal((d, dp)), rng.standard_normal(dp) + 1.0)
           for _ in range(1 + F)]
    dQ, dK, dV, (dqf, dkf) = orc.hla_operator_backward(Q, K, V, dO, F, dp, 1e-4, phi=phi,
                                                       feature_grads=True)
    assert dqf.shape == (B, H, N, dp) and dkf.shape == (B, H, N, F * dp)
    for h in range(H):
        np.testing.assert_allclose(orc.phi_backward(dqf[0, h], Q[0, h], *phi[0].astuple()), dQ[0, h],
                                   rtol=1e-12, atol=1e-14)
        acc = sum(orc.phi_backward(dkf[0, h][:, f * dp:(f + 1) * dp], K[0, h], *phi[1 + f].astuple())
                  for f in range(F))
        np.testing.assert_allclose(acc, dK[0, h], rtol=1e-12, atol=1e-14)
    Qf, Kf = np.abs(rng.standard_normal((B, H, N, dp))), np.abs(rng.standard_normal((B, H, N, F * dp)))
    dQ2, dK2, _, (dqf2, dkf2) = orc.hla_operator_backward(Qf, Kf, V, dO, F, dp, 1e-4, feature_grads=True)
    np.testing.assert_array_equal(dQ2, dqf2)
    np.testing.assert_array_equal(dK2, dkf2)

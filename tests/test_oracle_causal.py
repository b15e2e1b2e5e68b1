"""Pins for the oracle's causal variant (Sec. 4.4): the masked N x N matrix against the
sequential state updates the paper gives, against scalar loops, the rows whose value is known
(first row, last row), causality itself, and F = 1 against causal linear attention by prefix sums."""
import numpy as np
import pytest

from oracle import hla_oracle as orc


def _inputs(seed, n, dp, d, F):
    rng = np.random.default_rng(seed)
    q = np.abs(rng.standard_normal((n, dp))) + 0.05
    ks = [np.abs(rng.standard_normal((n, dp))) + 0.05 for _ in range(F)]
    return q, ks, rng.standard_normal((n, d))


@pytest.mark.parametrize("F,dp", [(1, 5), (2, 4), (3, 3), (3, 6), (2, 12)])
def test_masked_matrix_equals_sequential_updates(F, dp):
    q, ks, v = _inputs(80 + F, 23, dp, 5, F)
    a = orc.hla_causal_bruteforce(q, ks, v, 1e-6)
    b = orc.hla_causal_sequential(q, ks, v, 1e-6)
    np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-13)


def test_masked_matrix_against_scalar_loops():
    q, ks, v = _inputs(85, 9, 3, 4, 3)
    eps = 1e-3
    got = orc.hla_causal_bruteforce(q, ks, v, eps)
    for i in range(9):
        num = np.zeros(4)
        eta = 0.0
        for j in range(i + 1):          # keys up to and including the query's own position
            a = 1.0
            for f in range(3):
                a *= sum(q[i, c] * ks[f][j, c] for c in range(3))
            eta += a
            num += a * v[j]
        np.testing.assert_allclose(got[i], num / (eta + eps), rtol=1e-12, atol=1e-14)


def test_known_rows_and_causality():
    q, ks, v = _inputs(86, 40, 6, 7, 3)
    eps = 1e-6
    c = orc.hla_causal_bruteforce(q, ks, v, eps)
    full = orc.hla_bruteforce(q, ks, v, eps)[0]
    # the last token sees every key: its row is the non-causal one; the first sees only itself
    np.testing.assert_allclose(c[-1], full[-1], rtol=1e-12, atol=1e-14)
    a00 = np.prod([q[0] @ k[0] for k in ks])
    np.testing.assert_allclose(c[0], v[0] * a00 / (a00 + eps), rtol=1e-12, atol=1e-14)
    assert np.abs(c[5] - full[5]).max() > 1e-3          # the mask matters elsewhere
    # causality: changing tokens after position 17 (keys, values, queries) leaves rows 0..17 alone
    q2, ks2, v2 = q.copy(), [k.copy() for k in ks], v.copy()
    q2[18:] += 0.3
    v2[18:] -= 1.0
    for k in ks2:
        k[18:] *= 1.7
    c2 = orc.hla_causal_bruteforce(q2, ks2, v2, eps)
    np.testing.assert_array_equal(c[:18], c2[:18])
    assert np.abs(c[18:] - c2[18:]).max() > 1e-3
    # a subset of rows is evaluated exactly as in the full call
    np.testing.assert_array_equal(orc.hla_causal_bruteforce(q, ks, v, eps, rows=[3, 39, 11]), c[[3, 39, 11]])


def test_one_factor_is_causal_linear_attention_by_prefix_sums():
    q, ks, v = _inputs(87, 30, 5, 4, 1)
    kv = np.cumsum(ks[0][:, :, None] * v[:, None, :], axis=0)   # running sum of phi(k_j) (x) v_j
    kz = np.cumsum(ks[0], axis=0)
    want = np.einsum("na,nad->nd", q, kv) / (np.einsum("na,na->n", q, kz) + 1e-6)[:, None]
    np.testing.assert_allclose(orc.hla_causal_bruteforce(q, ks, v, 1e-6), want, rtol=1e-11, atol=1e-13)


def test_operator_level_causal_is_per_sequence():
    rng = np.random.default_rng(88)
    B, H, N, d, F, dp = 1, 2, 12, 4, 2, 3
    Q = np.abs(rng.standard_normal((B, H, N, dp)))
    K = np.abs(rng.standard_normal((B, H, N, F * dp)))
    V = rng.standard_normal((B, H, N, d))
    cu = [0, 5, 12]
    a = orc.hla_operator_forward(Q, K, V, F, dp, 1e-6, cu_seqlens=cu, causal=True, route="bruteforce")
    b = orc.hla_operator_forward(Q, K, V, F, dp, 1e-6, cu_seqlens=cu, causal=True, route="factorized")
    np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-13)
    # the first token of the second sequence sees only itself, not the first sequence
    for h in range(H):
        kf = [K[0, h, 5, f * dp:(f + 1) * dp] for f in range(F)]
        a55 = np.prod([Q[0, h, 5] @ k for k in kf])
        np.testing.assert_allclose(a[0, h, 5], V[0, h, 5] * a55 / (a55 + 1e-6), rtol=1e-12)


# ---- decay factors (Sec. 4.4; reading: mask entries lambda^(i-j)) --------------------------------
@pytest.mark.parametrize("F,dp,lam", [(1, 5, 0.9), (2, 4, 0.5), (3, 3, 0.97), (3, 6, 0.8)])
def test_decayed_mask_equals_decayed_state_updates(F, dp, lam):
    q, ks, v = _inputs(90 + F, 21, dp, 5, F)
    a = orc.hla_causal_bruteforce(q, ks, v, 1e-6, decay=lam)
    b = orc.hla_causal_sequential(q, ks, v, 1e-6, decay=lam)
    np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-13)
    # a subset of rows against all their keys is the same rows of the full result
    rows = [0, 7, 20]
    np.testing.assert_array_equal(orc.hla_causal_bruteforce(q, ks, v, 1e-6, rows=rows, decay=lam), a[rows])


def test_decayed_mask_against_scalar_loops_and_limits():
    q, ks, v = _inputs(95, 8, 3, 4, 2)
    eps, lam = 1e-3, 0.7
    got = orc.hla_causal_bruteforce(q, ks, v, eps, decay=lam)
    for i in range(8):
        num, eta = np.zeros(4), 0.0
        for j in range(i + 1):
            a = 1.0
            for f in range(2):
                a *= sum(q[i, c] * ks[f][j, c] for c in range(3))
            a *= lam ** (i - j)          # the token's own position keeps weight 1
            eta += a
            num += a * v[j]
        np.testing.assert_allclose(got[i], num / (eta + eps), rtol=1e-12, atol=1e-14)
    # decay 1 is the plain causal mask (bit for bit); decay -> 0 leaves every token with itself
    np.testing.assert_array_equal(orc.hla_causal_bruteforce(q, ks, v, eps, decay=1.0),
                                  orc.hla_causal_bruteforce(q, ks, v, eps))
    np.testing.assert_array_equal(orc.hla_causal_sequential(q, ks, v, eps, decay=1.0),
                                  orc.hla_causal_sequential(q, ks, v, eps))
    np.testing.assert_allclose(orc.hla_causal_bruteforce(q, ks, v, 0.0, decay=1e-200), v, rtol=1e-12)


def test_identical_keys_give_the_geometrically_weighted_mean():
    """With every key token equal, A_ij is the same for all j, so (eps = 0) o_i is the mean of
    v_0..v_i with weights lambda^(i-j): a closed form that involves no feature arithmetic."""
    rng = np.random.default_rng(96)
    n, dp, d, lam = 12, 4, 3, 0.6
    q = np.abs(rng.standard_normal((n, dp))) + 0.1
    k1 = np.tile(np.abs(rng.standard_normal((1, dp))) + 0.1, (n, 1))
    k2 = np.tile(np.abs(rng.standard_normal((1, dp))) + 0.1, (n, 1))
    v = rng.standard_normal((n, d))
    for fn in (orc.hla_causal_bruteforce, orc.hla_causal_sequential):
        got = fn(q, [k1, k2], v, 0.0, decay=lam)
        for i in range(n):
            w = lam ** np.arange(i, -1, -1)
            np.testing.assert_allclose(got[i], np.average(v[:i + 1], axis=0, weights=w), rtol=1e-11, atol=1e-13)


def test_operator_level_decay_restarts_with_every_sequence():
    rng = np.random.default_rng(97)
    H, d, F, dp, lam = 2, 4, 2, 3, 0.85
    cu = [0, 5, 5, 12]
    Q = np.abs(rng.standard_normal((1, H, 12, dp)))
    K = np.abs(rng.standard_normal((1, H, 12, F * dp)))
    V = rng.standard_normal((1, H, 12, d))
    for route in ("factorized", "bruteforce"):
        O = orc.hla_operator_forward(Q, K, V, F, dp, 1e-6, cu_seqlens=cu, causal=True, decay=lam, route=route)
        for (lo, hi) in ((0, 5), (5, 12)):
            for h in range(H):
                ref = orc.hla_causal_bruteforce(Q[0, h, lo:hi], [K[0, h, lo:hi, f * dp:(f + 1) * dp] for f in range(F)],
                                                V[0, h, lo:hi], 1e-6, decay=lam)
                np.testing.assert_allclose(O[0, h, lo:hi], ref, rtol=1e-11, atol=1e-13)


# ---- backward of the causal variant -------------------------------------------------------------
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


@pytest.mark.parametrize("F,dp,lam", [(2, 3, 1.0), (3, 3, 0.8), (3, 2, 1.0), (1, 4, 0.6)])
def test_causal_backward_routes_against_finite_differences(F, dp, lam):
    """Both routes against central differences of the forward (masked matrix), and against each
    other; the forward they differentiate is pinned above."""
    q, ks, v = _inputs(100 + F, 9, dp, 4, F)
    do = np.random.default_rng(101).standard_normal(v.shape)
    eps = 1e-3
    f = lambda: float((orc.hla_causal_bruteforce(q, ks, v, eps, decay=lam) * do).sum())
    a = orc.hla_causal_backward_bruteforce(q, ks, v, do, eps, decay=lam)
    b = orc.hla_causal_backward_sequential(q, ks, v, do, eps, decay=lam)
    np.testing.assert_allclose(a[0], _fd(f, q), rtol=2e-6, atol=1e-8)
    np.testing.assert_allclose(a[2], _fd(f, v), rtol=2e-6, atol=1e-8)
    for fk in range(F):
        np.testing.assert_allclose(a[1][fk], _fd(f, ks[fk]), rtol=2e-6, atol=1e-8)
        np.testing.assert_allclose(a[1][fk], b[1][fk], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(a[0], b[0], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(a[2], b[2], rtol=1e-10, atol=1e-12)


def test_causal_backward_known_rows():
    """The last token is seen by itself only: its key-side gradients come from query N-1 alone;
    the first query sees itself only, so dq_0 depends on token 0 alone (eps = 0: o_0 = v_0 exactly
    and every gradient through row 0 vanishes)."""
    q, ks, v = _inputs(105, 7, 3, 4, 2)
    do = np.random.default_rng(106).standard_normal(v.shape)
    dq, dks, dv = orc.hla_causal_backward_bruteforce(q, ks, v, do, 0.0, decay=0.9)
    np.testing.assert_allclose(dq[0], 0.0, atol=1e-12)
    # dv of the last token: A_{N-1,N-1} / eta_{N-1} * dO_{N-1}
    a_last = np.prod([q[-1] @ k[-1] for k in ks])
    eta_last = sum(0.9 ** (6 - j) * np.prod([q[-1] @ k[j] for k in ks]) for j in range(7))
    np.testing.assert_allclose(dv[-1], a_last / eta_last * do[-1], rtol=1e-12)


def test_operator_level_causal_backward_with_maps_and_packing():
    rng = np.random.default_rng(107)
    H, N, d, F, dp = 2, 8, 4, 2, 3
    cu = [0, 3, 8]
    Q, K, V, dO = (rng.standard_normal((1, H, N, d)) for _ in range(4))
    phi = [orc.PhiWeights(rng.standard_normal((d, d)), 0.3 * rng.standard_normal(d),
                          rng.standard_normal((d, dp)), rng.standard_normal(dp) + 1.5)
           for _ in range(1 + F)]
    eps, lam = 1e-4, 0.85
    f = lambda: float((orc.hla_operator_forward(Q, K, V, F, dp, eps, phi=phi, cu_seqlens=cu, route="bruteforce",
                                                causal=True, decay=lam) * dO).sum())
    for route in ("factorized", "bruteforce"):
        dQ, dK, dV = orc.hla_operator_backward(Q, K, V, dO, F, dp, eps, phi=phi, cu_seqlens=cu, route=route,
                                               causal=True, decay=lam)
        np.testing.assert_allclose(dQ, _fd(f, Q), rtol=5e-6, atol=5e-8)
        np.testing.assert_allclose(dK, _fd(f, K), rtol=5e-6, atol=5e-8)
        np.testing.assert_allclose(dV, _fd(f, V), rtol=5e-6, atol=5e-8)


def test_operator_level_causal_backward_with_value_modulation():
    """Causal variant followed by the value modulation (Secs. 4.4 and 4.5 composed): input and
    modulation-weight gradients of both routes against central differences of the forward, and
    the modulated causal output itself against the modulation applied by hand to the causal T."""
    import math
    rng = np.random.default_rng(108)
    H, N, d, F, dp = 2, 7, 4, 2, 3
    cu = [0, 3, 7]
    Q, K, V, dO = (rng.standard_normal((1, H, N, d)) for _ in range(4))
    phi = [orc.PhiWeights(rng.standard_normal((d, d)), 0.3 * rng.standard_normal(d),
                          rng.standard_normal((d, dp)), rng.standard_normal(dp) + 1.5)
           for _ in range(1 + F)]
    pv = lambda scale: orc.PhiVWeights(scale * rng.standard_normal((d, d)), 0.3 * rng.standard_normal(d),
                                       rng.standard_normal((d, d)) / math.sqrt(d), 0.3 * rng.standard_normal(d),
                                       1.0 + 0.2 * rng.standard_normal(d), 0.2 * rng.standard_normal(d))
    vmod = (pv(3.0), pv(1.0), 1e-5)
    eps, lam = 1e-4, 0.9
    fwd = lambda route: orc.hla_operator_forward(Q, K, V, F, dp, eps, phi=phi, cu_seqlens=cu, route=route,
                                                 causal=True, decay=lam, vmod=vmod)
    f = lambda: float((fwd("bruteforce") * dO).sum())
    T = orc.hla_operator_forward(Q, K, V, F, dp, eps, phi=phi, cu_seqlens=cu, route="bruteforce",
                                 causal=True, decay=lam)
    for h in range(H):
        want = orc.value_modulation_forward(T[0, h], V[0, h], *vmod)
        np.testing.assert_allclose(fwd("factorized")[0, h], want, rtol=1e-10, atol=1e-12)
    assert np.abs(fwd("bruteforce") - T).max() > 1e-3
    for route in ("factorized", "bruteforce"):
        dQ, dK, dV, vwg = orc.hla_operator_backward(Q, K, V, dO, F, dp, eps, phi=phi, cu_seqlens=cu, route=route,
                                                    causal=True, decay=lam, vmod=vmod, vmod_weight_grads=True)
        np.testing.assert_allclose(dQ, _fd(f, Q), rtol=5e-6, atol=5e-8)
        np.testing.assert_allclose(dK, _fd(f, K), rtol=5e-6, atol=5e-8)
        np.testing.assert_allclose(dV, _fd(f, V), rtol=5e-6, atol=5e-8)
        for m, grads in zip(vmod[:2], vwg):
            for arr, ga in zip(m.astuple(), grads):
                np.testing.assert_allclose(ga, _fd(f, arr), rtol=1e-5, atol=1e-7)

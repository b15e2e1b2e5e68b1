"""Pins for the CPU oracle's forward routes: each test fixes the oracle to something other than
itself (the plain definition, a closed form, a textbook special case, an invariant the paper
states), chosen so that a dropped term, a wrong index order or a transposed operand fails."""
import itertools
import math

import numpy as np
import pytest

from oracle import hla_oracle as orc


def _rand_feats(rng, n, dp, F, positive=True):
    q = rng.standard_normal((n, dp))
    ks = [rng.standard_normal((n, dp)) for _ in range(F)]
    if positive:
        q = np.abs(q)
        ks = [np.abs(k) for k in ks]
    return q, ks


# ---- Lemma 4.1 -------------------------------------------------------------------------------
@pytest.mark.parametrize("F", [2, 3, 4])
def test_lemma_product_of_dots_is_full_contraction(F):
    rng = np.random.default_rng(F)
    dp = 5
    q = rng.standard_normal(dp)
    rs = [rng.standard_normal(dp) for _ in range(F)]
    lhs = np.prod([q @ r for r in rs])
    # right-hand side written out with explicit index loops, not with the oracle's helper
    rhs = 0.0
    for idx in itertools.product(range(dp), repeat=F):
        rhs += np.prod([q[i] for i in idx]) * np.prod([rs[f][idx[f]] for f in range(F)])
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))
    # and the helper's flattening order matches those loops (first slot slowest)
    t = orc.outer_features([r[None, :] for r in rs])[0]
    tq = orc.outer_features([q[None, :]] * F)[0]
    assert t.shape == (dp ** F,)
    assert abs(float(tq @ t) - lhs) <= 1e-12 * max(1.0, abs(lhs))
    idx = tuple(range(F))  # element (0,1,2,...) sits at the row-major flat index
    flat = 0
    for i in idx:
        flat = flat * dp + (i % dp)
    assert abs(t[flat] - np.prod([rs[f][idx[f] % dp] for f in range(F)])) < 1e-14


# ---- factorized == brute force (Theorem 4.2) ---------------------------------------------------
@pytest.mark.parametrize("F,dp,d,n", [(1, 7, 5, 33), (2, 12, 8, 50), (3, 6, 8, 64), (3, 4, 3, 17),
                                      (4, 3, 4, 20)])
def test_factorized_equals_bruteforce(F, dp, d, n):
    rng = np.random.default_rng(100 + F)
    q, ks = _rand_feats(rng, n, dp, F)
    v = rng.standard_normal((n, d))
    o_bf, A, eta_bf = orc.hla_bruteforce(q, ks, v, 1e-6)
    o_fa, C, z, eta_fa = orc.hla_factorized(q, ks, v, 1e-6)
    assert C.shape == (dp ** F, d) and z.shape == (dp ** F,)
    np.testing.assert_allclose(eta_fa, eta_bf, rtol=1e-12)
    np.testing.assert_allclose(o_fa, o_bf, rtol=1e-11, atol=1e-13)


def test_factorized_equals_bruteforce_signed_features_distinct_key_maps():
    # Without the >=0 constraint and with eps=0 the algebraic identity still holds; signed,
    # clearly different key maps catch a swapped or reused key factor.
    rng = np.random.default_rng(7)
    q, ks = _rand_feats(rng, 40, 6, 3, positive=False)
    ks[1] = ks[1] * 3.0 + 1.0
    ks[2] = ks[2] ** 2
    v = rng.standard_normal((40, 4))
    A = (q @ ks[0].T) * (q @ ks[1].T) * (q @ ks[2].T)
    num_ref = A @ v
    Tq = orc.outer_features([q, q, q])
    C, z = orc.hla_state(ks, v)
    np.testing.assert_allclose(Tq @ C, num_ref, rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(Tq @ z, A.sum(1), rtol=1e-10, atol=1e-10)


def test_bruteforce_matches_scalar_loops():
    # the N x N route itself, against triple-nested scalar loops of Eq. (hla)
    rng = np.random.default_rng(3)
    n, dp, d, F = 6, 3, 2, 3
    q, ks = _rand_feats(rng, n, dp, F)
    v = rng.standard_normal((n, d))
    eps = 1e-3
    o, _, _ = orc.hla_bruteforce(q, ks, v, eps)
    for i in range(n):
        num = np.zeros(d)
        eta = 0.0
        for j in range(n):
            a = 1.0
            for f in range(F):
                a *= sum(q[i, c] * ks[f][j, c] for c in range(dp))
            eta += a
            num += a * v[j]
        np.testing.assert_allclose(o[i], num / (eta + eps), rtol=1e-13)


# ---- special cases with closed forms ------------------------------------------------------------
def test_F1_is_textbook_linear_attention():
    # Eq. (lin.att): phi(Q) (phi(K)^T V), normalised by phi(Q) sum_j phi(k_j)
    rng = np.random.default_rng(11)
    n, dp, d = 45, 9, 6
    q, ks = _rand_feats(rng, n, dp, 1)
    v = rng.standard_normal((n, d))
    ctx = ks[0].T @ v
    ref = (q @ ctx) / (q @ ks[0].sum(0))[:, None]
    o = orc.hla_factorized(q, ks, v, 0.0)[0]
    np.testing.assert_allclose(o, ref, rtol=1e-12)


def test_dphi1_output_is_query_independent_weighted_mean():
    rng = np.random.default_rng(12)
    n, d, F = 30, 5, 3
    q, ks = _rand_feats(rng, n, 1, F)
    q += 0.1
    v = rng.standard_normal((n, d))
    w = np.prod([k[:, 0] for k in ks], axis=0)
    ref = (w[:, None] * v).sum(0) / w.sum()
    for route in (orc.hla_factorized, orc.hla_bruteforce):
        o = route(q, ks, v, 0.0)[0]
        np.testing.assert_allclose(o, np.broadcast_to(ref, o.shape), rtol=1e-12)


def test_identical_keys_give_plain_mean_of_values():
    rng = np.random.default_rng(13)
    n, dp, d, F = 25, 6, 4, 3
    q, _ = _rand_feats(rng, n, dp, F)
    ks = [np.tile(np.abs(rng.standard_normal((1, dp))) + 0.1, (n, 1)) for _ in range(F)]
    v = rng.standard_normal((n, d))
    o = orc.hla_factorized(q + 0.1, ks, v, 0.0)[0]
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(0), o.shape), rtol=1e-12)


def test_one_hot_features_select_matching_tokens_exactly():
    # q_i = e_{c(i)}, k_f,j = e_{c_f(j)}: A_ij in {0,1}; o_i = mean of v over tokens whose F
    # key classes all equal c(i).  Integer-valued v keeps everything exact.
    rng = np.random.default_rng(14)
    n, dp, d, F = 60, 4, 3, 3
    cq = rng.integers(0, dp, n)
    cks = [rng.integers(0, 2, n) for _ in range(F)]  # 2 classes so matches are common
    eye = np.eye(dp)
    q = eye[cq]
    ks = [eye[c] for c in cks]
    v = rng.integers(-5, 6, (n, d)).astype(float)
    o = orc.hla_factorized(q, ks, v, 0.0 + 1e-300)[0]
    for i in range(n):
        sel = np.ones(n, bool)
        for c in cks:
            sel &= (c == cq[i])
        if sel.any():
            np.testing.assert_allclose(o[i], v[sel].mean(0), rtol=1e-14, atol=1e-14)
        else:
            assert np.all(o[i] == 0.0)  # eta = 0: 0/(0+eps) = 0


def test_single_token():
    rng = np.random.default_rng(15)
    q, ks = _rand_feats(rng, 1, 6, 3)
    v = rng.standard_normal((1, 8))
    eps = 0.5
    eta = np.prod([q[0] @ k[0] for k in ks])
    o = orc.hla_factorized(q, ks, v, eps)[0]
    np.testing.assert_allclose(o[0], v[0] * eta / (eta + eps), rtol=1e-13)


# ---- invariants the paper states -----------------------------------------------------------------
def test_rows_are_normalised_and_convex():
    rng = np.random.default_rng(16)
    n, dp, d, F = 70, 6, 5, 3
    q, ks = _rand_feats(rng, n, dp, F)
    eps = 1e-6
    ones = np.ones((n, d))
    o, _, _, eta = orc.hla_factorized(q, ks, ones, eps)
    np.testing.assert_allclose(o, np.broadcast_to((eta / (eta + eps))[:, None], o.shape),
                               rtol=1e-13)
    assert np.all(np.abs(o - 1.0) < 1e-5)
    v = rng.standard_normal((n, d))
    o = orc.hla_factorized(q, ks, v, eps)[0]
    assert np.all(o <= v.max(0) + 1e-12) and np.all(o >= v.min(0) - 1e-12)
    # explicit attention matrix: rows sum to one
    _, A, eta_bf = orc.hla_bruteforce(q, ks, v, 0.0)
    np.testing.assert_allclose((A / eta_bf[:, None]).sum(1), 1.0, rtol=1e-13)


def test_permutation_invariance_non_causal():
    rng = np.random.default_rng(17)
    n, dp, d, F = 40, 6, 4, 3
    q, ks = _rand_feats(rng, n, dp, F)
    v = rng.standard_normal((n, d))
    o = orc.hla_factorized(q, ks, v, 1e-6)[0]
    pk = rng.permutation(n)
    o_k = orc.hla_factorized(q, [k[pk] for k in ks], v[pk], 1e-6)[0]
    np.testing.assert_allclose(o_k, o, rtol=1e-11, atol=1e-13)
    pq = rng.permutation(n)
    o_q = orc.hla_factorized(q[pq], ks, v, 1e-6)[0]
    np.testing.assert_allclose(o_q, o[pq], rtol=1e-12, atol=1e-14)


def test_rational_function_homogeneity():
    # eps = 0: numerator and denominator are both homogeneous of degree F in the query features
    # and of degree 1 in each key map, so the output ignores positive rescaling of either; the
    # output is linear in V.
    rng = np.random.default_rng(18)
    n, dp, d, F = 30, 6, 4, 3
    q, ks = _rand_feats(rng, n, dp, F)
    v = rng.standard_normal((n, d))
    o, C, z, eta = orc.hla_factorized(q, ks, v, 0.0)
    o2, C2, z2, eta2 = orc.hla_factorized(2.5 * q, ks, v, 0.0)
    np.testing.assert_allclose(o2, o, rtol=1e-12)
    np.testing.assert_allclose(eta2, eta * 2.5 ** F, rtol=1e-12)
    ks3 = [ks[0], 0.3 * ks[1], ks[2]]
    o3, C3, z3, _ = orc.hla_factorized(q, ks3, v, 0.0)
    np.testing.assert_allclose(o3, o, rtol=1e-12)
    np.testing.assert_allclose(C3, 0.3 * C, rtol=1e-12)
    v2 = rng.standard_normal((n, d))
    o_lin = orc.hla_factorized(q, ks, 2.0 * v - 3.0 * v2, 0.0)[0]
    np.testing.assert_allclose(o_lin, 2.0 * o - 3.0 * orc.hla_factorized(q, ks, v2, 0.0)[0],
                               rtol=1e-10, atol=1e-12)


def test_sequential_state_update_reaches_batch_state():
    rng = np.random.default_rng(19)
    n, dp, d, F = 23, 4, 5, 3
    _, ks = _rand_feats(rng, n, dp, F)
    v = rng.standard_normal((n, d))
    C, z = orc.hla_state(ks, v)
    Cs, zs = orc.hla_sequential_state(ks, v)
    np.testing.assert_allclose(Cs, C, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(zs, z, rtol=1e-12)


def test_rank_bound_and_rank_above_dphi():
    rng = np.random.default_rng(20)
    n, dp, F = 60, 3, 2
    q, ks = _rand_feats(rng, n, dp, F, positive=False)
    _, A, _ = orc.hla_bruteforce(q, ks, np.zeros((n, 1)), 0.0)
    r = np.linalg.matrix_rank(A, tol=1e-9)
    assert dp < r <= dp ** F  # Hadamard product lifts the rank above d_phi, bounded by the product


# ---- feature maps ----------------------------------------------------------------------------------
def test_gelu_against_tabulated_normal_cdf():
    # Phi(1) = 0.8413447461, Phi(2) = 0.9772498681, Phi(0.5) = 0.6914624613 (standard tables)
    np.testing.assert_allclose(orc.gelu_erf(np.array([1.0, 2.0, 0.5, 0.0])),
                               [0.8413447461, 2 * 0.9772498681, 0.5 * 0.6914624613, 0.0],
                               rtol=0, atol=2e-10)
    x = np.linspace(-6, 6, 101)
    np.testing.assert_allclose(orc.gelu_erf(x) - orc.gelu_erf(-x), x, atol=1e-14)  # x(Phi(x)+Phi(-x))
    h = 1e-6
    fd = (orc.gelu_erf(x + h) - orc.gelu_erf(x - h)) / (2 * h)
    np.testing.assert_allclose(orc.gelu_erf_grad(x), fd, atol=1e-8)
    # pdf(1) = 0.2419707245: GELU'(1) = Phi(1) + pdf(1)
    assert abs(orc.gelu_erf_grad(np.array([1.0]))[0] - (0.8413447461 + 0.2419707245)) < 2e-10


def test_phi_forward_matches_scalar_loops():
    rng = np.random.default_rng(21)
    n, d, dp = 4, 5, 3
    x = rng.standard_normal((n, d))
    W1, b1 = rng.standard_normal((d, d)), rng.standard_normal(d)
    W2, b2 = rng.standard_normal((d, dp)), rng.standard_normal(dp)
    feat, h, u = orc.phi_forward(x, W1, b1, W2, b2)
    for i in range(n):
        hh = [b1[j] + sum(x[i, k] * W1[k, j] for k in range(d)) for j in range(d)]
        gg = [t * 0.5 * (1 + math.erf(t / math.sqrt(2))) for t in hh]
        for c in range(dp):
            uu = b2[c] + sum(gg[j] * W2[j, c] for j in range(d))
            assert abs(feat[i, c] - max(uu, 0.0)) < 1e-13
    assert (feat >= 0).all() and (feat == 0).any() and (feat > 0).any()


# ---- whole operator: layout, packing, routes --------------------------------------------------------
def test_operator_packed_sequences_do_not_leak():
    rng = np.random.default_rng(22)
    H, d, F, dp = 2, 4, 3, 3
    cu = [0, 5, 5, 16, 30]  # includes an empty sequence
    N = cu[-1]
    Q = np.abs(rng.standard_normal((1, H, N, dp)))
    K = np.abs(rng.standard_normal((1, H, N, F * dp)))
    V = rng.standard_normal((1, H, N, d))
    O = orc.hla_operator_forward(Q, K, V, F, dp, 1e-6, cu_seqlens=cu)
    for s in range(len(cu) - 1):
        lo, hi = cu[s], cu[s + 1]
        if hi == lo:
            continue
        Os = orc.hla_operator_forward(Q[:, :, lo:hi], K[:, :, lo:hi], V[:, :, lo:hi], F, dp, 1e-6)
        np.testing.assert_array_equal(O[:, :, lo:hi], Os)
    K2, V2 = K.copy(), V.copy()
    K2[:, :, :5] += 1.0
    V2[:, :, :5] -= 2.0
    O2 = orc.hla_operator_forward(Q, K2, V2, F, dp, 1e-6, cu_seqlens=cu)
    np.testing.assert_array_equal(O2[:, :, 5:], O[:, :, 5:])
    assert not np.allclose(O2[:, :, :5], O[:, :, :5])


def test_operator_routes_agree_with_feature_maps():
    rng = np.random.default_rng(23)
    B, H, N, d, F, dp = 2, 2, 20, 6, 3, 4
    Q, K, V = (rng.standard_normal((B, H, N, d)) for _ in range(3))
    phi = [orc.PhiWeights(rng.standard_normal((d, d)), rng.standard_normal(d),
                          rng.standard_normal((d, dp)), rng.standard_normal(dp) + 1.0)
           for _ in range(1 + F)]
    Oa = orc.hla_operator_forward(Q, K, V, F, dp, 1e-6, phi=phi, route="factorized")
    Ob = orc.hla_operator_forward(Q, K, V, F, dp, 1e-6, phi=phi, route="bruteforce")
    np.testing.assert_allclose(Oa, Ob, rtol=1e-10, atol=1e-13)
    # key map f feeds slot f: swapping two key maps' weights must give the same output (the
    # query tensor is symmetric), while replacing one by another must not.
    phi_sw = [phi[0], phi[2], phi[1], phi[3]]
    np.testing.assert_allclose(orc.hla_operator_forward(Q, K, V, F, dp, 1e-6, phi=phi_sw), Oa,
                               rtol=1e-10, atol=1e-13)
    phi_dup = [phi[0], phi[1], phi[1], phi[3]]
    assert not np.allclose(orc.hla_operator_forward(Q, K, V, F, dp, 1e-6, phi=phi_dup), Oa)

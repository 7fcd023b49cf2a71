"""Pins for the oracle's routing: invariants of the softmax-of-cosines rule and of Eq. 6, brute force.  CPU only."""
import math

import numpy as np

from oracle import seka_oracle as orc


def _setup(rng, B=3, T=10, Hq=6, H=2, d=8, M=4):
    Q = rng.standard_normal((B, T, Hq, d))
    proto = rng.standard_normal((H, M, d))
    proto /= np.linalg.norm(proto, axis=-1, keepdims=True)
    return Q, proto


def test_softmax_cos_invariants():
    rng = np.random.default_rng(20)
    Q, proto = _setup(rng)
    w = orc.route_softmax_cos(Q, proto, 0, Q.shape[1], 10.0)
    assert w.shape == (3, 2, 4)
    np.testing.assert_allclose(w.sum(-1), 1.0, atol=1e-14)
    assert (w > 0).all()
    # invariant to positive rescaling of the queries and of the prototypes
    np.testing.assert_allclose(orc.route_softmax_cos(3.7 * Q, proto, 0, Q.shape[1], 10.0), w, atol=1e-13)
    np.testing.assert_allclose(orc.route_softmax_cos(Q, 0.2 * proto, 0, Q.shape[1], 10.0), w, atol=1e-13)
    # equal prototypes -> uniform
    same = np.broadcast_to(proto[:, :1], proto.shape).copy()
    np.testing.assert_allclose(orc.route_softmax_cos(Q, same, 0, Q.shape[1], 10.0), 0.25, atol=1e-14)
    # tau = 0 -> uniform; large tau -> one-hot on the best-aligned expert
    np.testing.assert_allclose(orc.route_softmax_cos(Q, proto, 0, Q.shape[1], 0.0), 0.25, atol=1e-15)
    hot = orc.route_softmax_cos(Q, proto, 0, Q.shape[1], 1e6)
    q_bar = orc.mean_group_query(Q, 2, 0, Q.shape[1])
    best = np.einsum("bhd,hmd->bhm", q_bar, proto).argmax(-1)
    assert np.array_equal(hot.argmax(-1), best) and np.allclose(hot.max(-1), 1.0)
    # all-zero queries -> cos defined as 0 -> uniform
    np.testing.assert_allclose(orc.route_softmax_cos(0 * Q, proto, 0, Q.shape[1], 10.0), 0.25, atol=1e-15)


def test_softmax_cos_brute_force_and_token_range():
    rng = np.random.default_rng(21)
    B, T, Hq, H, d, M = 2, 7, 4, 2, 3, 3
    Q, proto = _setup(rng, B, T, Hq, H, d, M)
    t0, t1, tau = 2, 6, 4.0
    w = orc.route_softmax_cos(Q, proto, t0, t1, tau)
    G = Hq // H
    for b in range(B):
        for h in range(H):
            qb = [0.0] * d
            for t in range(t0, t1):
                for hq in range(h * G, (h + 1) * G):
                    for a in range(d):
                        qb[a] += Q[b, t, hq, a] / ((t1 - t0) * G)
            qn = math.sqrt(sum(x * x for x in qb))
            z = []
            for m in range(M):
                pn = math.sqrt(sum(proto[h, m, a] ** 2 for a in range(d)))
                z.append(tau * sum(qb[a] * proto[h, m, a] for a in range(d)) / (qn * pn))
            den = sum(math.exp(x) for x in z)
            for m in range(M):
                assert abs(w[b, h, m] - math.exp(z[m]) / den) < 1e-13


def test_eq6_invariants_and_prototype_form():
    rng = np.random.default_rng(22)
    B, T, Hq, H, d, M, Ktop = 3, 9, 4, 2, 16, 4, 5
    Q = rng.standard_normal((B, T, Hq, d))
    U_top = np.stack([[np.linalg.qr(rng.standard_normal((d, Ktop)))[0] for _ in range(M)] for _ in range(H)])
    sigma = np.sort(rng.random((H, M, Ktop)) + 0.1, axis=-1)[..., ::-1]
    alpha = orc.route_eq6(Q, U_top, sigma, T - 1, T)
    # largest coefficient has magnitude exactly 1; signs are those of the raw alignments
    np.testing.assert_allclose(np.abs(alpha).max(-1), 1.0, atol=1e-15)
    q_last = orc.mean_group_query(Q, H, T - 1, T)
    # the K-term sum collapses to one dot product with p_m = sum_k sigma_k u_k
    p = np.einsum("hmdk,hmk->hmd", U_top, sigma)
    raw = np.einsum("bhd,hmd->bhm", q_last, p)
    assert np.array_equal(np.sign(alpha), np.sign(raw))
    np.testing.assert_allclose(alpha, raw / np.abs(raw).max(-1, keepdims=True), atol=1e-13)
    # scale-invariant in the query, sign-flipping under q -> -q
    np.testing.assert_allclose(orc.route_eq6(2.5 * Q, U_top, sigma, T - 1, T), alpha, atol=1e-13)
    np.testing.assert_allclose(orc.route_eq6(-Q, U_top, sigma, T - 1, T), -alpha, atol=1e-13)
    # no alignment at all -> zero coefficients (no steering)
    assert np.array_equal(orc.route_eq6(0 * Q, U_top, sigma, T - 1, T), np.zeros((B, H, M)))


def test_mean_group_query_last_token():
    rng = np.random.default_rng(23)
    Q = rng.standard_normal((2, 5, 6, 4))
    qb = orc.mean_group_query(Q, 3, 4, 5)
    for h in range(3):
        np.testing.assert_allclose(qb[:, h], Q[:, 4, 2 * h:2 * h + 2].mean(1), atol=1e-15)


def test_project_queries_pins():
    """The projection against what fixes it: identity weights return the input, a one-hot weight row picks one
    input feature, and a tiny case agrees with sums written out term by term."""
    g = np.random.default_rng(3)
    B, T, Hq, D = 2, 5, 3, 4
    E = Hq * D
    X = g.standard_normal((B, T, E))
    assert np.array_equal(orc.project_queries(X, np.eye(E), Hq), X.reshape(B, T, Hq, D))
    W = np.zeros((E, E)); W[7, 2] = 3.0                     # output feature 7 = head 1, d 3 reads input feature 2
    Q = orc.project_queries(X, W, Hq)
    assert np.array_equal(Q[:, :, 1, 3], 3.0 * X[:, :, 2]) and np.count_nonzero(Q) == B * T
    W = g.standard_normal((E, 6)); X6 = g.standard_normal((1, 2, 6))
    Q = orc.project_queries(X6, W, Hq)
    for t_ in range(2):
        for n in range(E):
            want = sum(X6[0, t_, e] * W[n, e] for e in range(6))
            assert abs(Q[0, t_, n // D, n % D] - want) < 1e-12

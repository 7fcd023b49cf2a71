"""Pins of the oracle's offline stage (paper Sec. 3.1 and 3.4).  CPU only."""
import numpy as np

from oracle import seka_oracle as orc


def _planted(seed, n=400, H=2, d=12, k=3, noise=0.02):
    """Neutral and signal embeddings that share a planted k-dimensional subspace B (plus small noise)."""
    rng = np.random.default_rng(seed)
    B = np.linalg.qr(rng.standard_normal((H, d, k)))[0]
    z = rng.standard_normal((n, H, k)) * np.array([3.0, 2.0, 1.5])[:k]
    hn = np.einsum("nhk,hdk->nhd", z, B) + noise * rng.standard_normal((n, H, d))
    hs = np.einsum("nhk,hdk->nhd", z, B) + noise * rng.standard_normal((n, H, d))
    return hn, hs, B


def test_svd_reconstructs_the_cross_covariance():
    hn, hs, _ = _planted(0)
    U, S, k = orc.learn_projection(hn, hs, 0.9)
    for h in range(hn.shape[1]):
        omega = hn[:, h].T @ hs[:, h] / hn.shape[0]
        # U diag(S) V^T = Omega  <=>  U^T Omega has rows of norm S and U is orthogonal
        assert np.abs(U[h].T @ U[h] - np.eye(U.shape[1])).max() < 1e-12
        assert np.abs(np.linalg.norm(U[h].T @ omega, axis=1) - S[h]).max() < 1e-12
        assert np.all(np.diff(S[h]) <= 1e-15)
        # singular values are the square roots of the eigenvalues of Omega Omega^T (independent routine)
        ev = np.sort(np.linalg.eigvalsh(omega @ omega.T))[::-1]
        # (squaring loses the small ones: eigenvalue error 1e-15 * 77 becomes 1e-9 at sigma = 1e-5)
        assert np.abs(np.sqrt(np.maximum(ev, 0)) - S[h]).max() < 1e-8


def test_planted_subspace_is_recovered_and_rank_rule_finds_it():
    hn, hs, B = _planted(1)
    U, S, k = orc.learn_projection(hn, hs, 0.95)
    for h in range(2):
        assert k[h] == 3, (k, S[h][:5])
        P = U[h][:, :3] @ U[h][:, :3].T
        assert np.abs(P - B[h] @ B[h].T).max() < 5e-3


def test_rank_rule_on_hand_made_spectrum():
    # diagonal "embeddings": Omega = diag(4, 3, 2, 1) / 1 -> cumulative fractions 0.4, 0.7, 0.9, 1.0
    d = 4
    hn = np.eye(d).reshape(d, 1, d) * np.sqrt(d)
    hs = hn * np.array([4.0, 3.0, 2.0, 1.0])
    for gamma, want in ((0.3, 1), (0.4, 1), (0.41, 2), (0.7, 2), (0.85, 3), (0.9, 3), (0.95, 4), (1.0, 4)):
        _, S, k = orc.learn_projection(hn, hs, gamma)
        assert np.allclose(S[0], [4, 3, 2, 1]) and k[0] == want, (gamma, k)


def test_head_distance_brute_force():
    rng = np.random.default_rng(3)
    hp, hm = rng.standard_normal((5, 2, 3)), rng.standard_normal((5, 2, 3))
    D = orc.head_relevance_distance(hp, hm)
    for h in range(2):
        want = sum(sum((hp[i, h, j] - hm[i, h, j]) ** 2 for j in range(3)) ** 0.5 for i in range(5)) / 5
        assert abs(D[h] - want) < 1e-14
    assert np.all(orc.head_relevance_distance(hp, hp) == 0)

"""Pins for the oracle's key edit: closed forms of Appendix C, projector identities (Eq. 2),
AdaSEKA blend (Sec. 3.3) and brute-force scalar loops.  CPU only."""
import os

import numpy as np
import pytest

from oracle import seka_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _orthonormal(rng, d, r):
    q, _ = np.linalg.qr(rng.standard_normal((d, r)))
    return q


def _golden_cases():
    cases = []
    with open(os.path.join(GOLD, "appendix_c_closed_form.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            dr, u, g, k, kp = [s.split() for s in line.split("|")]
            d, r = int(dr[0]), int(dr[1])
            U = np.array(u, float).reshape(r, d).T          # column-major list
            cases.append((U, float(g[0]), np.array(k, float), np.array(kp, float)))
    return cases


@pytest.mark.parametrize("case", _golden_cases())
def test_hand_worked_closed_form(case):
    U, g, k, expected = case
    d, r = U.shape
    K = k.reshape(1, 1, 1, d)
    out = orc.edit_keys(K, U.reshape(1, 1, d, r), [g], np.ones((1, 1), np.uint8))
    np.testing.assert_allclose(out[0, 0, 0], expected, atol=1e-12)


def test_projector_symmetric_idempotent():
    rng = np.random.default_rng(1)
    for d, r in [(64, 8), (128, 32), (128, 64), (16, 16)]:
        P = orc.projector(_orthonormal(rng, d, r))
        assert np.abs(P - P.T).max() < 1e-12
        assert np.abs(P @ P - P).max() < 1e-12
        assert abs(np.trace(P) - r) < 1e-10


def test_edit_matches_orthogonal_decomposition():
    """(I + g U U^T) x = x_perp + (1+g) x_par, with x_par obtained by least squares
    (an independent route to the orthogonal projection), for positive, negative and large gains."""
    rng = np.random.default_rng(2)
    B, T, H, d, r = 2, 9, 3, 32, 5
    K = rng.standard_normal((B, T, H, d))
    U = np.stack([_orthonormal(rng, d, r) for _ in range(H)])[:, None]     # [H,1,d,r]
    mask = np.ones((B, T), np.uint8)
    for g in (1.0, -1.0, 0.37, -5.0, 2.5):
        out = orc.edit_keys(K, U, [g] * H, mask)
        for h in range(H):
            k = K[:, :, h, :].reshape(-1, d)
            coef, *_ = np.linalg.lstsq(U[h, 0], k.T, rcond=None)
            k_par = (U[h, 0] @ coef).T
            k_perp = k - k_par
            np.testing.assert_allclose(out[:, :, h, :].reshape(-1, d), k_perp + (1 + g) * k_par, atol=1e-12)
            # consequences: in-subspace coordinates scale by (1+g), orthogonal part and norms as predicted
            kp = out[:, :, h, :].reshape(-1, d)
            np.testing.assert_allclose(kp @ U[h, 0], (1 + g) * (k @ U[h, 0]), atol=1e-12)
            np.testing.assert_allclose((kp ** 2).sum(1), (k_perp ** 2).sum(1) + (1 + g) ** 2 * (k_par ** 2).sum(1), rtol=1e-12)


def test_gain_minus_one_removes_subspace_component():
    rng = np.random.default_rng(3)
    d, r = 24, 6
    U = _orthonormal(rng, d, r)
    K = rng.standard_normal((1, 7, 1, d))
    out = orc.edit_keys(K, U[None, None], [-1.0], np.ones((1, 7), np.uint8))
    assert np.abs(out[0, :, 0, :] @ U).max() < 1e-12


def test_full_rank_is_uniform_scaling():
    rng = np.random.default_rng(4)
    d = 12
    U = _orthonormal(rng, d, d)
    K = rng.standard_normal((2, 5, 1, d))
    out = orc.edit_keys(K, U[None, None], [0.75], np.ones((2, 5), np.uint8))
    np.testing.assert_allclose(out, 1.75 * K, atol=1e-12)


def test_only_highlighted_rows_of_selected_heads_change():
    rng = np.random.default_rng(5)
    B, T, H, d, r = 2, 11, 3, 16, 4
    K = rng.standard_normal((B, T, H, d))
    U = np.stack([_orthonormal(rng, d, r) for _ in range(H)])[:, None]
    mask = np.zeros((B, T), np.uint8)
    mask[0, 2:5] = 1
    mask[1, 10] = 7                              # any nonzero value highlights
    out = orc.edit_keys(K, U, [1.0, 0.0, -0.5], mask)
    changed = np.any(out != K, axis=-1)          # [B,T,H]
    expect = (mask != 0)[:, :, None] & np.array([True, False, True])[None, None, :]
    assert np.array_equal(changed, expect)
    assert np.array_equal(out[~expect], K[~expect])      # bit-identical elsewhere
    # empty mask and zero gain: identity
    assert np.array_equal(orc.edit_keys(K, U, [1.0] * H, np.zeros((B, T), np.uint8)), K)
    assert np.array_equal(orc.edit_keys(K, U, [0.0] * H, np.ones((B, T), np.uint8)), K)


def test_brute_force_scalar_loops():
    """k'_a = k_a + g * sum_m w_m sum_c sum_e U_m[a,c] U_m[e,c] k_e, written as scalar loops."""
    rng = np.random.default_rng(6)
    B, T, H, M, d, r = 2, 3, 2, 3, 4, 2
    K = rng.standard_normal((B, T, H, d))
    U = rng.standard_normal((H, M, d, r))         # the edit formula itself needs no orthonormality
    w = rng.standard_normal((B, H, M))
    gain = [0.5, -1.5]
    mask = np.array([[1, 0, 1], [0, 1, 1]], np.uint8)
    out = orc.edit_keys(K, U, gain, mask, w)
    for b in range(B):
        for t in range(T):
            for h in range(H):
                for a in range(d):
                    acc = 0.0
                    if mask[b, t]:
                        for m in range(M):
                            for c in range(r):
                                z = 0.0
                                for e in range(d):
                                    z += U[h, m, e, c] * K[b, t, h, e]
                                acc += w[b, h, m] * U[h, m, a, c] * z
                    assert abs(out[b, t, h, a] - (K[b, t, h, a] + gain[h] * acc)) < 1e-12


def test_adaseka_reduces_to_seka_and_blend_is_explicit_sum():
    rng = np.random.default_rng(7)
    B, T, H, M, d, r = 2, 6, 2, 4, 16, 3
    K = rng.standard_normal((B, T, H, d))
    U = np.stack([[_orthonormal(rng, d, r) for _ in range(M)] for _ in range(H)])   # [H,M,d,r]
    mask = (rng.random((B, T)) < 0.5).astype(np.uint8)
    gain = [1.0, 0.3]
    # one-hot routing on expert 2 == SEKA with that expert alone (Appendix D: SEKA is the single-expert case)
    w = np.zeros((B, H, M))
    w[:, :, 2] = 1.0
    a = orc.edit_keys(K, U, gain, mask, w)
    b = orc.edit_keys(K, U[:, 2:3], gain, mask, None)
    np.testing.assert_allclose(a, b, atol=1e-13)
    # general blend: low-rank concatenated form U_cat diag(c) U_cat^T equals the dense sum
    w = rng.standard_normal((B, H, M))
    dense = orc.edit_keys(K, U, gain, mask, w)
    for bi in range(B):
        for h in range(H):
            Ucat = np.concatenate([U[h, m] for m in range(M)], axis=1)            # [d, M*r]
            c = np.repeat(w[bi, h], r) * gain[h]
            for t in range(T):
                k = K[bi, t, h]
                ref = k + (Ucat @ (c * (Ucat.T @ k))) if mask[bi, t] else k
                np.testing.assert_allclose(dense[bi, t, h], ref, atol=1e-12)
    # the blend is symmetric but in general not idempotent
    P = orc.blended_projector(U[0], w[0, 0])
    assert np.abs(P - P.T).max() < 1e-12
    assert np.abs(P @ P - P).max() > 1e-3

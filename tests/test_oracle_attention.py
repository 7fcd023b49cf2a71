"""Pins for the oracle's attention: hand-worked two-token case, library scaled-dot-product
attention, brute-force scalar loops, the score-side form of Eq. 5, the query-side form (Sec. 2),
and special cases with textbook answers.  CPU only."""
import math
import os

import numpy as np
import torch

from oracle import seka_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _orthonormal(rng, d, r):
    q, _ = np.linalg.qr(rng.standard_normal((d, r)))
    return q


def _problem(rng, B=2, T=13, Hq=4, H=2, d=8, r=3, M=1):
    Q = rng.standard_normal((B, T, Hq, d))
    K = rng.standard_normal((B, T, H, d))
    V = rng.standard_normal((B, T, H, d))
    U = np.stack([[_orthonormal(rng, d, r) for _ in range(M)] for _ in range(H)])
    mask = (rng.random((B, T)) < 0.4).astype(np.uint8)
    return Q, K, V, U, mask


def test_hand_worked_two_tokens():
    gold = {}
    with open(os.path.join(GOLD, "two_token_attention.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, *vals = line.split()
                gold[name] = np.array(vals, float)
    ln2 = math.log(2.0)
    K = np.array([[ln2 * math.sqrt(2.0), 7.0], [0.0, 0.0]]).reshape(1, 2, 1, 2)
    Q = np.array([[0.3, -0.2], [1.0, 0.0]]).reshape(1, 2, 1, 2)
    V = np.array([[10.0, 0.0], [0.0, 5.0]]).reshape(1, 2, 1, 2)
    U = np.array([[1.0], [0.0]]).reshape(1, 1, 2, 1)
    mask = np.array([[1, 0]], np.uint8)
    O, L = orc.steered_attention(Q, K, V, U, [1.0], mask)
    np.testing.assert_allclose(O[0, 1, 0], gold["steered_O1"], atol=1e-12)
    np.testing.assert_allclose(O[0, 0, 0], gold["O0"], atol=1e-12)
    np.testing.assert_allclose(L[0, 0, 1], gold["steered_LSE1"][0], atol=1e-12)
    O, L = orc.causal_attention(Q, K, V)
    np.testing.assert_allclose(O[0, 1, 0], gold["plain_O1"], atol=1e-12)
    np.testing.assert_allclose(L[0, 0, 1], gold["plain_LSE1"][0], atol=1e-12)


def test_plain_attention_matches_library_sdpa():
    rng = np.random.default_rng(10)
    B, T, Hq, H, d = 2, 37, 6, 2, 16
    Q, K, V, _, _ = _problem(rng, B, T, Hq, H, d)
    O, _ = orc.causal_attention(Q, K, V)
    G = Hq // H
    q = torch.from_numpy(Q).permute(0, 2, 1, 3)
    k = torch.from_numpy(K).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)    # head hq reads KV head hq // G
    v = torch.from_numpy(V).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(O, ref, atol=1e-12)
    # custom scale
    O2, _ = orc.causal_attention(Q, K, V, scale=0.3)
    ref2 = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True, scale=0.3).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(O2, ref2, atol=1e-12)


def test_brute_force_tiny():
    """Everything by scalar loops and math.exp: edit, scores, softmax, weighted sum, GQA mapping."""
    rng = np.random.default_rng(11)
    B, T, Hq, H, d, r = 2, 4, 4, 2, 3, 2
    Q, K, V, U, _ = _problem(rng, B, T, Hq, H, d, r)
    mask = np.array([[0, 1, 1, 0], [1, 0, 0, 1]], np.uint8)
    gain = [0.8, -1.3]
    O, L = orc.steered_attention(Q, K, V, U, gain, mask)
    G = Hq // H
    for b in range(B):
        for hq in range(Hq):
            h = hq // G
            kp = [[K[b, t, h, a] for a in range(d)] for t in range(T)]
            for t in range(T):
                if mask[b, t]:
                    z = [sum(U[h, 0, e, c] * K[b, t, h, e] for e in range(d)) for c in range(r)]
                    for a in range(d):
                        kp[t][a] += gain[h] * sum(U[h, 0, a, c] * z[c] for c in range(r))
            for i in range(T):
                s = [sum(Q[b, i, hq, a] * kp[j][a] for a in range(d)) / math.sqrt(d) for j in range(i + 1)]
                e = [math.exp(x) for x in s]
                den = sum(e)
                for a in range(d):
                    o = sum(e[j] * V[b, j, h, a] for j in range(i + 1)) / den
                    assert abs(O[b, i, hq, a] - o) < 1e-12
                assert abs(L[b, hq, i] - math.log(den)) < 1e-12


def test_zero_gain_or_empty_mask_is_plain_attention():
    rng = np.random.default_rng(12)
    Q, K, V, U, mask = _problem(rng)
    plain, plain_l = orc.causal_attention(Q, K, V)
    a, al = orc.steered_attention(Q, K, V, U, [0.0, 0.0], mask)
    b, bl = orc.steered_attention(Q, K, V, U, [1.0, 2.0], np.zeros_like(mask))
    assert np.array_equal(a, plain) and np.array_equal(b, plain)
    assert np.array_equal(al, plain_l) and np.array_equal(bl, plain_l)


def _attention_from_scores(scores, V_h):
    T = scores.shape[0]
    s = np.where(np.tril(np.ones((T, T), bool)), scores, -np.inf)
    e = np.exp(s - s.max(1, keepdims=True))
    return (e / e.sum(1, keepdims=True)) @ V_h


def test_score_side_form_eq5():
    """Eq. 5: logits = A + B with B_ij = g q_i.P k_j / sqrt(d) on highlighted j only; keys untouched."""
    rng = np.random.default_rng(13)
    B, T, Hq, H, d, r, M = 2, 17, 4, 2, 8, 3, 3
    Q, K, V, U, mask = _problem(rng, B, T, Hq, H, d, r, M)
    w = rng.standard_normal((B, H, M))
    gain = [1.2, -0.7]
    O, _ = orc.steered_attention(Q, K, V, U, gain, mask, w)
    G = Hq // H
    for b in range(B):
        for hq in range(Hq):
            h = hq // G
            P = sum(w[b, h, m] * U[h, m] @ U[h, m].T for m in range(M))
            A = Q[b, :, hq] @ K[b, :, h].T / math.sqrt(d)
            Bias = gain[h] * (Q[b, :, hq] @ P @ K[b, :, h].T) / math.sqrt(d) * (mask[b] != 0)[None, :]
            np.testing.assert_allclose(O[b, :, hq], _attention_from_scores(A + Bias, V[b, :, h]), atol=1e-12)


def test_query_side_form():
    """Sec. 2: the same control by editing the query instead (P symmetric): on highlighted
    columns use q' = q + g P q against the unedited key."""
    rng = np.random.default_rng(14)
    B, T, Hq, H, d, r = 1, 15, 2, 1, 8, 4
    Q, K, V, U, mask = _problem(rng, B, T, Hq, H, d, r)
    g = 0.9
    O, _ = orc.steered_attention(Q, K, V, U, [g], mask)
    P = U[0, 0] @ U[0, 0].T
    for hq in range(Hq):
        q = Q[0, :, hq]
        q_edit = q + g * q @ P.T
        plain = q @ K[0, :, 0].T
        edited = q_edit @ K[0, :, 0].T
        scores = np.where((mask[0] != 0)[None, :], edited, plain) / math.sqrt(d)
        np.testing.assert_allclose(O[0, :, hq], _attention_from_scores(scores, V[0, :, 0]), atol=1e-12)


def test_full_rank_all_highlighted_is_rescaled_plain_attention():
    rng = np.random.default_rng(15)
    B, T, Hq, H, d = 1, 12, 2, 1, 6
    Q, K, V, _, _ = _problem(rng, B, T, Hq, H, d)
    U = _orthonormal(rng, d, d)[None, None]
    g = 0.6
    O, _ = orc.steered_attention(Q, K, V, U, [g], np.ones((B, T), np.uint8))
    ref, _ = orc.causal_attention(Q, K, V, scale=(1 + g) / math.sqrt(d))
    np.testing.assert_allclose(O, ref, atol=1e-12)


def test_row_zero_and_constant_values():
    rng = np.random.default_rng(16)
    Q, K, V, U, mask = _problem(rng)
    G = Q.shape[2] // K.shape[2]
    O, _ = orc.steered_attention(Q, K, V, U, [3.0, -2.0], mask)
    for hq in range(Q.shape[2]):
        np.testing.assert_allclose(O[:, 0, hq], V[:, 0, hq // G], atol=1e-14)
    Vc = np.broadcast_to(V[:, :1], V.shape).copy()          # every token has the same value row
    O, _ = orc.steered_attention(Q, K, Vc, U, [3.0, -2.0], mask)
    for hq in range(Q.shape[2]):
        np.testing.assert_allclose(O[:, :, hq], Vc[:, :, hq // G], atol=1e-13)


def test_lse_is_log_of_denominator():
    rng = np.random.default_rng(17)
    Q, K, V, U, mask = _problem(rng, B=1, T=9, Hq=2, H=1, d=4)
    Kp = orc.edit_keys(K, U, [1.0], mask)
    _, L = orc.causal_attention(Q, Kp, V)
    for i in range(9):
        s = Q[0, i, 1] @ Kp[0, : i + 1, 0].T / 2.0
        assert abs(L[0, 1, i] - math.log(np.exp(s).sum())) < 1e-12


def test_row_sampler_agrees_with_full_attention():
    rng = np.random.default_rng(18)
    Q, K, V, U, mask = _problem(rng, B=2, T=33, Hq=4, H=2, d=8)
    Kp = orc.edit_keys(K, U, [1.0, 0.5], mask)
    O, L = orc.causal_attention(Q, Kp, V)
    rows = [(0, 0, 0), (1, 3, 32), (0, 2, 17), (1, 1, 1)]
    o, l = orc.attention_rows(Q, Kp, V, rows)
    for n, (b, hq, i) in enumerate(rows):
        np.testing.assert_allclose(o[n], O[b, i, hq], atol=1e-13)
        assert abs(l[n] - L[b, hq, i]) < 1e-13

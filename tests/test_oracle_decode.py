"""Pins of the oracle's generation-step attention.  CPU only."""
import numpy as np

from oracle import seka_oracle as orc


def _case(seed, B=2, T=13, H=2, G=3, d=8):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, T, H * G, d)), rng.standard_normal((B, T, H, d)), rng.standard_normal((B, T, H, d)))


def test_equals_last_row_of_causal_attention():
    Q, K, V = _case(0)
    O, L = orc.causal_attention(Q, K, V)
    o, l = orc.decode_attention(Q[:, -1], K, V)
    assert np.abs(o - O[:, -1]).max() < 1e-12 and np.abs(l - L[:, :, -1]).max() < 1e-12


def test_ragged_lengths_equal_the_matching_causal_rows():
    Q, K, V = _case(1)
    lens = [5, 13]
    O, L = orc.causal_attention(Q, K, V)
    q = np.stack([Q[b, lens[b] - 1] for b in range(2)])
    o, l = orc.decode_attention(q, K, V, lens)
    for b in range(2):
        assert np.abs(o[b] - O[b, lens[b] - 1]).max() < 1e-12
        assert np.abs(l[b] - L[b, :, lens[b] - 1]).max() < 1e-12


def test_brute_force_scalar_loops():
    Q, K, V = _case(2, B=1, T=4, H=1, G=2, d=3)
    q = Q[:, 2]
    o, l = orc.decode_attention(q, K, V, [3], scale=0.7)
    for hq in range(2):
        w = [np.exp(0.7 * sum(q[0, hq, i] * K[0, j, 0, i] for i in range(3))) for j in range(3)]
        for i in range(3):
            assert abs(o[0, hq, i] - sum(w[j] * V[0, j, 0, i] for j in range(3)) / sum(w)) < 1e-12
        assert abs(l[0, hq] - np.log(sum(w))) < 1e-12


def test_single_cached_token_returns_its_value():
    Q, K, V = _case(3)
    o, _ = orc.decode_attention(Q[:, 0], K, V, [1, 1])
    G = Q.shape[2] // K.shape[2]
    for hq in range(Q.shape[2]):
        assert np.abs(o[:, hq] - V[:, 0, hq // G]).max() < 1e-12


def test_edited_cache_is_what_the_new_query_sees():
    # steering persists through the cache: decode over edit_keys(K) == last row of steered attention
    rng = np.random.default_rng(4)
    Q, K, V = _case(4, d=8)
    U = np.linalg.qr(rng.standard_normal((2, 1, 8, 2)))[0]
    mask = np.zeros((2, 13), np.uint8); mask[:, 3:7] = 1
    O, _ = orc.steered_attention(Q, K, V, U, [1.5, -0.5], mask)
    o, _ = orc.decode_attention(Q[:, -1], orc.edit_keys(K, U, [1.5, -0.5], mask), V)
    assert np.abs(o - O[:, -1]).max() < 1e-12

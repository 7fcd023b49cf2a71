"""Pins of the dual-projector edit (paper Eq. 2 and Eq. 4) in the oracle.  CPU only."""
import numpy as np

from oracle import seka_oracle as orc


def _orth(rng, H, d):
    out = np.empty((H, d, d))
    for h in range(H):
        q, r = np.linalg.qr(rng.standard_normal((d, d)))
        out[h] = q * np.sign(np.diag(r))
    return out


def _case(seed=0, B=2, T=9, H=3, d=8):
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((B, T, H, d))
    Up, Un = _orth(rng, H, d), _orth(rng, H, d)
    mask = (rng.random((B, T)) < 0.5).astype(np.uint8)
    mask[0, 0] = 1
    return K, Up, Un, mask


def test_hand_worked_two_dimensional_case():
    # d = 2, U+ = U- = identity: P+ = e1 e1^T (k+ = 1), P- = e2 e2^T (k- = 1, trailing column).
    # k = (3, 5), g+ = 0.5, g- = -1  =>  k' = (3 + 0.25*3, 5 - 0.5*5) = (3.75, 2.5)   (Eq. 4)
    K = np.array([3.0, 5.0]).reshape(1, 1, 1, 2)
    I = np.eye(2).reshape(1, 2, 2)
    out = orc.edit_keys_eq4(K, I, I, [1], [1], 0.5, -1.0, np.ones((1, 1), np.uint8))
    assert np.allclose(out.ravel(), [3.75, 2.5], atol=1e-15)


def test_two_forms_of_eq4_agree():
    K, Up, Un, mask = _case()
    kp, kn = [2, 3, 1], [5, 2, 7]
    gp, gn = np.array([0.8, -0.3, 1.7]), np.array([0.4, -1.1, 0.9])
    direct = orc.edit_keys_eq4(K, Up, Un, kp, kn, gp, gn, mask)
    U, gain, w, a = orc.eq4_as_low_rank(Up, Un, kp, kn, gp, gn, K.shape[0])
    assert U.shape[3] % 8 == 0 and np.all(gain == 1.0)
    hook = orc.edit_keys(K, U, gain, mask, w=w, key_scale=a)
    assert np.abs(direct - hook).max() < 1e-12
    # unhighlighted rows are bit-identical to the input in both
    off = mask == 0
    assert np.array_equal(direct[off], K[off]) and np.array_equal(hook[off], K[off])
    # and the edit is not a no-op
    assert np.abs(direct - K).max() > 0.1


def test_negative_gain_zero_is_the_single_projector_form():
    K, Up, Un, mask = _case(1)
    kp = [3, 3, 3]
    direct = orc.edit_keys_eq4(K, Up, Un, kp, [4, 4, 4], 1.2, 0.0, mask)
    single = orc.edit_keys(K, Up[:, None, :, :3], np.full(3, 0.6), mask)      # g = g+ / 2
    assert np.abs(direct - single).max() < 1e-12


def test_trailing_block_empty_or_full():
    K, Up, Un, mask = _case(2)
    d = K.shape[-1]
    # k- = d: no trailing vectors, P- = 0
    a = orc.edit_keys_eq4(K, Up, Un, [2, 2, 2], [d, d, d], 0.0, 5.0, mask)
    assert np.abs(a - K).max() < 1e-12
    # k- = 0: P- = I, k' = (1 + g-/2) k on highlighted rows
    b = orc.edit_keys_eq4(K, Up, Un, [2, 2, 2], [0, 0, 0], 0.0, 0.5, mask)
    on = mask != 0
    assert np.abs(b[on] - 1.25 * K[on]).max() < 1e-12


def test_projector_properties_of_the_trailing_block():
    _, _, Un, _ = _case(3)
    P = Un[0][:, 3:] @ Un[0][:, 3:].T
    Q = Un[0][:, :3] @ Un[0][:, :3].T
    assert np.abs(P @ P - P).max() < 1e-12 and np.abs(P - P.T).max() < 1e-12
    assert np.abs(P + Q - np.eye(P.shape[0])).max() < 1e-12          # complement identity used by eq4_as_low_rank
    assert np.abs(P @ Q).max() < 1e-12


def test_steered_attention_accepts_key_scale():
    rng = np.random.default_rng(5)
    B, T, H, G, d = 1, 7, 2, 2, 8
    Q = rng.standard_normal((B, T, H * G, d))
    K, Up, Un, mask = _case(5, B=B, T=T, H=H, d=d)
    V = rng.standard_normal((B, T, H, d))
    U, gain, w, a = orc.eq4_as_low_rank(Up, Un, [2, 3], [4, 1], 1.0, -0.6, B)
    O1, L1 = orc.steered_attention(Q, K, V, U, gain, mask, w=w, key_scale=a)
    O2, L2 = orc.causal_attention(Q, orc.edit_keys_eq4(K, Up, Un, [2, 3], [4, 1], 1.0, -0.6, mask), V)
    assert np.abs(O1 - O2).max() < 1e-12 and np.abs(L1 - L2).max() < 1e-12

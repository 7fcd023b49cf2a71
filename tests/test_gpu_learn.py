"""GPU parity of the offline stage (seka_learn_projection, seka_head_distance; paper Sec. 3.1 and 3.4) against the
fp64 oracle.  Singular vectors are unique only up to sign, and only where their singular value is isolated, so
the comparison is on singular values, the selected rank, the projector of the leading block, isolated vectors up
to sign, and the defining properties (orthonormal columns, ||u_c^T Omega|| = sigma_c) for the rest."""
import numpy as np
import pytest

from oracle import seka_oracle as orc
from paper_2603_01281_amd import inputs
from tests import helpers as H

pytestmark = pytest.mark.gpu

# fp32 one-sided Jacobi: singular values carry an absolute error of a few ulp of sigma_1 (times sqrt(d) for the
# length-d dot products); a vector's error is that over its gap to the neighbouring singular values.
SIGMA_TOL = 2e-5          # of sigma_1
GAP = 0.02                # of sigma_1: "isolated"
# projector of the leading block (Davis-Kahan): error <= 2 |delta Omega| / gap, |delta Omega| <= SIGMA_TOL sigma_1
ORTHO_TOL = 1e-4

CASES = {
    # name: (dtype, B, S, Hkv, D, gamma, generator options)
    "f32_D128": ("f32", 2, 1024, 2, 128, 0.90, {}),
    "bf16_D128": ("bf16", 4, 1024, 4, 128, 0.85, {"rank": 16, "decay": 0.85}),
    "bf16_D64_ragged_n": ("bf16", 1, 301, 3, 64, 0.80, {"rank": 6, "decay": 0.7}),
    "f32_D64_n_below_D": ("f32", 1, 40, 2, 64, 0.90, {"rank": 5, "decay": 0.6, "noise": 0.0, "shift": 0.0}),
    "f32_single_token": ("f32", 1, 1, 2, 64, 0.50, {"rank": 3}),
    "gamma_one": ("f32", 1, 512, 1, 64, 1.0, {"rank": 8}),
}


def _widen(x, dtype):
    return (inputs.bf16_bits_to_f32(x) if dtype == "bf16" else x).astype(np.float64)


@pytest.mark.parametrize("name", list(CASES))
def test_learn_projection_matches_oracle(seka, name):
    import torch
    dtype, B, S, Hkv, D, gamma, opts = CASES[name]
    print(f"learn case {name}", flush=True)
    n = B * S
    ha, hb = inputs.paired_key_samples(n, Hkv, D, seed=5, dtype=dtype, **opts)
    ref_U, ref_S, ref_k = orc.learn_projection(_widen(ha, dtype), _widen(hb, dtype), gamma)

    ha_d = H.to_device(ha, dtype).view(B, S, Hkv, D)
    hb_d = H.to_device(hb, dtype).view(B, S, Hkv, D)
    U = torch.full((Hkv, D, D), float("nan"), device="cuda")
    sig = torch.full((Hkv, D), float("nan"), device="cuda")
    k = torch.full((Hkv,), -1, dtype=torch.int32, device="cuda")
    r_pad = 32
    Up = torch.full((Hkv, D, r_pad), float("nan"), device="cuda",
                    dtype=torch.bfloat16 if dtype == "bf16" else torch.float32)
    seka.seka_learn_projection(ha_d, hb_d, gamma, U, sig, k, U_packed=Up)
    torch.cuda.synchronize()
    got_U, got_S, got_k = H.to_f64(U), H.to_f64(sig), k.cpu().numpy()
    assert np.isfinite(got_U).all() and np.isfinite(got_S).all()

    for h in range(Hkv):
        s1 = ref_S[h, 0]
        assert np.abs(got_S[h] - ref_S[h]).max() <= SIGMA_TOL * s1, (name, h, np.abs(got_S[h] - ref_S[h]).max() / s1)
        assert np.all(np.diff(got_S[h]) <= 0)
        # rank rule (Eq. 3): the oracle's cumulative share must clear gamma by more than the fp32 error for the
        # integer to be decided; the seeds here do
        frac = np.cumsum(ref_S[h]) / ref_S[h].sum()
        kr = int(ref_k[h])
        if gamma < 1.0:
            assert frac[kr - 1] - gamma > 1e-4 and (kr == 1 or gamma - frac[kr - 2] > 1e-4), (name, h, frac[:kr + 1])
            assert got_k[h] == kr, (name, h, got_k[h], kr)
        else:
            # gamma = 1 asks for all of the mass: the trailing values are rounding noise on both sides, so only
            # "everything that matters" is fixed
            assert got_k[h] >= int(np.sum(ref_S[h] > 1e-4 * s1)), (name, h, got_k[h])
        live = got_S[h] > 1e-5 * got_S[h, 0]
        Ug = got_U[h]
        assert np.all(Ug[:, ~live] == 0.0)
        G = Ug[:, live].T @ Ug[:, live]
        assert np.abs(G - np.eye(G.shape[0])).max() <= ORTHO_TOL, (name, h, np.abs(G - np.eye(G.shape[0])).max())
        # every live column is a left singular vector of Omega for its singular value
        omega = _widen(ha, dtype)[:, h].T @ _widen(hb, dtype)[:, h] / n
        rows = np.linalg.norm(Ug[:, live].T @ omega, axis=1)
        assert np.abs(rows - got_S[h][live]).max() <= 5 * SIGMA_TOL * s1, (name, h)
        # leading block, where the rank rule cuts at a gap
        if kr < D and (ref_S[h, kr - 1] - ref_S[h, kr]) >= GAP * s1 and gamma < 1.0:
            P_got = Ug[:, :kr] @ Ug[:, :kr].T
            P_ref = ref_U[h][:, :kr] @ ref_U[h][:, :kr].T
            tol = 2 * SIGMA_TOL * s1 / (ref_S[h, kr - 1] - ref_S[h, kr])
            assert np.abs(P_got - P_ref).max() <= tol, (name, h, np.abs(P_got - P_ref).max(), tol)
        # isolated singular values: the vector itself, up to sign
        for c in range(D):
            lo = ref_S[h, c - 1] - ref_S[h, c] if c else np.inf
            hi = ref_S[h, c] - ref_S[h, c + 1] if c + 1 < D else np.inf
            if min(lo, hi) >= GAP * s1:
                assert abs(abs(Ug[:, c] @ ref_U[h][:, c]) - 1.0) <= 5e-6, (name, h, c)
        # the packed steering basis: leading min(k, r_pad) columns in the tensor dtype, zero beyond
        kp = min(int(got_k[h]), r_pad)
        want = U[h, :, :r_pad].clone()
        want[:, kp:] = 0
        assert torch.equal(Up[h], want.to(Up.dtype)), (name, h)


def test_learned_basis_recovers_the_planted_frame(seka):
    """The relevant context's key offsets live in a known subspace; the learned leading block must span it."""
    import torch
    n, Hkv, D, rank = 4096, 2, 128, 4
    print("learn planted frame", flush=True)
    g = np.random.default_rng(17)
    frame = np.linalg.qr(g.standard_normal((Hkv, D, rank)))[0]
    z = g.standard_normal((n, Hkv, rank)) * np.array([4.0, 3.0, 2.5, 2.0])
    sig_part = np.einsum("nhk,hdk->nhd", z, frame)
    ha = inputs.store(sig_part + 0.02 * g.standard_normal((n, Hkv, D)), "f32")
    hb = inputs.store(sig_part + 0.02 * g.standard_normal((n, Hkv, D)), "f32")
    U = torch.empty((Hkv, D, D), device="cuda")
    sig = torch.empty((Hkv, D), device="cuda")
    k = torch.empty((Hkv,), dtype=torch.int32, device="cuda")
    seka.seka_learn_projection(torch.from_numpy(ha).cuda().view(4, 1024, Hkv, D),
                               torch.from_numpy(hb).cuda().view(4, 1024, Hkv, D), 0.97, U, sig, k)
    torch.cuda.synchronize()
    got_U = H.to_f64(U)
    assert k.cpu().tolist() == [rank] * Hkv
    for h in range(Hkv):
        P = got_U[h][:, :rank] @ got_U[h][:, :rank].T
        assert np.abs(P - frame[h] @ frame[h].T).max() < 5e-3      # sampling noise of the planted data, not arithmetic


@pytest.mark.parametrize("dtype,B,S,Hkv,D", [("bf16", 2, 777, 4, 128), ("f32", 1, 130, 3, 64), ("f32", 1, 1, 2, 128)])
def test_head_distance_matches_oracle(seka, dtype, B, S, Hkv, D):
    import torch
    print(f"head distance {dtype} n={B * S} Hkv={Hkv} D={D}", flush=True)
    n = B * S
    hp, hm = inputs.paired_key_samples(n, Hkv, D, seed=8, dtype=dtype)
    ref = orc.head_relevance_distance(_widen(hp, dtype), _widen(hm, dtype))
    out = torch.full((Hkv,), float("nan"), device="cuda")
    seka.seka_head_distance(H.to_device(hp, dtype).view(B, S, Hkv, D), H.to_device(hm, dtype).view(B, S, Hkv, D), out)
    torch.cuda.synchronize()
    got = H.to_f64(out)
    assert np.abs(got - ref).max() <= 1e-5 * np.abs(ref).max(), (got, ref)
    same = torch.full((Hkv,), float("nan"), device="cuda")
    seka.seka_head_distance(H.to_device(hp, dtype).view(B, S, Hkv, D), H.to_device(hp, dtype).view(B, S, Hkv, D), same)
    torch.cuda.synchronize()
    assert torch.all(same == 0)


def test_learned_basis_steers_the_prefill(seka):
    """Offline stage -> inference: the packed basis the GPU learns (per-head rank from the gamma rule, zero-padded
    to a common width) steers seka_attention_prefill like the basis the oracle learns.  Singular vectors are only
    fixed up to sign, which the projector U U^T does not see."""
    import torch
    print("learn -> prefill", flush=True)
    n, Hkv, Hq, D, r_pad, gamma = 2048, 2, 8, 128, 32, 0.85
    ha, hb = inputs.paired_key_samples(n, Hkv, D, seed=12, dtype="bf16", rank=16, decay=0.85)
    wide = lambda x: inputs.bf16_bits_to_f32(x).astype(np.float64)
    ref_U, _, ref_k = orc.learn_projection(wide(ha), wide(hb), gamma)
    U_ref = np.zeros((Hkv, 1, D, r_pad))
    for h in range(Hkv):
        assert ref_k[h] <= r_pad
        U_ref[h, 0, :, :ref_k[h]] = ref_U[h][:, :ref_k[h]]
    U_ref = wide(inputs.store(U_ref, "bf16"))                        # the basis as a bf16 tensor would hold it

    U = torch.empty((Hkv, D, D), device="cuda")
    sig = torch.empty((Hkv, D), device="cuda")
    k = torch.empty((Hkv,), dtype=torch.int32, device="cuda")
    Up = torch.empty((Hkv, D, r_pad), device="cuda", dtype=torch.bfloat16)
    seka.seka_learn_projection(H.to_device(ha, "bf16").view(2, n // 2, Hkv, D), H.to_device(hb, "bf16").view(2, n // 2, Hkv, D),
                               gamma, U, sig, k, U_packed=Up)
    torch.cuda.synchronize()
    assert k.cpu().tolist() == [int(x) for x in ref_k]

    inp = inputs.make_layer("learned", "bf16", B=2, S=300, Hq=Hq, Hkv=Hkv, D=D, M=1, r=r_pad, gain=1.5,
                            mask_recipe=("cover", 0.25, 0.25, 3), seed=31)
    o = H.oracle_inputs(inp)
    dev = H.DeviceInputs(inp)
    O = torch.empty_like(dev.Q)
    seka.seka_attention_prefill(dev.Q, dev.K, dev.V, O, Up.view(Hkv, 1, D, r_pad), dev.gain, dev.mask, scale=inp.scale)
    torch.cuda.synchronize()
    ref_O, _ = orc.steered_attention(o["Q"], o["K"], o["V"], U_ref, inp.gain, inp.mask, scale=inp.scale)
    plain_O, _ = orc.causal_attention(o["Q"], o["K"], o["V"], scale=inp.scale)
    assert np.abs(ref_O - plain_O).max() > 1e-2, "steering with the learned basis has no visible effect: vacuous"
    H.assert_close_bf16(H.to_f64(O), ref_O, "prefill steered with the learned basis")

"""GPU parity of the dual-projector edit (paper Eq. 2 and Eq. 4, negative-side gain included) through the C ABI:
fused attention and standalone edit, fp32 and bf16, low-rank and dense forms of the fused edit."""
import numpy as np
import pytest

from oracle import seka_oracle as orc
from paper_2603_01281_amd import inputs
from tests import helpers as H

pytestmark = pytest.mark.gpu

CASES = {
    # name: (dtype, D, S, Hq, Hkv, k+, k-, g+, g-)
    "f32_D64": ("f32", 64, 200, 4, 2, [5, 9], [3, 12], [0.8, -0.4], [0.6, -1.0]),
    "bf16_low_rank": ("bf16", 128, 700, 8, 2, [10, 16], [6, 3], [1.0, 0.7], [-0.5, 0.8]),       # 2 x 16 columns
    "bf16_dense": ("bf16", 128, 700, 8, 2, [40, 33], [24, 12], [0.9, 1.4], [0.6, -0.7]),         # 2 x 40 columns
    "bf16_D64": ("bf16", 64, 300, 4, 2, [8, 6], [4, 8], [1.0, -0.6], [0.5, 0.9]),
}


@pytest.mark.parametrize("name", list(CASES))
def test_dual_projector_edit(seka, name):
    import torch
    dtype, D, S, Hq, Hkv, kp, kn, gp, gn = CASES[name]
    print(f"eq4 case {name}", flush=True)
    B = 2
    base = inputs.make_layer("eq4", dtype, B=B, S=S, Hq=Hq, Hkv=Hkv, D=D, M=1, r=8, gain=1.0,
                             mask_recipe=("cover", 0.15, 0.15, 3), seed=7)
    Up, Un = inputs.singular_vector_sets(Hkv, D, seed=7)
    U64, gain, w64, a = orc.eq4_as_low_rank(Up, Un, kp, kn, np.array(gp), np.array(gn), B)
    U_store = inputs.store(U64, dtype)                       # what the GPU reads; the oracle widens the same bits
    U_ref = base.widen(U_store)
    w32 = w64.astype(np.float32)
    Q, K, V = base.widen(base.Q), base.widen(base.K), base.widen(base.V)

    dev = H.DeviceInputs(base)
    U_dev = H.to_device(U_store, dtype)
    w_dev = torch.from_numpy(w32).cuda()
    ref_O, ref_L = orc.steered_attention(Q, K, V, U_ref, gain, base.mask, w=w32.astype(np.float64), scale=base.scale, key_scale=a)
    O = torch.full_like(dev.Q, float("nan"))
    lse = dev.lse_buffer()
    seka.seka_attention_prefill(dev.Q, dev.K, dev.V, O, U_dev, list(gain), dev.mask, w=w_dev, lse=lse, scale=base.scale,
                                key_scale=list(a))
    K_out = torch.empty_like(dev.K)
    seka.seka_edit_keys(dev.K, K_out, U_dev, list(gain), dev.mask, w=w_dev, key_scale=list(a))
    torch.cuda.synchronize()
    ref_K = orc.edit_keys(K, U_ref, gain, base.mask, w=w32.astype(np.float64), key_scale=a)
    # the generalised form really is Eq. 4 (up to the storage rounding of U)
    direct_K = orc.edit_keys_eq4(K, Up, Un, kp, kn, np.array(gp), np.array(gn), base.mask)
    assert np.abs(ref_K - direct_K).max() < (1e-5 if dtype == "f32" else 5e-2)
    # negative-side gain matters in this case (otherwise the test would not see key_scale at all)
    no_scale = orc.edit_keys(K, U_ref, gain, base.mask, w=w32.astype(np.float64))
    assert np.abs(no_scale - ref_K).max() > 0.05 * np.abs(K).max()

    if dtype == "f32":
        H.assert_close_f32(H.to_f64(O), ref_O, f"{name} O")
        H.assert_close_f32(H.to_f64(lse), ref_L, f"{name} LSE")
        H.assert_close_f32(H.to_f64(K_out), ref_K, f"{name} edited K")
    else:
        H.assert_close_bf16(H.to_f64(O), ref_O, f"{name} O")
        H.assert_lse_close_bf16(H.to_f64(lse), ref_L, f"{name} LSE")
        gmax = float(np.abs(w32).max() * 2 + np.abs(a).max())
        H.assert_edit_close_bf16(H.to_f64(K_out), ref_K, gmax, f"{name} edited K")
    off = base.mask == 0
    assert np.array_equal(H.to_f64(K_out)[off], K[off]), "unhighlighted rows must be copied bit-exactly"
    plain_O, _ = orc.causal_attention(Q, K, V, scale=base.scale)
    assert np.abs(ref_O - plain_O).max() > (1e-4 if dtype == "f32" else 5e-2), "steering has no visible effect: vacuous"

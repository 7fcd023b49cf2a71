"""GPU parity of seka_attention_prefill_ragged: a padded batch of prompts of different lengths."""
import numpy as np
import pytest

from oracle import seka_oracle as orc
from paper_2603_01281_amd import inputs
from tests import helpers as H

pytestmark = pytest.mark.gpu

CASES = {
    # name: (dtype, S, Hq, Hkv, D, r, lens)
    "bf16_D128": ("bf16", 700, 8, 2, 128, 32, [700, 259, 1, 64]),
    "bf16_D128_dense": ("bf16", 520, 4, 1, 128, 64, [130, 520, 0]),
    "bf16_D64": ("bf16", 300, 4, 2, 64, 16, [300, 111]),
    "f32_D64": ("f32", 150, 4, 2, 64, 8, [150, 70, 3]),
}


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("steered", [True, False])
def test_ragged_prefill(seka, name, steered):
    import torch
    dtype, S, Hq, Hkv, D, r, lens = CASES[name]
    B = len(lens)
    print(f"ragged case {name} steered={steered}", flush=True)
    inp = inputs.make_layer("ragged", dtype, B=B, S=S, Hq=Hq, Hkv=Hkv, D=D, M=1, r=r, gain=1.25,
                            mask_recipe=("cover", 0.3, 0.3, 4), seed=21)
    dev = H.DeviceInputs(inp)
    o = H.oracle_inputs(inp)
    lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
    O = torch.full_like(dev.Q, float("nan"))
    lse = torch.full((B, Hq, S), float("nan"), dtype=torch.float32, device="cuda")
    if steered:
        seka.seka_attention_prefill_ragged(dev.Q, dev.K, dev.V, O, lens_dev, dev.U, dev.gain, dev.mask, lse=lse, scale=inp.scale)
    else:
        seka.seka_attention_prefill_ragged(dev.Q, dev.K, dev.V, O, lens_dev, lse=lse, scale=inp.scale)
    torch.cuda.synchronize()
    got_O, got_L = H.to_f64(O), H.to_f64(lse)
    saw_effect = False
    for b, n in enumerate(lens):
        # padding rows are left untouched
        assert np.isnan(got_O[b, n:]).all() and np.isnan(got_L[b, :, n:]).all(), f"prompt {b}: padding rows were written"
        if n == 0:
            continue
        sl = lambda x: x[b:b + 1, :n]
        if steered:
            # highlight bits in the padding must not matter: the reference only sees the first n tokens
            ref_O, ref_L = orc.steered_attention(sl(o["Q"]), sl(o["K"]), sl(o["V"]), o["U"], inp.gain, inp.mask[b:b + 1, :n], scale=inp.scale)
            plain_O, _ = orc.causal_attention(sl(o["Q"]), sl(o["K"]), sl(o["V"]), scale=inp.scale)
            saw_effect |= np.abs(ref_O - plain_O).max() > 1e-3
        else:
            ref_O, ref_L = orc.causal_attention(sl(o["Q"]), sl(o["K"]), sl(o["V"]), scale=inp.scale)
        if dtype == "f32":
            H.assert_close_f32(got_O[b:b + 1, :n], ref_O, f"{name} prompt {b} O")
            H.assert_close_f32(got_L[b:b + 1, :, :n], ref_L, f"{name} prompt {b} LSE")
        else:
            H.assert_close_bf16(got_O[b:b + 1, :n], ref_O, f"{name} prompt {b} O")
            H.assert_lse_close_bf16(got_L[b:b + 1, :, :n], ref_L, f"{name} prompt {b} LSE", n_keys=n)
    assert saw_effect or not steered, "steering has no visible effect: vacuous"
    assert inp.mask[:, :].any()

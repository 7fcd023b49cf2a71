"""GPU parity of seka_attention_decode (generation step over a cache of edited keys) against the fp64 oracle."""
import numpy as np
import pytest

from oracle import seka_oracle as orc
from paper_2603_01281_amd import inputs
from tests import helpers as H

pytestmark = pytest.mark.gpu

CASES = {
    # name: (dtype, B, S, Hq, Hkv, D, lens)
    "bf16_G4": ("bf16", 3, 1500, 8, 2, 128, [1500, 777, 1]),
    "bf16_G7_splits": ("bf16", 1, 5000, 14, 2, 128, None),
    "bf16_G1_D64": ("bf16", 2, 300, 3, 3, 64, [299, 64]),
    "bf16_G16": ("bf16", 1, 400, 16, 1, 128, [333]),
    "bf16_G32_two_head_chunks": ("bf16", 1, 1100, 32, 1, 128, [1061]),
    "bf16_G20_two_head_chunks": ("bf16", 2, 700, 40, 2, 128, [700, 33]),
    "bf16_G5_D64_splits": ("bf16", 2, 3000, 10, 2, 64, [3000, 1031]),
    "f32_G2": ("f32", 2, 257, 4, 2, 128, [257, 100]),
    "f32_D64_G3": ("f32", 1, 130, 6, 2, 64, None),
    "empty_prompt": ("bf16", 2, 128, 4, 2, 128, [0, 128]),
}


@pytest.mark.parametrize("name", list(CASES))
def test_decode_matches_oracle(seka, name):
    import torch
    dtype, B, S, Hq, Hkv, D, lens = CASES[name]
    print(f"decode case {name}", flush=True)
    inp = inputs.make_layer("dec", dtype, B=B, S=S, Hq=Hq, Hkv=Hkv, D=D, M=1, r=8, gain=1.0,
                            mask_recipe=("cover", 0.1, 0.1, 2), seed=11)
    dev = H.DeviceInputs(inp)
    Q, K, V = inp.widen(inp.Q), inp.widen(inp.K), inp.widen(inp.V)
    # the cache holds edited keys: run the standalone hook in place, as a serving loop would after prefill
    seka.seka_edit_keys(dev.K, dev.K, dev.U, dev.gain, dev.mask)
    torch.cuda.synchronize()
    K_cache = H.to_f64(dev.K)                                   # exactly what the decode kernel reads
    assert np.abs(K_cache - K).max() > 0.1                      # the edit happened
    ln = np.full(B, S, np.int32) if lens is None else np.asarray(lens, np.int32)
    q_rows = np.stack([Q[b, max(int(ln[b]) - 1, 0)] for b in range(B)])          # the newest token's queries
    q_dev = torch.stack([dev.Q[b, max(int(ln[b]) - 1, 0)] for b in range(B)]).contiguous()
    O = torch.full_like(q_dev, float("nan"))
    lse = torch.empty((B, Hq), dtype=torch.float32, device="cuda")
    lens_dev = None if lens is None else torch.from_numpy(ln).cuda()
    seka.seka_attention_decode(q_dev, dev.K, dev.V, O, seq_lens=lens_dev, lse=lse, scale=inp.scale)
    torch.cuda.synchronize()
    got_O, got_L = H.to_f64(O), H.to_f64(lse)
    live = ln > 0
    ref_O, ref_L = orc.decode_attention(q_rows[live], K_cache[live], V[live], ln[live], scale=inp.scale)
    if dtype == "f32":
        H.assert_close_f32(got_O[live], ref_O, f"{name} O")
        H.assert_close_f32(got_L[live], ref_L, f"{name} LSE")
    else:
        H.assert_close_bf16(got_O[live], ref_O, f"{name} O")
        H.assert_lse_close_bf16(got_L[live], ref_L, f"{name} LSE", path="decode")
    if not live.all():
        assert np.all(got_O[~live] == 0.0) and np.all(np.isneginf(got_L[~live]))


def test_decode_agrees_with_last_prefill_row(seka):
    """The fused prefill (edit on chip) and decode over the persisted edited cache see the same keys."""
    import torch
    inp = inputs.make_config(2, seed=3, S=900, Hq=8, Hkv=2)
    dev = H.DeviceInputs(inp)
    O_pre = torch.empty_like(dev.Q)
    seka.seka_attention_prefill(dev.Q, dev.K, dev.V, O_pre, dev.U, dev.gain, dev.mask, scale=inp.scale)
    Kc = dev.K.clone()
    seka.seka_edit_keys(dev.K, Kc, dev.U, dev.gain, dev.mask)
    q = dev.Q[:, -1].contiguous()
    O_dec = torch.empty_like(q)
    seka.seka_attention_decode(q, Kc, dev.V, O_dec, scale=inp.scale)
    torch.cuda.synchronize()
    d = np.abs(H.to_f64(O_dec) - H.to_f64(O_pre[:, -1]))
    assert d.max() <= H.BF16_MAX

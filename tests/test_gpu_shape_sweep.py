"""GPU parity of the bf16 D = 128 prefill kernels over sequence lengths around every boundary of the tile loop
(32-key blocks, 64-key tiles, the three ring stages, one to several row blocks per workgroup pair) and over the
four workgroup shapes (query heads per KV head divisible by 4, by 7, by 2, odd)."""
import numpy as np
import pytest

from oracle import seka_oracle as orc
from paper_2603_01281_amd import inputs
from tests import helpers as H

pytestmark = pytest.mark.gpu

LENGTHS = [1, 2, 31, 32, 33, 63, 64, 65, 96, 97, 127, 128, 129, 191, 192, 193, 255, 256, 257, 320, 383, 385, 449, 513, 577, 640, 705]
GROUPS = {"G4": (4, 1), "G7": (7, 1), "G2": (4, 2), "G1": (3, 3)}        # name: (Hq, Hkv)


@pytest.mark.parametrize("rank", [16, 48])          # low-rank edit / dense edit (different paths through the tile loop)
@pytest.mark.parametrize("group", list(GROUPS))
def test_lengths_around_tile_boundaries(seka, group, rank):
    import torch
    Hq, Hkv = GROUPS[group]
    lengths = LENGTHS if (group == "G4" and rank == 16) else LENGTHS[::3] + [1000]
    worst = 0.0
    for S in lengths:
        print(f"sweep {group} r={rank} S={S}", flush=True)
        inp = inputs.make_layer("sweep", "bf16", B=2, S=S, Hq=Hq, Hkv=Hkv, D=128, M=1, r=rank, gain=1.0,
                                mask_recipe=("cover", 0.3, 0.3, 2) if S >= 8 else ("all",), seed=100 + S)
        dev = H.DeviceInputs(inp)
        o = H.oracle_inputs(inp)
        O = torch.full_like(dev.Q, float("nan"))
        lse = torch.full((2, Hq, S), float("nan"), dtype=torch.float32, device="cuda")
        seka.seka_attention_prefill(dev.Q, dev.K, dev.V, O, dev.U, dev.gain, dev.mask, lse=lse, scale=inp.scale)
        torch.cuda.synchronize()
        ref_O, ref_L = orc.steered_attention(o["Q"], o["K"], o["V"], o["U"], inp.gain, inp.mask, scale=inp.scale)
        H.assert_close_bf16(H.to_f64(O), ref_O, f"{group} r={rank} S={S} O")
        H.assert_lse_close_bf16(H.to_f64(lse), ref_L, f"{group} S={S} LSE", n_keys=S)
        Op = torch.full_like(dev.Q, float("nan"))
        lse.fill_(float("nan"))
        seka.seka_attention_plain(dev.Q, dev.K, dev.V, Op, lse=lse, scale=inp.scale)
        torch.cuda.synchronize()
        ref_P, ref_PL = orc.causal_attention(o["Q"], o["K"], o["V"], scale=inp.scale)
        H.assert_close_bf16(H.to_f64(Op), ref_P, f"{group} S={S} plain O")
        H.assert_lse_close_bf16(H.to_f64(lse), ref_PL, f"{group} S={S} plain LSE", path="plain")
        worst = max(worst, float(np.abs(H.to_f64(O) - ref_O).max()))
    print(f"{group}: worst |dO| {worst:.4f}", flush=True)

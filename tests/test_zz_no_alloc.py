"""seka_attention_decode_static (the entry point for callers that cannot allocate) against seka_attention_decode:
two calls in a row through the C ABI, the second with a smaller input, each compared bit for bit with the
workspace-taking entry point and, to the usual bars, with the oracle."""
import ctypes

import numpy as np
import pytest

from oracle import seka_oracle as orc
from paper_2603_01281_amd import inputs
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _decode_both(seka, inp, dev, lens):
    import torch
    B, S, Hq, Hkv, D = inp.B, inp.S, inp.Hq, inp.Hkv, inp.D
    ln = np.asarray(lens, np.int32)
    q_dev = torch.stack([dev.Q[b, max(int(ln[b]) - 1, 0)] for b in range(B)]).contiguous()
    lens_dev = torch.from_numpy(ln).cuda()
    sh = seka.seka_shape(B, S, Hq, Hkv, D, seka.SEKA_BF16, float(inp.scale))
    need = seka.lib.seka_decode_workspace_bytes(ctypes.byref(sh))
    assert 0 < need <= seka.SEKA_DECODE_STATIC_MAX_BYTES
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    outs = []
    for static in (False, True):
        O = torch.full_like(q_dev, float("nan"))
        lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device="cuda")
        args = [q_dev.data_ptr(), dev.K.data_ptr(), dev.V.data_ptr(), O.data_ptr(), lse.data_ptr(), lens_dev.data_ptr(),
                ctypes.byref(sh)]
        if static:
            rc = seka.lib.seka_attention_decode_static(*args, stream)
        else:
            rc = seka.lib.seka_attention_decode(*args, ws.data_ptr(), need, stream)
        assert rc == 0, seka.lib.seka_status_string(rc)
        torch.cuda.synchronize()
        outs.append((O, lse))
    (O_ws, L_ws), (O_st, L_st) = outs
    assert torch.equal(O_ws, O_st), "static-buffer result differs from the workspace result (O)"
    assert torch.equal(L_ws, L_st), "static-buffer result differs from the workspace result (LSE)"
    q_rows = np.stack([inp.widen(inp.Q)[b, max(int(ln[b]) - 1, 0)] for b in range(B)])
    ref_O, ref_L = orc.decode_attention(q_rows, inp.widen(inp.K), inp.widen(inp.V), ln, scale=inp.scale)
    H.assert_close_bf16(H.to_f64(O_st), ref_O, "decode_static O")
    H.assert_lse_close_bf16(H.to_f64(L_st), ref_L, "decode_static LSE", path="decode")


def test_decode_static_two_calls_second_smaller(seka):
    print("decode_static: B=3 S=3000 G=4 (several splits), then B=2 S=700", flush=True)
    big = inputs.make_layer("dec_static", "bf16", B=3, S=3000, Hq=8, Hkv=2, D=128, M=1, r=8, gain=1.0,
                            mask_recipe=("none",), seed=21)
    small = inputs.make_layer("dec_static", "bf16", B=2, S=700, Hq=8, Hkv=2, D=128, M=1, r=8, gain=1.0,
                              mask_recipe=("none",), seed=22)
    dev_big, dev_small = H.DeviceInputs(big), H.DeviceInputs(small)
    _decode_both(seka, big, dev_big, [3000, 1777, 5])
    _decode_both(seka, small, dev_small, [700, 64])


@pytest.mark.parametrize("dtype,B,S,Hq,Hkv,D,lens", [
    ("bf16", 1, 20000, 14, 2, 128, [20000]),          # 39 splits, seven heads per workgroup
    ("bf16", 2, 9000, 40, 2, 128, [9000, 4097]),      # two head chunks of ten heads
    ("bf16", 2, 5000, 6, 3, 64, [4999, 0]),           # D = 64, an empty prompt
    ("f32", 2, 2600, 4, 2, 128, [2600, 513]),         # fp32 kernel
])
def test_decode_static_many_splits_repeated(seka, dtype, B, S, Hq, Hkv, D, lens):
    """Shapes with many splits, seven and ten heads per workgroup, D = 64 and the fp32 kernel: three calls in a row
    on the library's buffer, each bit-identical to the workspace entry point (nothing in the buffer has to
    survive or be cleared between calls)."""
    import torch
    print(f"decode_static repeated: {dtype} B={B} S={S} Hq={Hq} Hkv={Hkv} D={D} lens={lens}", flush=True)
    inp = inputs.make_layer("dec_static_merge", dtype, B=B, S=S, Hq=Hq, Hkv=Hkv, D=D, M=1, r=8, gain=1.0,
                            mask_recipe=("none",), seed=31)
    dev = H.DeviceInputs(inp)
    ln = np.asarray(lens, np.int32)
    q_dev = torch.stack([dev.Q[b, max(int(ln[b]) - 1, 0)] for b in range(B)]).contiguous()
    lens_dev = torch.from_numpy(ln).cuda()
    code = seka.SEKA_BF16 if dtype == "bf16" else seka.SEKA_F32
    sh = seka.seka_shape(B, S, Hq, Hkv, D, code, float(inp.scale))
    need = seka.lib.seka_decode_workspace_bytes(ctypes.byref(sh))
    assert need > B * Hq * (D + 2) * 4, "this case is meant to have several splits"
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream

    def run(static):
        O = torch.full_like(q_dev, float("nan"))
        lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device="cuda")
        args = [q_dev.data_ptr(), dev.K.data_ptr(), dev.V.data_ptr(), O.data_ptr(), lse.data_ptr(), lens_dev.data_ptr(),
                ctypes.byref(sh)]
        rc = (seka.lib.seka_attention_decode_static(*args, stream) if static
              else seka.lib.seka_attention_decode(*args, ws.data_ptr(), need, stream))
        assert rc == 0, seka.lib.seka_status_string(rc)
        torch.cuda.synchronize()
        return O, lse

    O_ws, L_ws = run(False)
    for rep in range(3):
        O_st, L_st = run(True)
        assert torch.equal(O_ws, O_st) and torch.equal(L_ws, L_st), f"call {rep}: static result differs from the workspace result"
    live = ln > 0
    q_rows = np.stack([inp.widen(inp.Q)[b, max(int(ln[b]) - 1, 0)] for b in range(B)])
    ref_O, ref_L = orc.decode_attention(q_rows[live], inp.widen(inp.K)[live], inp.widen(inp.V)[live], ln[live], scale=inp.scale)
    if dtype == "bf16":
        H.assert_close_bf16(H.to_f64(O_ws)[live], ref_O, "decode O")
        H.assert_lse_close_bf16(H.to_f64(L_ws)[live], ref_L, "decode LSE", path="decode")
    else:
        H.assert_close_f32(H.to_f64(O_ws)[live], ref_O, "decode O")


def test_decode_static_rejects_what_does_not_fit(seka):
    """Partial states beyond the library's buffer are a workspace error on the host: nothing is launched."""
    import torch
    sh = seka.seka_shape(64, 65536, 64, 8, 128, seka.SEKA_BF16, 0.0)
    assert seka.lib.seka_decode_workspace_bytes(ctypes.byref(sh)) > seka.SEKA_DECODE_STATIC_MAX_BYTES
    t = torch.empty(16, dtype=torch.uint8, device="cuda")      # never dereferenced: the size check comes first
    far = 1 << 40
    rc = seka.lib.seka_attention_decode_static(t.data_ptr(), t.data_ptr() + far, t.data_ptr() + 2 * far,
                                               t.data_ptr() + 3 * far, None, None, ctypes.byref(sh), None)
    assert rc == 8

"""GPU parity of seka_attention_prefill_packed: a batch of prompts stored back to back, without padding."""
import numpy as np
import pytest

from oracle import seka_oracle as orc
from paper_2603_01281_amd import inputs
from tests import helpers as H

pytestmark = pytest.mark.gpu

CASES = {
    # name: (dtype, Hq, Hkv, D, M, r, lens, extra rows after the last prompt, bound passed as max_len)
    "bf16_D128": ("bf16", 8, 2, 128, 1, 32, [700, 259, 1, 64], 0, 700),
    "bf16_D128_odd_starts": ("bf16", 4, 1, 128, 1, 16, [77, 301, 513], 5, 640),      # mask rows not 16-byte aligned
    "bf16_D128_dense_experts": ("bf16", 4, 1, 128, 2, 32, [130, 0, 520], 0, 520),   # per-prompt coefficients, empty prompt
    "bf16_D64": ("bf16", 4, 2, 64, 1, 16, [300, 111], 3, 300),
    "f32_D64": ("f32", 4, 2, 64, 1, 8, [150, 70, 3], 0, 150),
}


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("steered", [True, False])
def test_packed_prefill(seka, name, steered):
    import torch
    dtype, Hq, Hkv, D, M, r, lens, extra, max_len = CASES[name]
    B = len(lens)
    Smax = max(lens)
    print(f"packed case {name} steered={steered}", flush=True)
    inp = inputs.make_layer("packed", dtype, B=B, S=Smax, Hq=Hq, Hkv=Hkv, D=D, M=M, r=r, gain=1.25,
                            mask_recipe=("cover", 0.3, 0.3, 4), seed=23)
    o = H.oracle_inputs(inp)
    dev = H.DeviceInputs(inp)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(cu[-1]) + extra
    pack = lambda t: torch.cat([t[b, :n] for b, n in enumerate(lens)] + [t[0, :extra]], dim=0).contiguous()
    Qp, Kp, Vp, maskp = pack(dev.Q), pack(dev.K), pack(dev.V), pack(dev.mask)
    assert Qp.shape[0] == total
    w = None
    if M > 1:
        g = np.random.default_rng(5)
        w_np = g.random((B, Hkv, M)).astype(np.float32)
        w_np /= w_np.sum(-1, keepdims=True)
        w = torch.from_numpy(w_np).cuda()
    O = torch.full_like(Qp, float("nan"))
    lse = torch.full((Hq, total), float("nan"), dtype=torch.float32, device="cuda")
    cu_dev = torch.from_numpy(cu).cuda()
    if steered:
        seka.seka_attention_prefill_packed(Qp, Kp, Vp, O, cu_dev, max_len, dev.U, dev.gain, maskp, w=w, lse=lse, scale=inp.scale)
    else:
        seka.seka_attention_prefill_packed(Qp, Kp, Vp, O, cu_dev, max_len, lse=lse, scale=inp.scale)
    torch.cuda.synchronize()
    got_O, got_L = H.to_f64(O), H.to_f64(lse)
    # rows after the last prompt belong to nobody and are left alone
    assert np.isnan(got_O[cu[-1]:]).all() and np.isnan(got_L[:, cu[-1]:]).all()
    saw_effect = False
    for b, n in enumerate(lens):
        if n == 0:
            continue
        sl = lambda x: x[b:b + 1, :n]
        if steered:
            ref_O, ref_L = orc.steered_attention(sl(o["Q"]), sl(o["K"]), sl(o["V"]), o["U"], inp.gain, inp.mask[b:b + 1, :n],
                                                 w=None if w is None else w_np[b:b + 1].astype(np.float64), scale=inp.scale)
            plain_O, _ = orc.causal_attention(sl(o["Q"]), sl(o["K"]), sl(o["V"]), scale=inp.scale)
            saw_effect |= np.abs(ref_O - plain_O).max() > 1e-3
        else:
            ref_O, ref_L = orc.causal_attention(sl(o["Q"]), sl(o["K"]), sl(o["V"]), scale=inp.scale)
        gO = got_O[cu[b]:cu[b + 1]][None]                       # [1, n, Hq, D]
        gL = got_L[:, cu[b]:cu[b + 1]][None]                    # [1, Hq, n]
        if dtype == "f32":
            H.assert_close_f32(gO, ref_O, f"{name} prompt {b} O")
            H.assert_close_f32(gL, ref_L, f"{name} prompt {b} LSE")
        else:
            H.assert_close_bf16(gO, ref_O, f"{name} prompt {b} O")
            H.assert_lse_close_bf16(gL, ref_L, f"{name} prompt {b} LSE", n_keys=int(cu[b + 1] - cu[b]))
    assert saw_effect or not steered, "steering has no visible effect: vacuous"


def test_packed_offsets_are_clamped(seka):
    """Offsets that point outside the tensors are clamped on the device: the call completes and prompts whose
    offsets are sane still get the right answer."""
    import torch
    print("packed clamp", flush=True)
    inp = inputs.make_layer("packed", "bf16", B=2, S=200, Hq=4, Hkv=2, D=128, M=1, r=8, gain=1.0,
                            mask_recipe=("cover", 0.2, 0.2, 2), seed=4)
    o = H.oracle_inputs(inp)
    dev = H.DeviceInputs(inp)
    Qp = torch.cat([dev.Q[0], dev.Q[1]]).contiguous()
    Kp = torch.cat([dev.K[0], dev.K[1]]).contiguous()
    Vp = torch.cat([dev.V[0], dev.V[1]]).contiguous()
    O = torch.zeros_like(Qp)
    cu = torch.tensor([0, 200, 1 << 30, -7], dtype=torch.int32, device="cuda")      # prompts 1 and 2 are nonsense
    seka.seka_attention_prefill_packed(Qp, Kp, Vp, O, cu, 200, scale=inp.scale)
    torch.cuda.synchronize()
    ref_O, _ = orc.causal_attention(o["Q"][:1], o["K"][:1], o["V"][:1], scale=inp.scale)
    H.assert_close_bf16(H.to_f64(O[:200])[None], ref_O, "prompt 0 beside nonsense offsets")
    assert torch.isfinite(O.float()).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_route_ragged(seka, dtype):
    """seka_route_ragged, padded with lengths and packed, against the oracle called prompt by prompt on each
    prompt's own token range (Sec. 3.3: the routing query sits at the end of each prompt)."""
    import torch
    Hq, Hkv, D, M, Ktop = 8, 2, 128, 4, 5
    lens = [517, 1, 0, 130, 64]
    B, S = len(lens), max(lens)
    print(f"route ragged {dtype}", flush=True)
    Q = inputs.gaussian((B, S, Hq, D), 11, "Q", dtype)
    Qd = H.to_device(Q, dtype)
    Q64 = inputs.bf16_bits_to_f32(Q).astype(np.float64) if dtype == "bf16" else Q.astype(np.float64)
    proto = inputs.unit_prototypes(Hkv, M, D, 11)
    pd = torch.from_numpy(proto).cuda()
    g = np.random.default_rng(12)
    U_top = np.stack([[np.linalg.qr(g.standard_normal((D, Ktop)))[0] for _ in range(M)] for _ in range(Hkv)])
    sigma = np.sort(g.random((Hkv, M, Ktop)) + 0.1, axis=-1)[..., ::-1].copy()
    p6 = torch.from_numpy(np.einsum("hmdk,hmk->hmd", U_top, sigma).astype(np.float32)).cuda()
    lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cu_dev = torch.from_numpy(cu).cuda()
    extra = 3                                            # rows after the last prompt, never read as a prompt's
    Qp = torch.cat([Qd[b, :n] for b, n in enumerate(lens)] + [Qd[0, :extra]], dim=0).contiguous()
    for window in (1, 50, S, 4 * S):
        ref_w = np.zeros((B, Hkv, M))
        ref_a = np.zeros((B, Hkv, M))
        for b, n in enumerate(lens):
            if n == 0:
                ref_w[b] = 1.0 / M                       # no query: every cosine is 0
                continue
            t0 = max(0, n - window)
            ref_w[b] = orc.route_softmax_cos(Q64[b:b + 1], proto, t0, n, 10.0)[0]
            ref_a[b] = orc.route_eq6(Q64[b:b + 1], U_top, sigma, t0, n)[0]
        for layout in ("padded", "packed"):
            kw = dict(seq_lens=lens_dev) if layout == "padded" else dict(cu_seqlens=cu_dev, max_len=S)
            Qin = Qd if layout == "padded" else Qp
            w = seka.seka_route_ragged(Qin, pd, window, mode=seka.SEKA_ROUTE_SOFTMAX_COS, tau=10.0, **kw)
            a = seka.seka_route_ragged(Qin, p6, window, mode=seka.SEKA_ROUTE_PAPER_EQ6, tau=0.0, **kw)
            assert np.abs(H.to_f64(w) - ref_w).max() <= H.ROUTE_ABS, (layout, window)
            assert np.abs(H.to_f64(a) - ref_a).max() <= H.ROUTE_ABS, (layout, window)
    # equal lengths and the whole prompt: the same numbers as seka_route
    full = torch.full((B,), S, dtype=torch.int32, device="cuda")
    assert torch.equal(seka.seka_route_ragged(Qd, pd, S, seq_lens=full), seka.seka_route(Qd, pd, 0, S))


@pytest.mark.parametrize("name", ["bf16_D128_dense_experts", "bf16_D128_odd_starts", "f32_D64"])
def test_packed_edit_keys(seka, name):
    """seka_edit_keys_packed against the oracle's edit, prompt by prompt with that prompt's expert weights; rows
    that belong to no prompt stay as they were, out of place and in place."""
    import torch
    dtype, Hq, Hkv, D, M, r, lens, extra, max_len = CASES[name]
    B, Smax = len(lens), max(lens)
    print(f"packed edit {name}", flush=True)
    inp = inputs.make_layer("packed_edit", dtype, B=B, S=Smax, Hq=Hq, Hkv=Hkv, D=D, M=M, r=r, gain=1.25,
                            mask_recipe=("cover", 0.3, 0.3, 4), seed=29)
    o = H.oracle_inputs(inp)
    dev = H.DeviceInputs(inp)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(cu[-1]) + extra
    pack = lambda t: torch.cat([t[b, :n] for b, n in enumerate(lens)] + [t[0, :extra]], dim=0).contiguous()
    Kp, maskp = pack(dev.K), pack(dev.mask)
    if extra:
        maskp[cu[-1]:] = 1                                # a set bit outside every prompt must not edit anything
    w, w_np = None, None
    if M > 1:
        g = np.random.default_rng(6)
        w_np = g.random((B, Hkv, M)).astype(np.float32)
        w_np /= w_np.sum(-1, keepdims=True)
        w = torch.from_numpy(w_np).cuda()
    cu_dev = torch.from_numpy(cu).cuda()
    K_out = torch.full_like(Kp, float("nan"))
    seka.seka_edit_keys_packed(Kp, K_out, cu_dev, max_len, dev.U, dev.gain, maskp, w=w)
    K_io = Kp.clone()
    seka.seka_edit_keys_packed(K_io, K_io, cu_dev, max_len, dev.U, dev.gain, maskp, w=w)
    torch.cuda.synchronize()
    got, got_io = H.to_f64(K_out), H.to_f64(K_io)
    assert np.isnan(got[cu[-1]:]).all()                   # nobody's rows: not written
    assert np.array_equal(got_io[cu[-1]:], H.to_f64(Kp)[cu[-1]:])
    changed = False
    for b, n in enumerate(lens):
        if n == 0:
            continue
        ref = orc.edit_keys(o["K"][b:b + 1, :n], o["U"], inp.gain, inp.mask[b:b + 1, :n],
                            w=None if w_np is None else w_np[b:b + 1].astype(np.float64))[0]
        for res, what in ((got[cu[b]:cu[b + 1]], "out of place"), (got_io[cu[b]:cu[b + 1]], "in place")):
            if dtype == "bf16":
                H.assert_edit_close_bf16(res, ref, 1.25, f"{name} prompt {b} {what}")
            else:
                assert np.abs(res - ref).max() <= H.F32_ABS, (name, b, what)
        changed |= bool(np.abs(ref - o["K"][b, :n]).max() > 1e-3)
    assert changed

"""C-ABI checks that need no GPU: the library loads, exports every declared symbol, and rejects
bad arguments on the host before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2603_01281_amd import binding
    return binding


def test_exports_every_declared_symbol(B):
    header = open(os.path.join(ROOT, "include", "seka.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(seka_[a-z_0-9]+)\s*\(", header))
    assert {"seka_route", "seka_edit_keys", "seka_attention_prefill", "seka_attention_plain",
            "seka_route_workspace_bytes", "seka_status_string",
            "seka_attention_decode", "seka_decode_workspace_bytes", "seka_attention_prefill_ragged",
            "seka_learn_workspace_bytes", "seka_learn_projection", "seka_head_distance",
            "seka_attention_prefill_packed", "seka_route_ragged", "seka_route_ragged_workspace_bytes", "seka_edit_keys_packed", "seka_project_route",
            "seka_project_route_workspace_bytes"} <= names
    for n in names:
        assert hasattr(B.lib, n), f"libseka.so does not export {n}"


def test_status_strings(B):
    seen = set()
    for code in range(0, 9):
        s = B.lib.seka_status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert B.lib.seka_status_string(1234) == b"unknown status"


FAKE = 0x10000   # aligned, never dereferenced: validation fails before any launch


def _shape(B, **kw):
    d = dict(B=1, S=128, Hq=4, Hkv=2, D=64, dtype=B.SEKA_F32, softmax_scale=0.0)
    d.update(kw)
    return B.seka_shape(d["B"], d["S"], d["Hq"], d["Hkv"], d["D"], d["dtype"], d["softmax_scale"])


def _steer(B, Hkv=2, **kw):
    gains = (ctypes.c_float * Hkv)(*([1.0] * Hkv))
    d = dict(M=1, r=8, U=FAKE, w=None, gain=gains, mask=FAKE, key_scale=None)
    d.update(kw)
    st = B.seka_steer(d["M"], d["r"], d["U"], d["w"], d["gain"], d["mask"], d["key_scale"])
    st._keep = (gains, d["key_scale"])
    return st


def test_attention_rejects_bad_arguments(B):
    L = B.lib
    ok = _shape(B)
    call = lambda q, k, v, o, sh: L.seka_attention_plain(q, k, v, o, None, ctypes.byref(sh), None)
    assert call(None, FAKE, FAKE, FAKE, ok) == 1                      # NULL
    assert call(FAKE, FAKE, FAKE, None, ok) == 1
    assert L.seka_attention_plain(FAKE, FAKE, FAKE, FAKE, None, None, None) == 1
    assert call(FAKE, FAKE, FAKE, FAKE * 4, _shape(B, D=96)) == 2     # head dim
    assert call(FAKE, FAKE, FAKE, FAKE * 4, _shape(B, Hq=5)) == 2     # Hq % Hkv
    assert call(FAKE, FAKE, FAKE, FAKE * 4, _shape(B, S=0)) == 2
    assert call(FAKE, FAKE, FAKE, FAKE * 4, _shape(B, Hkv=128, Hq=128)) == 2
    assert call(FAKE, FAKE, FAKE, FAKE * 4, _shape(B, dtype=7)) == 3  # dtype
    assert call(FAKE + 4, FAKE, FAKE, FAKE * 4, ok) == 4              # alignment
    assert call(FAKE, FAKE, FAKE, FAKE, ok) == 5                      # O aliases Q
    assert call(FAKE * 4, FAKE, FAKE * 8, FAKE + 64, ok) == 5         # O overlaps K


def test_steering_rejects_bad_arguments(B):
    L = B.lib
    ok = _shape(B)
    far = FAKE * 64
    call = lambda st, sh=ok: L.seka_attention_prefill(FAKE, FAKE * 4, FAKE * 8, far, None, ctypes.byref(sh), ctypes.byref(st), None)
    assert call(_steer(B, U=None)) == 1
    assert call(_steer(B, M=0)) == 2
    assert call(_steer(B, M=4, r=64)) == 2          # M*r > 128
    assert call(_steer(B, r=80)) == 2               # r > D
    assert call(_steer(B, key_scale=(ctypes.c_float * 2)(1.0, float("inf")))) == 2     # key scale must be finite
    assert call(_steer(B, U=FAKE + 2)) == 4
    bad_gain = (ctypes.c_float * 2)(1.0, float("nan"))
    assert call(_steer(B, gain=bad_gain)) == 2
    bf = _shape(B, dtype=B.SEKA_BF16)
    assert call(_steer(B, r=5), bf) == 6            # bf16 needs r % 8 == 0
    # edit_keys: partial overlap of input and output
    st = _steer(B)
    assert L.seka_edit_keys(FAKE, FAKE + 64, ctypes.byref(ok), ctypes.byref(st), None) == 5
    assert L.seka_edit_keys(FAKE, None, ctypes.byref(ok), ctypes.byref(st), None) == 1
    assert L.seka_edit_keys(FAKE, FAKE, ctypes.byref(ok), None, None) == 1
    # packed layout: offsets are required, the row count must be positive, partial overlap is refused
    assert L.seka_edit_keys_packed(FAKE, FAKE, ctypes.byref(ok), ctypes.byref(st), None, 100, None) == 1
    assert L.seka_edit_keys_packed(FAKE, FAKE, ctypes.byref(ok), ctypes.byref(st), FAKE * 9, 0, None) == 2
    assert L.seka_edit_keys_packed(FAKE, FAKE, ctypes.byref(ok), ctypes.byref(st), FAKE * 9 + 1, 100, None) == 4
    assert L.seka_edit_keys_packed(FAKE, FAKE + 64, ctypes.byref(ok), ctypes.byref(st), FAKE * 9, 100, None) == 5


def test_route_rejects_bad_arguments(B):
    L = B.lib
    ok = _shape(B)
    need = L.seka_route_workspace_bytes(ctypes.byref(ok), 0, 128)
    assert need > 0 and need % 16 == 0
    assert L.seka_route_workspace_bytes(ctypes.byref(ok), 5, 5) == 0
    call = lambda **kw: L.seka_route(kw.get("Q", FAKE), ctypes.byref(kw.get("sh", ok)), kw.get("proto", FAKE * 2), kw.get("M", 4),
                                     kw.get("t0", 0), kw.get("t1", 128), kw.get("mode", 0), kw.get("tau", 10.0),
                                     kw.get("w", FAKE * 3), kw.get("ws", FAKE * 5), kw.get("wsb", need), None)
    assert call(Q=None) == 1
    assert call(M=0) == 2 and call(M=17) == 2
    assert call(t0=10, t1=10) == 2 and call(t1=129) == 2 and call(t0=-1) == 2
    assert call(mode=9) == 6
    assert call(tau=float("inf")) == 2
    assert call(ws=None) == 8 and call(wsb=need - 1) == 8
    assert call(ws=FAKE * 5 + 8) == 4


def test_route_ragged_rejects_bad_arguments(B):
    L = B.lib
    ok = _shape(B)
    need = L.seka_route_ragged_workspace_bytes(ctypes.byref(ok), 1)
    assert need > 0 and need % 16 == 0
    assert L.seka_route_ragged_workspace_bytes(ctypes.byref(ok), 0) == 0
    # a window beyond the prompt needs what the whole prompt needs
    assert L.seka_route_ragged_workspace_bytes(ctypes.byref(ok), 1 << 30) == L.seka_route_workspace_bytes(ctypes.byref(ok), 0, ok.S)
    call = lambda **kw: L.seka_route_ragged(kw.get("Q", FAKE), ctypes.byref(kw.get("sh", ok)), kw.get("proto", FAKE * 2), kw.get("M", 4),
                                            kw.get("lens", FAKE * 7), kw.get("cu", None), kw.get("total", 0), kw.get("window", 1),
                                            kw.get("mode", 0), kw.get("tau", 10.0), kw.get("w", FAKE * 3), kw.get("ws", FAKE * 5),
                                            kw.get("wsb", need), None)
    assert call(Q=None) == 1 and call(w=None) == 1
    assert call(lens=None) == 1                                   # neither lengths nor offsets
    assert call(window=0) == 2 and call(M=0) == 2
    assert call(lens=None, cu=FAKE * 7, total=0) == 2             # packed layout needs its row count
    assert call(lens=FAKE * 7 + 2) == 4 and call(lens=None, cu=FAKE * 7 + 2, total=10) == 4
    assert call(mode=9) == 6
    assert call(ws=None) == 8 and call(wsb=need - 1) == 8


def test_project_route_rejects_bad_arguments(B):
    L = B.lib
    ok = _shape(B, S=256, Hq=8, Hkv=2, D=128, dtype=B.SEKA_BF16)
    need = L.seka_project_route_workspace_bytes(ctypes.byref(ok))
    assert need > 0 and need % 16 == 0
    assert L.seka_project_route_workspace_bytes(ctypes.byref(_shape(B, S=200, Hq=8, Hkv=2, D=128, dtype=B.SEKA_BF16))) == 0
    far = FAKE * 4096
    call = lambda **kw: L.seka_project_route(kw.get("X", FAKE), kw.get("W", FAKE * 64), kw.get("E", 256), kw.get("Q", far),
                                             ctypes.byref(kw.get("sh", ok)), kw.get("proto", FAKE * 2), kw.get("M", 4), kw.get("mode", 0),
                                             kw.get("tau", 10.0), kw.get("w", FAKE * 3), kw.get("ws", FAKE * 5), kw.get("wsb", need), None)
    assert call(X=None) == 1 and call(Q=None) == 1 and call(proto=None) == 1
    assert call(E=100) == 2 and call(E=0) == 2 and call(M=0) == 2
    assert call(sh=_shape(B, S=200, Hq=8, Hkv=2, D=128, dtype=B.SEKA_BF16)) == 6      # S not a multiple of 128
    assert call(sh=_shape(B, S=256, Hq=8, Hkv=2, D=64, dtype=B.SEKA_BF16)) == 6       # D = 64
    assert call(sh=_shape(B, S=256, Hq=8, Hkv=2, D=128)) == 6                          # fp32
    assert call(Q=FAKE) == 5                                                           # output over the input
    assert call(ws=None) == 8 and call(wsb=need - 1) == 8
    assert call(mode=9) == 6


def test_decode_rejects_bad_arguments(B):
    L = B.lib
    ok = _shape(B)
    need = L.seka_decode_workspace_bytes(ctypes.byref(ok))
    assert need > 0 and need % 4 == 0
    far, ws = FAKE * 64, FAKE * 128
    call = lambda q, o, sh=ok, w=ws, wb=need, lens=None: L.seka_attention_decode(q, FAKE * 4, FAKE * 8, o, None, lens, ctypes.byref(sh), w, wb, None)
    assert call(None, far) == 1
    assert call(FAKE, far, _shape(B, D=96)) == 2
    assert call(FAKE + 2, far) == 4
    assert call(FAKE, far, lens=FAKE + 2) == 4
    assert call(FAKE, FAKE) == 5                      # O aliases q
    assert call(FAKE, far, w=None) == 8
    assert call(FAKE, far, wb=need - 1) == 8
    assert L.seka_decode_workspace_bytes(ctypes.byref(_shape(B, Hq=5))) == 0


def test_learn_rejects_bad_arguments(B):
    L = B.lib
    ok = _shape(B)
    need = L.seka_learn_workspace_bytes(ctypes.byref(ok))
    assert need > 0 and need % 16 == 0
    big = 1 << 32                                     # far apart: no two fake ranges overlap
    hn, hs, U, sg, k, ws = (FAKE + i * big for i in range(6))

    def call(hn=hn, hs=hs, sh=ok, gamma=0.9, U=U, sg=sg, k=k, Up=None, r_pad=0, ws=ws, wb=need):
        return L.seka_learn_projection(hn, hs, ctypes.byref(sh), gamma, U, sg, k, Up, r_pad, ws, wb, None)
    assert call(hn=None) == 1
    assert call(k=None) == 1
    assert call(gamma=0.0) == 2
    assert call(gamma=1.5) == 2
    assert call(gamma=float("nan")) == 2
    assert call(sh=_shape(B, D=96)) == 2
    assert call(Up=FAKE + 7 * big, r_pad=0) == 2
    assert call(Up=FAKE + 7 * big, r_pad=129) == 2
    assert call(U=U + 4) == 4
    assert call(k=k + 2) == 4
    assert call(U=hn) == 5                            # an output over an input
    assert call(sg=U) == 5                            # two outputs over each other
    assert call(ws=None) == 8
    assert call(wb=need - 1) == 8
    hd = lambda hp=hn, hm=hs, out=U, sh=ok, w=ws, wb=need: L.seka_head_distance(hp, hm, ctypes.byref(sh), out, w, wb, None)
    assert hd(hp=None) == 1
    assert hd(out=None) == 1
    assert hd(out=U + 2) == 4
    assert hd(out=hn) == 5
    assert hd(w=None) == 8
    assert hd(wb=15) == 8
    assert hd(sh=_shape(B, dtype=7)) == 3


def test_packed_rejects_bad_arguments(B):
    L = B.lib
    L.seka_attention_prefill_packed.argtypes = [ctypes.c_void_p] * 5 + [ctypes.POINTER(B.seka_shape), ctypes.POINTER(B.seka_steer),
                                                ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    ok = _shape(B)
    big = 1 << 32
    q, k, v, o, cu = (FAKE + i * big for i in range(5))
    call = lambda cu=cu, total=300, sh=ok, o=o: L.seka_attention_prefill_packed(q, k, v, o, None, ctypes.byref(sh), None, cu, total, None)
    assert call(cu=None) == 1
    assert call(cu=cu + 2) == 4
    assert call(total=0) == 2
    assert call(total=1 << 31) == 2
    assert call(sh=_shape(B, Hq=5)) == 2
    assert call(o=q) == 5


def test_batch_sizes_beyond_a_grid_axis_are_rejected(B):
    """The routing, edit and decode launches carry the batch on a grid axis limited to 65535 workgroups: larger
    batches are a shape error on the host, not a failed launch."""
    L = B.lib
    big = B.seka_shape(70000, 16, 4, 1, 64, B.SEKA_F32, 0.0)
    assert L.seka_route(FAKE, ctypes.byref(big), FAKE * 2, 2, 0, 16, 0, 10.0, FAKE * 3, FAKE * 4, 1 << 40, None) == 2
    assert L.seka_route(FAKE, ctypes.byref(B.seka_shape(40000, 16, 4, 2, 64, B.SEKA_F32, 0.0)), FAKE * 2, 2, 0, 16, 0, 10.0,
                        FAKE * 3, FAKE * 4, 1 << 40, None) == 2          # B * Hkv counts
    st = _steer(B, Hkv=1)
    assert L.seka_edit_keys(FAKE, FAKE * 1000, ctypes.byref(big), ctypes.byref(st), None) == 2
    assert L.seka_attention_decode(FAKE, FAKE * 4, FAKE * 8, FAKE * 64, None, None, ctypes.byref(big), FAKE * 128,
                                   1 << 40, None) == 2

"""ctypes binding of libseka (the C ABI declared in include/seka.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
PyTorch tensors are used as device buffers (data_ptr) and for the current HIP stream.
Importing this module raises if the shared library has not been built
(`python -m paper_2603_01281_amd.build`); there is no CPU fallback.
"""
import ctypes
import os

# PyTorch ships its own HIP runtime (same soname as the system one).  Loading it first makes the
# library below share that runtime, so device pointers and stream handles mean the same thing to
# both; the other order leaves this process with a runtime that reports no device to our launches.
import torch  # noqa: F401  (must precede the CDLL call)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libseka.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_01281_amd.build`")

lib = ctypes.CDLL(LIB_PATH)

SEKA_OK = 0
SEKA_F32, SEKA_BF16 = 0, 1
SEKA_ROUTE_SOFTMAX_COS, SEKA_ROUTE_PAPER_EQ6 = 0, 1
SEKA_MAX_RANK, SEKA_MAX_KV_HEADS, SEKA_MAX_EXPERTS = 128, 64, 16


class seka_shape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("S", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("D", ctypes.c_int32), ("dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float)]


class seka_steer(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int32), ("r", ctypes.c_int32), ("U", ctypes.c_void_p), ("w", ctypes.c_void_p),
                ("gain", ctypes.POINTER(ctypes.c_float)), ("mask", ctypes.c_void_p),
                ("key_scale", ctypes.POINTER(ctypes.c_float))]


_vp, _i32, _f32, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
_shape_p, _steer_p = ctypes.POINTER(seka_shape), ctypes.POINTER(seka_steer)

lib.seka_status_string.restype = ctypes.c_char_p
lib.seka_status_string.argtypes = [_i32]
lib.seka_last_launch_error.restype = ctypes.c_char_p
lib.seka_last_launch_error.argtypes = []
lib.seka_route_workspace_bytes.restype = _sz
lib.seka_route_workspace_bytes.argtypes = [_shape_p, _i32, _i32]
lib.seka_route.restype = _i32
lib.seka_route.argtypes = [_vp, _shape_p, _vp, _i32, _i32, _i32, _i32, _f32, _vp, _vp, _sz, _vp]
lib.seka_project_route_workspace_bytes.restype = _sz
lib.seka_project_route_workspace_bytes.argtypes = [_shape_p]
lib.seka_project_route.restype = _i32
lib.seka_project_route.argtypes = [_vp, _vp, _i32, _vp, _shape_p, _vp, _i32, _i32, _f32, _vp, _vp, _sz, _vp]
lib.seka_edit_keys_packed.restype = _i32
lib.seka_edit_keys_packed.argtypes = [_vp, _vp, _shape_p, _steer_p, _vp, ctypes.c_int64, _vp]
lib.seka_route_ragged_workspace_bytes.restype = _sz
lib.seka_route_ragged_workspace_bytes.argtypes = [_shape_p, _i32]
lib.seka_route_ragged.restype = _i32
lib.seka_route_ragged.argtypes = [_vp, _shape_p, _vp, _i32, _vp, _vp, ctypes.c_int64, _i32, _i32, _f32, _vp, _vp, _sz, _vp]
lib.seka_edit_keys.restype = _i32
lib.seka_edit_keys.argtypes = [_vp, _vp, _shape_p, _steer_p, _vp]
lib.seka_attention_prefill.restype = _i32
lib.seka_attention_prefill.argtypes = [_vp, _vp, _vp, _vp, _vp, _shape_p, _steer_p, _vp]
lib.seka_decode_workspace_bytes.restype = _sz
lib.seka_decode_workspace_bytes.argtypes = [_shape_p]
lib.seka_attention_decode.restype = _i32
lib.seka_attention_decode.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _shape_p, _vp, _sz, _vp]
lib.seka_attention_decode_static.restype = _i32
lib.seka_attention_decode_static.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _shape_p, _vp]
lib.seka_attention_prefill_ragged.restype = _i32
lib.seka_attention_prefill_ragged.argtypes = [_vp, _vp, _vp, _vp, _vp, _shape_p, _steer_p, _vp, _vp]
lib.seka_learn_workspace_bytes.restype = _sz
lib.seka_learn_workspace_bytes.argtypes = [_shape_p]
lib.seka_learn_projection.restype = _i32
lib.seka_learn_projection.argtypes = [_vp, _vp, _shape_p, _f32, _vp, _vp, _vp, _vp, _i32, _vp, _sz, _vp]
lib.seka_head_distance.restype = _i32
lib.seka_head_distance.argtypes = [_vp, _vp, _shape_p, _vp, _vp, _sz, _vp]
lib.seka_attention_prefill_packed.restype = _i32
lib.seka_attention_prefill_packed.argtypes = [_vp, _vp, _vp, _vp, _vp, _shape_p, _steer_p, _vp, ctypes.c_int64, _vp]
lib.seka_attention_plain.restype = _i32
lib.seka_attention_plain.argtypes = [_vp, _vp, _vp, _vp, _vp, _shape_p, _vp]


class SekaError(RuntimeError):
    def __init__(self, status):
        self.status = status
        detail = f" ({lib.seka_last_launch_error().decode()})" if status == 7 else ""
        super().__init__(f"seka status {status}: {lib.seka_status_string(status).decode()}{detail}")


def _check(status):
    if status != SEKA_OK:
        raise SekaError(status)


def _torch():
    return torch


def _dtype_code(t):
    torch = _torch()
    if t.dtype == torch.float32:
        return SEKA_F32
    if t.dtype == torch.bfloat16:
        return SEKA_BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _dev(t, name):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous tensor in device memory")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return _torch().cuda.current_stream().cuda_stream
    return stream


def _shape(B, S, Hq, Hkv, D, dtype, scale):
    return seka_shape(B, S, Hq, Hkv, D, dtype, float(scale))


def _steer(U, gain, mask, w, Hkv, key_scale=None, tokens=None, D=None, dtype=None, B=None):
    """U [Hkv,M,D,r] device tensor; gain: host sequence of Hkv floats; mask [B,S] (or [total]) uint8 device; w [B,Hkv,M]
    fp32 device or None; key_scale: host sequence of Hkv floats or None (all ones).  tokens: the number of mask
    bytes the call will index; D, dtype, B: what U, mask and w must agree with."""
    torch = _torch()
    if U.dim() != 4:
        raise ValueError("U must be [Hkv, M, D, r]")
    if U.shape[0] != Hkv or (D is not None and U.shape[2] != D):
        raise ValueError(f"U is {tuple(U.shape)}, expected [Hkv={Hkv}, M, D={D}, r]")
    if dtype is not None and U.dtype != dtype:
        raise TypeError(f"U must have the tensors' dtype {dtype}, got {U.dtype}")
    if mask is None or mask.dtype != torch.uint8:
        raise TypeError("mask must be a uint8 tensor")
    if tokens is not None and mask.numel() != tokens:
        raise ValueError(f"mask has {mask.numel()} entries, expected one per token ({tokens})")
    if len(gain) != Hkv or (key_scale is not None and len(key_scale) != Hkv):
        raise ValueError(f"gain / key_scale must have one entry per KV head ({Hkv})")
    if w is not None:
        if w.dtype != torch.float32 or w.dim() != 3 or w.shape[1] != Hkv or w.shape[2] != U.shape[1] or \
                (B is not None and w.shape[0] != B):
            raise ValueError(f"w must be fp32 [B={B}, Hkv={Hkv}, M={U.shape[1]}], got {w.dtype} {tuple(w.shape)}")
    gains = (ctypes.c_float * Hkv)(*[float(g) for g in gain])
    scales = None
    if key_scale is not None:
        scales = (ctypes.c_float * Hkv)(*[float(a) for a in key_scale])
    st = seka_steer(int(U.shape[1]), int(U.shape[3]), _dev(U, "U"), _dev(w, "w"), gains, _dev(mask, "mask"), scales)
    st._keepalive = (gains, scales)
    return st


def seka_route_workspace_bytes(B, S, Hq, Hkv, D, dtype, t0, t1):
    sh = _shape(B, S, Hq, Hkv, D, dtype, 0.0)
    return lib.seka_route_workspace_bytes(ctypes.byref(sh), t0, t1)


def seka_route(Q, proto, t0, t1, mode=SEKA_ROUTE_SOFTMAX_COS, tau=10.0, w_out=None, workspace=None, stream=None):
    """Q [B,S,Hq,D] (fp32|bf16), proto [Hkv,M,D] fp32 -> w_out [B,Hkv,M] fp32 (allocated if None)."""
    torch = _torch()
    B, S, Hq, D = Q.shape
    Hkv, M, _ = proto.shape
    sh = _shape(B, S, Hq, Hkv, D, _dtype_code(Q), 0.0)
    if w_out is None:
        w_out = torch.empty((B, Hkv, M), dtype=torch.float32, device=Q.device)
    need = lib.seka_route_workspace_bytes(ctypes.byref(sh), t0, t1)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=Q.device)
    _check(lib.seka_route(_dev(Q, "Q"), ctypes.byref(sh), _dev(proto, "proto"), M, t0, t1, mode, float(tau),
                          _dev(w_out, "w_out"), _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                          _stream(stream)))
    return w_out


def seka_route_ragged(Q, proto, window, seq_lens=None, cu_seqlens=None, max_len=None, mode=SEKA_ROUTE_SOFTMAX_COS,
                      tau=10.0, w_out=None, workspace=None, stream=None):
    """Per-prompt routing over the last `window` tokens of each prompt.  Padded: Q [B,S,Hq,D] with seq_lens [B]
    int32 device tensor.  Packed: Q [total,Hq,D] with cu_seqlens [B+1] int32 device tensor and max_len."""
    torch = _torch()
    Hkv, M, _ = proto.shape
    if cu_seqlens is not None:
        total, Hq, D = Q.shape
        B, S = cu_seqlens.numel() - 1, int(max_len)
    else:
        B, S, Hq, D = Q.shape
        total = 0
    sh = _shape(B, S, Hq, Hkv, D, _dtype_code(Q), 0.0)
    if w_out is None:
        w_out = torch.empty((B, Hkv, M), dtype=torch.float32, device=Q.device)
    need = lib.seka_route_ragged_workspace_bytes(ctypes.byref(sh), window)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=Q.device)
    _check(lib.seka_route_ragged(_dev(Q, "Q"), ctypes.byref(sh), _dev(proto, "proto"), M, _dev(seq_lens, "seq_lens"),
                                 _dev(cu_seqlens, "cu_seqlens"), total, window, mode, float(tau), _dev(w_out, "w_out"),
                                 _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                                 _stream(stream)))
    return w_out


def seka_project_route_workspace_bytes(B, S, Hq, Hkv, D, dtype):
    sh = _shape(B, S, Hq, Hkv, D, dtype, 0.0)
    return lib.seka_project_route_workspace_bytes(ctypes.byref(sh))


def seka_project_route(X, Wq, Q_out, Hkv, proto=None, mode=SEKA_ROUTE_SOFTMAX_COS, tau=10.0, w_out=None,
                       workspace=None, stream=None):
    """X [B,S,E] bf16, Wq [Hq*D,E] bf16 -> Q_out [B,S,Hq,D] bf16 and, with proto [Hkv,M,D], the routing weights
    w_out [B,Hkv,M] of the whole prompt (allocated if None).  Returns w_out (None without proto)."""
    torch = _torch()
    B, S, Hq, D = Q_out.shape
    E = X.shape[2]
    sh = _shape(B, S, Hq, Hkv, D, _dtype_code(Q_out), 0.0)
    M = 0
    if proto is not None:
        M = proto.shape[1]
        if w_out is None:
            w_out = torch.empty((B, Hkv, M), dtype=torch.float32, device=X.device)
        if workspace is None:
            workspace = torch.empty(max(lib.seka_project_route_workspace_bytes(ctypes.byref(sh)), 16), dtype=torch.uint8, device=X.device)
    else:
        w_out = None
    nbytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.seka_project_route(_dev(X, "X"), _dev(Wq, "Wq"), E, _dev(Q_out, "Q_out"), ctypes.byref(sh), _dev(proto, "proto"),
                                  M, mode, float(tau), _dev(w_out, "w_out"), _dev(workspace, "workspace"), nbytes, _stream(stream)))
    return w_out


def seka_edit_keys(K_in, K_out, U, gain, mask, w=None, stream=None, key_scale=None):
    """K_in/K_out [B,S,Hkv,D]; K_out may be K_in itself (in place)."""
    B, S, Hkv, D = K_in.shape
    sh = _shape(B, S, Hkv, Hkv, D, _dtype_code(K_in), 0.0)
    st = _steer(U, gain, mask, w, Hkv, key_scale, tokens=B * S, D=D, dtype=K_in.dtype, B=B)
    _check(lib.seka_edit_keys(_dev(K_in, "K_in"), _dev(K_out, "K_out"), ctypes.byref(sh), ctypes.byref(st), _stream(stream)))
    return K_out


def seka_edit_keys_packed(K_in, K_out, cu_seqlens, max_len, U, gain, mask, w=None, stream=None, key_scale=None):
    """Unpadded batch: K_in/K_out [total,Hkv,D], mask [total], w [B,Hkv,M]; cu_seqlens [B+1] int32 device tensor."""
    total, Hkv, D = K_in.shape
    B = cu_seqlens.numel() - 1
    sh = _shape(B, max_len, Hkv, Hkv, D, _dtype_code(K_in), 0.0)
    st = _steer(U, gain, mask, w, Hkv, key_scale, tokens=total, D=D, dtype=K_in.dtype, B=B)
    _check(lib.seka_edit_keys_packed(_dev(K_in, "K_in"), _dev(K_out, "K_out"), ctypes.byref(sh), ctypes.byref(st),
                                     _dev(cu_seqlens, "cu_seqlens"), total, _stream(stream)))
    return K_out


def seka_attention_prefill(Q, K, V, O, U, gain, mask, w=None, lse=None, scale=0.0, stream=None, key_scale=None):
    B, S, Hq, D = Q.shape
    Hkv = K.shape[2]
    sh = _shape(B, S, Hq, Hkv, D, _dtype_code(Q), scale)
    st = _steer(U, gain, mask, w, Hkv, key_scale, tokens=B * S, D=D, dtype=Q.dtype, B=B)
    _check(lib.seka_attention_prefill(_dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"), _dev(O, "O"), _dev(lse, "lse"),
                                      ctypes.byref(sh), ctypes.byref(st), _stream(stream)))
    return O


def seka_attention_plain(Q, K, V, O, lse=None, scale=0.0, stream=None):
    B, S, Hq, D = Q.shape
    Hkv = K.shape[2]
    sh = _shape(B, S, Hq, Hkv, D, _dtype_code(Q), scale)
    _check(lib.seka_attention_plain(_dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"), _dev(O, "O"), _dev(lse, "lse"),
                                    ctypes.byref(sh), _stream(stream)))
    return O


def seka_learn_workspace_bytes(B, S, Hkv, D, dtype):
    sh = _shape(B, S, Hkv, Hkv, D, dtype, 0.0)
    return lib.seka_learn_workspace_bytes(ctypes.byref(sh))


def seka_decode_workspace_bytes(B, S, Hq, Hkv, D, dtype):
    sh = _shape(B, S, Hq, Hkv, D, dtype, 0.0)
    return lib.seka_decode_workspace_bytes(ctypes.byref(sh))


def seka_attention_decode(q, K, V, O, seq_lens=None, lse=None, scale=0.0, workspace=None, stream=None):
    """q/O [B,Hq,D]; K/V [B,S,Hkv,D] caches; seq_lens [B] int32 device tensor or None."""
    torch = _torch()
    B, Hq, D = q.shape
    S, Hkv = K.shape[1], K.shape[2]
    sh = _shape(B, S, Hq, Hkv, D, _dtype_code(q), scale)
    need = lib.seka_decode_workspace_bytes(ctypes.byref(sh))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    _check(lib.seka_attention_decode(_dev(q, "q"), _dev(K, "K"), _dev(V, "V"), _dev(O, "O"), _dev(lse, "lse"),
                                     _dev(seq_lens, "seq_lens"), ctypes.byref(sh), _dev(workspace, "workspace"),
                                     workspace.numel() * workspace.element_size(), _stream(stream)))
    return O


SEKA_DECODE_STATIC_MAX_BYTES = 8 << 20


def seka_attention_decode_static(q, K, V, O, seq_lens=None, lse=None, scale=0.0, stream=None):
    """seka_attention_decode on the library-owned partial-state buffer: no workspace, no allocation."""
    B, Hq, D = q.shape
    S, Hkv = K.shape[1], K.shape[2]
    sh = _shape(B, S, Hq, Hkv, D, _dtype_code(q), scale)
    _check(lib.seka_attention_decode_static(_dev(q, "q"), _dev(K, "K"), _dev(V, "V"), _dev(O, "O"), _dev(lse, "lse"),
                                            _dev(seq_lens, "seq_lens"), ctypes.byref(sh), _stream(stream)))
    return O


def seka_attention_prefill_ragged(Q, K, V, O, seq_lens, U=None, gain=None, mask=None, w=None, lse=None, scale=0.0,
                                  stream=None, key_scale=None):
    """Padded batch: seq_lens [B] int32 device tensor; U/gain/mask None for unsteered attention."""
    B, S, Hq, D = Q.shape
    Hkv = K.shape[2]
    sh = _shape(B, S, Hq, Hkv, D, _dtype_code(Q), scale)
    st = ctypes.byref(_steer(U, gain, mask, w, Hkv, key_scale, tokens=B * S, D=D, dtype=Q.dtype, B=B)) if U is not None else None
    _check(lib.seka_attention_prefill_ragged(_dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"), _dev(O, "O"), _dev(lse, "lse"),
                                             ctypes.byref(sh), st, _dev(seq_lens, "seq_lens"), _stream(stream)))
    return O


def seka_learn_projection(h_neutral, h_signal, gamma, U_out, sigma_out, k_out, U_packed=None, workspace=None,
                          stream=None):
    """h_* [B,S,Hkv,D]; U_out [Hkv,D,D] fp32, sigma_out [Hkv,D] fp32, k_out [Hkv] int32; U_packed [Hkv,D,r_pad]."""
    torch = _torch()
    B, S, Hkv, D = h_neutral.shape
    sh = _shape(B, S, Hkv, Hkv, D, _dtype_code(h_neutral), 0.0)
    need = lib.seka_learn_workspace_bytes(ctypes.byref(sh))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=h_neutral.device)
    r_pad = U_packed.shape[2] if U_packed is not None else 0
    _check(lib.seka_learn_projection(_dev(h_neutral, "h_neutral"), _dev(h_signal, "h_signal"), ctypes.byref(sh),
                                     float(gamma), _dev(U_out, "U_out"), _dev(sigma_out, "sigma_out"),
                                     _dev(k_out, "k_out"), _dev(U_packed, "U_packed"), r_pad,
                                     _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                                     _stream(stream)))
    return U_out, sigma_out, k_out


def seka_head_distance(h_pos, h_neg, D_out, workspace=None, stream=None):
    """h_* [B,S,Hkv,D]; D_out [Hkv] fp32."""
    torch = _torch()
    B, S, Hkv, D = h_pos.shape
    sh = _shape(B, S, Hkv, Hkv, D, _dtype_code(h_pos), 0.0)
    if workspace is None:
        workspace = torch.empty(max(lib.seka_learn_workspace_bytes(ctypes.byref(sh)), 16), dtype=torch.uint8,
                                device=h_pos.device)
    _check(lib.seka_head_distance(_dev(h_pos, "h_pos"), _dev(h_neg, "h_neg"), ctypes.byref(sh), _dev(D_out, "D_out"),
                                  _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                                  _stream(stream)))
    return D_out


def seka_attention_prefill_packed(Q, K, V, O, cu_seqlens, max_len, U=None, gain=None, mask=None, w=None, lse=None,
                                  scale=0.0, stream=None, key_scale=None):
    """Unpadded batch: Q/O [total,Hq,D], K/V [total,Hkv,D], mask [total], lse [Hq,total]; cu_seqlens [B+1] int32
    device tensor; max_len >= the longest prompt.  U/gain/mask None for unsteered attention."""
    total, Hq, D = Q.shape
    Hkv = K.shape[1]
    B = cu_seqlens.numel() - 1
    sh = _shape(B, max_len, Hq, Hkv, D, _dtype_code(Q), scale)
    st = ctypes.byref(_steer(U, gain, mask, w, Hkv, key_scale, tokens=total, D=D, dtype=Q.dtype, B=B)) if U is not None else None
    _check(lib.seka_attention_prefill_packed(_dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"), _dev(O, "O"), _dev(lse, "lse"),
                                             ctypes.byref(sh), st, _dev(cu_seqlens, "cu_seqlens"), total,
                                             _stream(stream)))
    return O

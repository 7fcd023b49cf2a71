"""Seeded synthetic inputs for the SEKA prefill path (shared by tests, bench and smoke).

This module holds none of the method's arithmetic: it only draws random
tensors of the benchmark shapes, rounds them to the storage dtype and draws
highlight spans.  Random numbers come from numpy's counter-based Philox
generator, keyed by (seed, stream id), so every tensor is reproducible on its own.

The workloads stand in for the paper's real prompts (Sec. 5 and Sec. 6 measure on
~4.4k-token retrieval prompts with a few contiguous highlighted passages):
Llama-3-8B- and Qwen2.5-7B-shaped heads, N(0,1) activations, a few contiguous
highlighted spans, orthonormal subspace bases from the QR of a Gaussian matrix.
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

# ----------------------------------------------------------------------------
# bf16 storage helpers (bit patterns in uint16; round-to-nearest-even)
# ----------------------------------------------------------------------------


def f32_to_bf16_bits(x):
    """Round float32 values to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + rounding) >> 16).astype(np.uint16)


def bf16_bits_to_f32(bits):
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32)


def _rng(seed, stream):
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream)]))


# stream ids, one per tensor kind (layer index is added in the upper bits)
_STREAM = {"Q": 1, "K": 2, "V": 3, "U": 4, "mask": 5, "proto": 6, "gain": 7, "sigma": 8, "svd": 9, "samples": 10}


def _stream(kind, layer=0):
    return _STREAM[kind] + 1000 * layer


@dataclass
class SekaInputs:
    """One layer's worth of inputs.  Q/K/V/U are in storage form:
    float32 arrays for dtype 'f32', uint16 bf16 bit patterns for dtype 'bf16'."""
    name: str
    dtype: str
    B: int
    S: int
    Hq: int
    Hkv: int
    D: int
    M: int
    r: int
    scale: float
    Q: np.ndarray
    K: np.ndarray
    V: np.ndarray
    U: np.ndarray                 # [Hkv, M, D, r]
    gain: np.ndarray              # [Hkv] float32 (host side)
    mask: np.ndarray              # [B, S] uint8
    proto: Optional[np.ndarray] = None   # [Hkv, M, D] float32, unit rows (AdaSEKA)
    tau: float = 10.0
    spans: list = field(default_factory=list)   # per batch entry: list of (start, length)

    def widen(self, x):
        """Storage form -> float64 (exact)."""
        if self.dtype == "bf16":
            return bf16_bits_to_f32(x).astype(np.float64)
        return np.asarray(x, dtype=np.float64)

    @property
    def G(self):
        return self.Hq // self.Hkv


def _store(x32, dtype):
    if dtype == "bf16":
        return f32_to_bf16_bits(x32)
    return np.ascontiguousarray(x32, dtype=np.float32)


def gaussian(shape, seed, kind, dtype, layer=0, mult=1.0):
    x = _rng(seed, _stream(kind, layer)).standard_normal(size=shape, dtype=np.float32)
    if mult != 1.0:
        x *= np.float32(mult)
    return _store(x, dtype)


def orthonormal_bases(Hkv, M, D, r, seed, dtype, layer=0):
    """U[Hkv, M, D, r]: Q factor of the QR of a D x r Gaussian (sign-fixed so diag(R) > 0),
    computed in float64 and then rounded to the storage dtype."""
    g = _rng(seed, _stream("U", layer))
    U = np.empty((Hkv, M, D, r), dtype=np.float64)
    for h in range(Hkv):
        for m in range(M):
            A = g.standard_normal(size=(D, r))
            Qf, Rf = np.linalg.qr(A)
            U[h, m] = Qf * np.sign(np.diag(Rf))[None, :]
    return _store(U.astype(np.float32), dtype)


def singular_vector_sets(Hkv, D, seed, layer=0):
    """Stand-ins for the left singular vectors of the two cross-covariance matrices of one layer
    (paper Sec. 3.1): two independent D x D orthogonal matrices per KV head, float64."""
    g = _rng(seed, _stream("svd", layer))
    out = np.empty((2, Hkv, D, D), dtype=np.float64)
    for s in range(2):
        for h in range(Hkv):
            Qf, Rf = np.linalg.qr(g.standard_normal(size=(D, D)))
            out[s, h] = Qf * np.sign(np.diag(Rf))[None, :]
    return out[0], out[1]


def store(x, dtype):
    """float array -> storage form of `dtype` ("f32": float32, "bf16": uint16 bit patterns, round to nearest even)."""
    return _store(np.asarray(x, dtype=np.float32), dtype)


def paired_key_samples(n, Hkv, D, seed, dtype, rank=12, decay=0.8, noise=0.05, shift=0.5, layer=0):
    """Stand-ins for the key embeddings of n sample tokens under two contexts (paper Sec. 3.1: the same
    tokens seen with a neutral and with a relevant prompt).  Per KV head a `rank`-dimensional latent code z_t
    drives both views through two different orthonormal frames, component i scaled by decay**i, so the
    cross-covariance has `rank` well separated leading singular values over a noise floor; the second view
    also carries a constant offset (the context's mean shift).  Returns (h_a, h_b), storage form, [n, Hkv, D]."""
    g = _rng(seed, _stream("samples", layer))
    z = g.standard_normal(size=(n, Hkv, rank))
    amp = 2.0 * decay ** np.arange(rank)
    fa = np.empty((Hkv, D, rank))
    fb = np.empty((Hkv, D, rank))
    for h in range(Hkv):
        fa[h] = np.linalg.qr(g.standard_normal(size=(D, rank)))[0]
        fb[h] = np.linalg.qr(g.standard_normal(size=(D, rank)))[0]
    ha = np.einsum("nhk,hdk->nhd", z * amp, fa) + noise * g.standard_normal(size=(n, Hkv, D))
    hb = np.einsum("nhk,hdk->nhd", z, fb) + noise * g.standard_normal(size=(n, Hkv, D))
    hb += shift * g.standard_normal(size=(1, Hkv, D)) / np.sqrt(D)
    return _store(ha.astype(np.float32), dtype), _store(hb.astype(np.float32), dtype)


def unit_prototypes(Hkv, M, D, seed, layer=0):
    p = _rng(seed, _stream("proto", layer)).standard_normal(size=(Hkv, M, D))
    p /= np.linalg.norm(p, axis=-1, keepdims=True)
    return np.ascontiguousarray(p, dtype=np.float32)


def draw_spans(S, lengths, g):
    """Non-overlapping span starts by rejection; spans are not aligned to any tile size."""
    placed = []
    for L in lengths:
        L = int(min(L, S))
        for _ in range(10000):
            s = int(g.integers(0, S - L + 1))
            if all(s + L <= a or a + La <= s for a, La in placed):
                placed.append((s, L))
                break
        else:
            raise RuntimeError("could not place span")
    return sorted(placed)


def split_total(total, parts, g):
    """Split `total` tokens into `parts` positive span lengths."""
    total = max(int(total), parts)
    cuts = np.sort(g.choice(np.arange(1, total), size=parts - 1, replace=False)) if parts > 1 else np.array([], int)
    edges = np.concatenate([[0], cuts, [total]])
    return [int(x) for x in np.diff(edges)]


def span_mask(B, S, seed, recipe, layer=0):
    """recipe: ('fixed', start, length) | ('cover', lo, hi, nspans) | ('lengths', n, lo, hi) | ('none',) | ('all',)"""
    mask = np.zeros((B, S), dtype=np.uint8)
    spans = []
    for b in range(B):
        g = _rng(seed, _stream("mask", layer) + 100000 * (b + 1))
        kind = recipe[0]
        if kind == "fixed":
            sp = [(recipe[1], recipe[2])]
        elif kind == "cover":
            _, lo, hi, n = recipe
            frac = lo if lo == hi else float(g.uniform(lo, hi))
            sp = draw_spans(S, split_total(round(frac * S), n, g), g)
        elif kind == "lengths":
            _, n, lo, hi = recipe
            sp = draw_spans(S, [int(x) for x in g.integers(lo, hi + 1, size=n)], g)
        elif kind == "none":
            sp = []
        elif kind == "all":
            sp = [(0, S)]
        else:
            raise ValueError(kind)
        for s, L in sp:
            mask[b, s:s + L] = 1
        spans.append(sp)
    return mask, spans


def make_layer(name, dtype, B, S, Hq, Hkv, D, M, r, gain, mask_recipe, seed=0, layer=0,
               qkv_mult=1.0, with_proto=False, tau=10.0, scale=None):
    """Draw one layer of inputs.  `gain` is a float (all heads) or a per-head sequence."""
    Q = gaussian((B, S, Hq, D), seed, "Q", dtype, layer, qkv_mult)
    K = gaussian((B, S, Hkv, D), seed, "K", dtype, layer, qkv_mult)
    V = gaussian((B, S, Hkv, D), seed, "V", dtype, layer, qkv_mult)
    U = orthonormal_bases(Hkv, M, D, r, seed, dtype, layer)
    mask, spans = span_mask(B, S, seed, mask_recipe, layer)
    g = np.full(Hkv, gain, dtype=np.float32) if np.isscalar(gain) else np.asarray(gain, dtype=np.float32)
    proto = unit_prototypes(Hkv, M, D, seed, layer) if with_proto else None
    return SekaInputs(name=name, dtype=dtype, B=B, S=S, Hq=Hq, Hkv=Hkv, D=D, M=M, r=r,
                      scale=float(scale if scale is not None else 1.0 / np.sqrt(D)),
                      Q=Q, K=K, V=V, U=U, gain=g, mask=mask, proto=proto, tau=tau, spans=spans)


# ----------------------------------------------------------------------------
# The five benchmark configurations (shapes as the benchmark definition lists them)
# ----------------------------------------------------------------------------

CONFIG_SHAPES = {
    1: dict(dtype="f32", B=1, S=256, Hq=4, Hkv=2, D=64, M=1, r=8),
    2: dict(dtype="bf16", B=1, S=4096, Hq=32, Hkv=8, D=128, M=1, r=32),
    3: dict(dtype="bf16", B=4, S=8192, Hq=32, Hkv=8, D=128, M=1, r=32),
    4: dict(dtype="bf16", B=8, S=4096, Hq=32, Hkv=8, D=128, M=4, r=32),
    5: dict(dtype="bf16", B=1, S=32768, Hq=28, Hkv=4, D=128, M=1, r=64),
}


def layer_gains_cfg3(seed=0, layers=32, lo=0.25, hi=2.0, first=8, last=23):
    """Per-layer gain of the 32-layer stack: U[lo, hi] on layers first..last (0-indexed, inclusive), 0 elsewhere."""
    g = _rng(seed, _stream("gain")).uniform(lo, hi, size=layers)
    out = np.zeros(layers, dtype=np.float32)
    out[first:last + 1] = g[first:last + 1]
    return out


def make_config(cfg, seed=0, layer=0, **over):
    """Inputs of benchmark configuration `cfg` (1..5).  Keyword overrides (e.g. S=..., B=...)
    give reduced versions of the same recipe for parity tests the CPU oracle finishes in seconds."""
    p = dict(CONFIG_SHAPES[cfg])
    p.update({k: v for k, v in over.items() if k in p})
    extra = {k: v for k, v in over.items() if k not in p}
    S = p["S"]
    if cfg == 1:
        lo = extra.pop("span_start", S // 4)
        return make_layer("cfg1", gain=extra.pop("gain", 0.5), mask_recipe=("fixed", lo, max(1, S // 8)),
                          seed=seed, layer=layer, qkv_mult=0.125, **p, **extra)
    if cfg == 2:
        return make_layer("cfg2", gain=extra.pop("gain", 1.0), mask_recipe=extra.pop("mask_recipe", ("cover", 0.10, 0.10, 3)),
                          seed=seed, layer=layer, **p, **extra)
    if cfg == 3:
        g = extra.pop("gain", None)
        if g is None:
            g = float(layer_gains_cfg3(seed)[layer])
        return make_layer("cfg3", gain=g, mask_recipe=extra.pop("mask_recipe", ("cover", 0.05, 0.20, 4)),
                          seed=seed, layer=layer, **p, **extra)
    if cfg == 4:
        return make_layer("cfg4", gain=extra.pop("gain", 1.0), mask_recipe=extra.pop("mask_recipe", ("cover", 0.10, 0.10, 3)),
                          seed=seed, layer=layer, with_proto=True, tau=10.0, **p, **extra)
    if cfg == 5:
        hi = min(512, max(64, S // 16))
        return make_layer("cfg5", gain=extra.pop("gain", 1.5), mask_recipe=extra.pop("mask_recipe", ("lengths", 8, min(64, hi), hi)),
                          seed=seed, layer=layer, **p, **extra)
    raise ValueError(cfg)

"""Shared test plumbing: move seeded inputs to the GPU, run the oracle on the same buffers, compare."""
import numpy as np

from oracle import seka_oracle as orc

# Tolerances of the benchmark definition: bf16 inputs with fp32 accumulation, fp32 path, routing weights.
BF16_MAX, BF16_MEAN = 2e-2, 2e-3
F32_ABS = 1e-4
ROUTE_ABS = 1e-5


def to_device(x, dtype):
    """Storage-form numpy array (float32, or uint16 bf16 bit patterns) -> device tensor."""
    import torch
    if dtype == "bf16":
        return torch.from_numpy(x.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(x).cuda()


def to_f64(t):
    """Device tensor -> float64 numpy."""
    return t.detach().float().cpu().numpy().astype(np.float64)


class DeviceInputs:
    def __init__(self, inp):
        import torch
        self.inp = inp
        self.Q = to_device(inp.Q, inp.dtype)
        self.K = to_device(inp.K, inp.dtype)
        self.V = to_device(inp.V, inp.dtype)
        self.U = to_device(inp.U, inp.dtype)
        self.mask = torch.from_numpy(inp.mask).cuda()
        self.proto = torch.from_numpy(inp.proto).cuda() if inp.proto is not None else None
        self.gain = [float(g) for g in inp.gain]

    def empty_like_q(self):
        import torch
        return torch.empty_like(self.Q)

    def lse_buffer(self):
        import torch
        return torch.empty((self.inp.B, self.inp.Hq, self.inp.S), dtype=torch.float32, device="cuda")


def oracle_inputs(inp):
    """float64 views of exactly the stored (dtype-rounded) inputs."""
    return dict(Q=inp.widen(inp.Q), K=inp.widen(inp.K), V=inp.widen(inp.V), U=inp.widen(inp.U))


def assert_close_bf16(got, ref, what=""):
    d = np.abs(got - ref)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    print(f"[O bf16] {what}: max {d.max():.3g} mean {d.mean():.3g}", flush=True)
    assert d.max() <= BF16_MAX, f"{what}: max |diff| {d.max():.4g} > {BF16_MAX}"
    assert d.mean() <= BF16_MEAN, f"{what}: mean |diff| {d.mean():.4g} > {BF16_MEAN}"


# LSE = m + log(l) per query row, bf16 paths.  Error sources, per path:
#   plain / decode: scores are exact products accumulated in fp32 (~1e-6); the row sum l is formed from the
#     probabilities AFTER their rounding to bf16 (the values the PV product uses), each off by at most 2^-8
#     relative (round to nearest, 8 significant bits), so l and hence log(l) are off by at most 2^-8 = 3.9e-3,
#     reached only by a row that one key dominates; over many keys the roundings average out.
#   steered, edit on chip: on top of that, an edited key is rounded to bf16 before scoring (and its subspace
#     coordinates before the second product), so its score carries about 2^-8 |q||k'| scale / sqrt(3 D) ~ 2e-3 rms
#     (worst keys ~1e-2 for unit-variance inputs); LSE moves by the probability-weighted mean of these errors,
#     which a row with one dominant highlighted key inherits undamped.
LSE_BOUNDS = {"steered": (2e-2, 2e-3), "plain": (5e-3, 5e-4), "decode": (5e-3, 5e-4)}


def assert_lse_close_bf16(got, ref, what="", path="steered", amp=2.0, n_keys=None):
    """Steered path only: the score error of an edited key is proportional to its size, so the mean bound scales
    with the key magnification amp = |a| + |g| sum_m |w_m| of k' = a k + g P k (2 in the benchmark configurations,
    for which the bound is stated); and in prompts shorter than one key tile (n_keys < 64) most rows hold a few
    keys only and inherit their score errors undamped (the mean over rows is then about the rms score error
    itself, ~2.5e-3 at amp = 2, not its average over many keys): three times the bound."""
    mx, mean = LSE_BOUNDS[path]
    if path == "steered":
        mean *= max(1.0, amp / 2.0)
        if n_keys is not None and n_keys < 64:
            mean *= 3.0
    d = np.abs(got - ref)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    print(f"[lse {path}] {what}: max {d.max():.3g} mean {d.mean():.3g}", flush=True)
    assert d.max() <= mx, f"{what}: max |diff| {d.max():.4g} > {mx}"
    assert d.mean() <= mean, f"{what}: mean |diff| {d.mean():.4g} > {mean:.3g}"


def assert_close_f32(got, ref, what="", tol=F32_ABS):
    d = np.abs(got - ref)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    assert d.max() <= tol, f"{what}: max |diff| {d.max():.4g} > {tol}"


def assert_edit_close_bf16(got, ref, gain_abs, what=""):
    """Edited keys are stored in bf16: one rounding of the exact value (|err| <= 2^-8 |k'|) plus the
    error of the correction itself (coordinates z rounded to bf16 before the second product,
    fp32 accumulation), which is bounded by a few 1e-3 for unit-variance keys and |g| ~ 1."""
    bound = 2.0 ** -8 * np.abs(ref) + 6e-3 * max(1.0, gain_abs)
    d = np.abs(got - ref)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    worst = (d - bound).max()
    assert worst <= 0, f"{what}: edited key off by {d.max():.4g}, exceeds bound by {worst:.4g}"
    assert d.mean() <= BF16_MEAN, f"{what}: mean |diff| {d.mean():.4g}"


def sample_rows(inp, per_head=24, heads=None, seed=0):
    """(b, hq, i) rows to check at sizes where the full score matrix is too large: first and last row,
    rows around every tile boundary multiple of 64 near the ends, rows around highlighted spans, random rows."""
    g = np.random.default_rng(seed)
    rows = []
    S = inp.S
    for b in range(inp.B):
        hs = heads if heads is not None else sorted(set([0, inp.Hq - 1] + [int(x) for x in g.integers(0, inp.Hq, size=2)]))
        special = {0, 1, S - 1, S - 2, 63, 64, 65, 127, 128, 255, 256, S // 2, S - 64, S - 65}
        for (s, L) in inp.spans[b]:
            special.update({s - 1, s, s + 1, s + L - 1, s + L, s + L + 1})
        special = sorted(i for i in special if 0 <= i < S)
        for hq in hs:
            rnd = [int(x) for x in g.integers(0, S, size=per_head)]
            for i in special + rnd:
                rows.append((b, hq, i))
    return rows

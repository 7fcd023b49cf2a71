"""GPU parity of seka_project_route: the query projection with the routing sums in its epilogue."""
import numpy as np
import pytest

from oracle import seka_oracle as orc
from paper_2603_01281_amd import inputs
from tests import helpers as H

pytestmark = pytest.mark.gpu


# E / 64 slices: 3, 1 and 5 (loop ends in its tail), 2, 4 and 8 (even counts: the loop ends without a tail, as at E = 4096)
@pytest.mark.parametrize("shape", [(2, 256, 8, 2, 192), (1, 384, 4, 4, 64), (3, 128, 6, 3, 320),
                                   (1, 256, 4, 2, 128), (2, 128, 8, 2, 256), (1, 128, 4, 1, 512)])
def test_project_route(seka, shape):
    import torch
    B, S, Hq, Hkv, E = shape
    D, M = 128, 4
    print(f"project_route B={B} S={S} Hq={Hq} Hkv={Hkv} E={E}", flush=True)
    X = inputs.gaussian((B, S, 1, E), 51, "Q", "bf16")[:, :, 0].copy()            # bf16 bit patterns
    W = inputs.gaussian((Hq * D, 1, 1, E), 52, "K", "bf16", 0, 1.0 / np.sqrt(E))[:, 0, 0].copy()
    proto = inputs.unit_prototypes(Hkv, M, D, 51)
    Xd, Wd = H.to_device(X, "bf16"), H.to_device(W, "bf16")
    pd = torch.from_numpy(proto).cuda()
    Q = torch.full((B, S, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    w = seka.seka_project_route(Xd, Wd, Q, Hkv, proto=pd, mode=seka.SEKA_ROUTE_SOFTMAX_COS, tau=10.0)
    torch.cuda.synchronize()
    X64 = inputs.bf16_bits_to_f32(X).astype(np.float64)
    W64 = inputs.bf16_bits_to_f32(W).astype(np.float64)
    ref_Q = orc.project_queries(X64, W64, Hq)
    got_Q = H.to_f64(Q)
    # one bf16 rounding of the exact value plus the fp32 accumulation over E terms
    bound = 2.0 ** -8 * np.abs(ref_Q) + 1e-5 * np.sqrt(E)
    assert np.isfinite(got_Q).all() and (np.abs(got_Q - ref_Q) <= bound).all(), f"max |dQ| {np.abs(got_Q - ref_Q).max():.4g}"
    # the routing is that of the rounded queries the call produced
    ref_w = orc.route_softmax_cos(got_Q, proto, 0, S, 10.0)
    assert np.abs(H.to_f64(w) - ref_w).max() <= H.ROUTE_ABS
    w2 = seka.seka_route(Q, pd, 0, S, seka.SEKA_ROUTE_SOFTMAX_COS, 10.0)
    assert np.abs(H.to_f64(w) - H.to_f64(w2)).max() <= 1e-6
    # Eq. 6 rule through the same epilogue, and the projection alone
    a = seka.seka_project_route(Xd, Wd, Q, Hkv, proto=pd, mode=seka.SEKA_ROUTE_PAPER_EQ6, tau=0.0)
    a2 = seka.seka_route(Q, pd, 0, S, seka.SEKA_ROUTE_PAPER_EQ6, 0.0)
    assert np.abs(H.to_f64(a) - H.to_f64(a2)).max() <= 1e-6
    Q2 = torch.full_like(Q, float("nan"))
    assert seka.seka_project_route(Xd, Wd, Q2, Hkv) is None
    torch.cuda.synchronize()
    assert torch.equal(Q2, Q)

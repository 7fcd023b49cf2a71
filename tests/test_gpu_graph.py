"""The entry points only enqueue kernels on the caller's stream (no allocation, no synchronisation, no memset
nodes), so a layer's calls can be captured into a HIP graph.  Every replay is compared with the eager result, with
eager work and synchronisations between the replays."""
import numpy as np
import pytest

from paper_2603_01281_amd import inputs
from tests import helpers as H

pytestmark = pytest.mark.gpu


def test_layer_calls_replay_from_a_graph(seka):
    import torch
    inp = inputs.make_layer("graph", "bf16", B=2, S=777, Hq=8, Hkv=2, D=128, M=2, r=32, gain=1.0,
                            mask_recipe=("cover", 0.2, 0.2, 3), seed=41, with_proto=True)
    dev = H.DeviceInputs(inp)
    B, S, Hq, Hkv, D, M = inp.B, inp.S, inp.Hq, inp.Hkv, inp.D, inp.M
    O = torch.zeros_like(dev.Q)
    lse = torch.zeros((B, Hq, S), dtype=torch.float32, device="cuda")
    Kc = torch.zeros_like(dev.K)
    w = torch.zeros((B, Hkv, M), dtype=torch.float32, device="cuda")
    qd = dev.Q[:, -1].contiguous()
    Od = torch.zeros_like(qd)
    ws_route = torch.empty(max(seka.seka_route_workspace_bytes(B, S, Hq, Hkv, D, seka.SEKA_BF16, 0, S), 16), dtype=torch.uint8, device="cuda")
    ws_dec = torch.empty(max(seka.seka_decode_workspace_bytes(B, S, Hq, Hkv, D, seka.SEKA_BF16), 16), dtype=torch.uint8, device="cuda")

    def layer(stream=None):
        seka.seka_route(dev.Q, dev.proto, 0, S, seka.SEKA_ROUTE_SOFTMAX_COS, inp.tau, w_out=w, workspace=ws_route, stream=stream)
        seka.seka_attention_prefill(dev.Q, dev.K, dev.V, O, dev.U, dev.gain, dev.mask, w=w, lse=lse, scale=inp.scale, stream=stream)
        seka.seka_edit_keys(dev.K, Kc, dev.U, dev.gain, dev.mask, w=w, stream=stream)
        seka.seka_attention_decode(qd, Kc, dev.V, Od, workspace=ws_dec, stream=stream)

    layer()
    torch.cuda.synchronize()
    want = [t.clone() for t in (w, O, lse, Kc, Od)]
    assert float(O.abs().max()) > 0 and float(Od.abs().max()) > 0

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        layer(side.cuda_stream)                      # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            layer(side.cuda_stream)
    torch.cuda.synchronize()
    for replay in range(3):
        for t in (w, O, lse, Kc, Od):
            t.fill_(float(replay + 1))               # eager work between the replays: results must come from the replay
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref, name in zip((w, O, lse, Kc, Od), want, ("w", "O", "lse", "K'", "O_decode")):
            assert torch.equal(got, ref), f"replay {replay}: {name} differs from the eager result"

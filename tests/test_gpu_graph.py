"""HIP graph capture of the layer: the library enqueues only kernels on the
caller's stream (no allocation, no host copy, no memset node), so a stack of
layers can be captured once and replayed.  Every replay is checked against the
eager result, with eager work and synchronisations between replays."""
import numpy as np
import pytest
import torch

import paper_2605_14438_amd as beam
from paper_2605_14438_amd import synth

import helpers as hp

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg", [
    synth.LayerConfig("graph_decode", 9, T=8, H=2048, N=128, K=8, I=768, dtype="bf16", keep=0.3),
    synth.LayerConfig("graph_prefill", 9, T=640, H=512, N=16, K=4, I=256, dtype="bf16", keep=0.5),
], ids=lambda c: c.name)
def test_layer_stack_graph_replay_equals_eager(cfg):
    print(f"graph replay {cfg}", flush=True)
    n_layers = 3
    layers = []
    for l in range(n_layers):
        d = synth.make_layer(cfg, sweep=l)
        layers.append(hp.upload(cfg, d))
    x0 = layers[0]["x"]
    s = hp.shape_of(cfg)
    nb = beam.beam_block_workspace_bytes(s, 0)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    bufs = [torch.empty_like(x0), torch.empty_like(x0)]

    def run_stack():
        h = x0
        for l, g in enumerate(layers):
            out = bufs[l & 1]
            beam.beam_moe_block_forward(s, 0, h, g["w_router"], g["b_router"], g["w_mask"],
                                        g["b_mask"], g["w_gate_up"], g["w_down"], None, h, out,
                                        None, None, None, None, ws, nb,
                                        torch.cuda.current_stream().cuda_stream)
            h = out
        return h

    eager = run_stack().clone()
    torch.cuda.synchronize()
    assert torch.isfinite(eager.float()).all() and not torch.equal(eager, x0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        run_stack()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            h_graph = run_stack()
    torch.cuda.synchronize()
    for i in range(4):
        bufs[0].zero_()
        bufs[1].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(h_graph, eager), f"replay {i} differs from the eager result"
        again = run_stack().clone()           # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(again, eager)

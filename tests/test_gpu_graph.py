"""HIP graph capture of the layer: the library enqueues only kernels on the
caller's stream (no allocation, no host copy, no memset node), so a stack of
layers can be captured once and replayed.  Every replay is checked against the
eager result, with eager work and synchronisations between replays, and every
layer of a replayed stack against the oracle's block update (App. A.3)."""
import numpy as np
import pytest
import torch

import oracle
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


@pytest.mark.parametrize("cfg,packed", [
    (synth.LayerConfig("stack_decode", 9, T=8, H=2048, N=128, K=8, I=768, dtype="bf16", keep=0.3),
     True),
    (synth.LayerConfig("stack_decode", 9, T=2, H=2048, N=128, K=8, I=768, dtype="bf16", keep=0.5),
     False),                                   # the three-kernel path of tiny batches
    (synth.LayerConfig("stack_prefill", 9, T=640, H=512, N=16, K=4, I=256, dtype="bf16", keep=0.5),
     False),
], ids=lambda v: f"{v.name}-T{v.T}" if hasattr(v, "name") else ("packed" if v else "plain"))
def test_replayed_stack_matches_the_oracle_layer_by_layer(cfg, packed):
    """Three blocks h' = h + layer(h) (App. A.3 without a shared expert) replayed from one
    HIP graph.  Every layer's output is kept, and layer l is checked against the oracle's
    block update fed the GPU's own output of layer l-1 (so that errors do not compound
    into the comparison): indices bit for bit and the output inside the tolerance, on the
    tokens whose routing decisions under that input are outside the guard band."""
    print(f"graph stack vs oracle {cfg} packed={packed}", flush=True)
    n_layers = 3
    host, layers = [], []
    for l in range(n_layers):
        d = synth.make_layer(cfg, sweep=l)
        g = hp.upload(cfg, d)
        if packed:
            g["w_gate_up"], g["w_down"] = hp.pack_weights(cfg, g["w_gate_up"], g["w_down"])
        host.append(d)
        layers.append(g)
    x0 = layers[0]["x"]
    s = hp.shape_of(cfg, packed=packed)
    nb = beam.beam_block_workspace_bytes(s, 0)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    outs = [torch.empty_like(x0) for _ in range(n_layers)]
    T, K = cfg.T, cfg.K
    ids = [torch.empty((T, K), dtype=torch.int32, device="cuda") for _ in range(n_layers)]
    mids = [torch.empty((T, K), dtype=torch.int32, device="cuda") for _ in range(n_layers)]

    def run_stack():
        h = x0
        for l, g in enumerate(layers):
            beam.beam_moe_block_forward(s, 0, h, g["w_router"], g["b_router"], g["w_mask"],
                                        g["b_mask"], g["w_gate_up"], g["w_down"], None, h,
                                        outs[l], ids[l], None, mids[l], None, ws, nb,
                                        torch.cuda.current_stream().cuda_stream)
            h = outs[l]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        run_stack()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run_stack()
    torch.cuda.synchronize()
    for replay in range(2):
        for o in outs:
            o.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        h_in = x0.float().cpu().numpy()
        for l, d in enumerate(host):
            ref = oracle.block_forward(h_in, d["w_router"], d["b_router"], d["w_mask"],
                                       d["b_mask"], d["w_gate_up"], d["w_down"], K,
                                       residual=h_in)
            r = oracle.logits(h_in, d["w_router"], d["b_router"])
            a = oracle.logits(h_in, d["w_mask"], d["b_mask"])
            clear = oracle.decision_margin(r, a, K) >= hp.GUARD
            assert clear.mean() > 0.9
            assert np.array_equal(ids[l].cpu().numpy()[clear], ref["topk_ids"][clear])
            assert np.array_equal(mids[l].cpu().numpy()[clear], ref["masked_ids"][clear])
            got = outs[l].float().cpu().numpy().astype(np.float64)
            part = ref["out"] - h_in.astype(np.float64)          # the experts' part
            err = np.abs(got - ref["out"])[clear]
            tol = (2e-2 * np.sqrt((part[clear] ** 2).mean()) + 2.0 ** -8 * np.abs(ref["out"]))[clear]
            print(f"  replay {replay} layer {l}: {int(clear.sum())}/{T} tokens compared, "
                  f"kept pairs {int((ref['masked_ids'] >= 0).sum())}, "
                  f"worst/bound {float((err / tol).max()):.3f}", flush=True)
            assert (err <= tol).all()
            h_in = outs[l].float().cpu().numpy()                   # the GPU's own output feeds on

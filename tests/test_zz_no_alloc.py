"""The allocation-free entry point (beam_moe_forward_noalloc) against the entry point it
is a variant of (beam_moe_forward): same bits, on two calls in a row that share the
library's device array, the second with a smaller input; and both against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_14438_amd as beam
from paper_2605_14438_amd import binding, synth

import helpers as hp

pytestmark = pytest.mark.gpu


def _noalloc(cfg, g, packed):
    s = hp.shape_of(cfg, packed=packed)
    out = hp.out_tensor(cfg)
    beam.beam_moe_forward_noalloc(s, g["x"], g["w_router"], g["b_router"], g["w_mask"],
                                  g["b_mask"], g["w_gate_up"], g["w_down"], out, hp.stream_ptr())
    return out


@pytest.mark.parametrize("packed", [False, True], ids=["plain", "packed"])
def test_noalloc_equals_workspace_entry_point_twice_in_a_row(packed):
    big = synth.CONFIGS["qwen3_decode"].with_(T=200, keep=0.3)      # streaming kernels, 200 x 8 slots
    small = synth.CONFIGS["qwen3_decode"].with_(T=5, keep=0.5)      # one launch for Top-K + grouping
    outs = []
    for cfg in (big, small):                                        # the second call is the smaller one
        print(f"noalloc {cfg} packed={packed}", flush=True)
        d = hp.make_tie_free(cfg)
        g = hp.upload(cfg, d)
        if packed:
            g["w_gate_up"], g["w_down"] = hp.pack_weights(cfg, g["w_gate_up"], g["w_down"])
        out = _noalloc(cfg, g, packed)          # no synchronisation in between: stream order
        outs.append((cfg, d, g, out))
    torch.cuda.synchronize()
    for cfg, d, g, out in outs:
        res = hp.forward(cfg, g, prepacked=packed)                  # caller's workspace
        assert torch.equal(out, res["out_raw"])
        ref = oracle.moe_forward(d["x"], d["w_router"], d["b_router"], d["w_mask"], d["b_mask"],
                                 d["w_gate_up"], d["w_down"], cfg.K)
        assert np.array_equal(res["masked_ids"], ref["masked_ids"])
        literal, ratio = hp.output_error(out.float().cpu().numpy().astype(np.float64),
                                         ref["out"], cfg.dtype)
        print(f"  T={cfg.T}: max|err|/RMS={literal:.4f} worst/bound={ratio:.3f}", flush=True)
        assert ratio <= 1.0
        zero = (ref["masked_ids"] >= 0).sum(axis=1) == 0
        if zero.any():
            assert (out[torch.from_numpy(zero).cuda()].view(torch.int16) == 0).all()
    # the array keeps the last call's contents: the larger input again, after the smaller one
    cfg, d, g, first = outs[0]
    again = _noalloc(cfg, g, packed)
    torch.cuda.synchronize()
    assert torch.equal(again, first)


def test_noalloc_other_paths_and_limits():
    # fp32 generic kernels, the three-kernel path of tiny batches, a prefill-sized batch
    cases = [synth.CONFIGS["tiny"],
             synth.CONFIGS["qwen3_decode"].with_(T=2, keep=0.6),
             synth.LayerConfig("noalloc_prefill", 2, T=900, H=512, N=16, K=4, I=256, dtype="bf16",
                               keep=0.5, router_skew="zipf")]
    for cfg in cases:
        print(f"noalloc {cfg}", flush=True)
        d = hp.make_tie_free(cfg)
        g = hp.upload(cfg, d)
        out = _noalloc(cfg, g, False)
        torch.cuda.synchronize()
        res = hp.forward(cfg, g)
        assert torch.equal(out, res["out_raw"])
    # beyond the array's size: refused on the host, nothing enqueued, output untouched
    cfg = synth.CONFIGS["qwen3_decode"].with_(T=396)
    s = hp.shape_of(cfg)
    assert beam.beam_workspace_bytes(s) > binding.BEAM_NOALLOC_WORKSPACE_BYTES
    ok = 0x1000
    st = beam.beam_moe_forward_noalloc(s, ok, ok, None, ok, None, ok, ok, ok, None, check=False)
    assert st == binding.BEAM_ERR_WORKSPACE
    s395 = hp.shape_of(cfg.with_(T=395))
    assert beam.beam_workspace_bytes(s395) <= binding.BEAM_NOALLOC_WORKSPACE_BYTES

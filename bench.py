#!/usr/bin/env python3
"""Benchmark of the binary-masked MoE layer forward (beam_moe_forward) on one
MI355X.

A step is one pass of the whole hot path -- router + mask logits, Top-K,
binary mask, grouping by expert, gate/up GEMM + SiLU, down GEMM, masked
aggregation -- over one batch of synthetic tokens, inputs resident in HBM.

The headline workload is the Qwen3-30B-A3B-shaped decode layer (64 tokens,
hidden 2048, 128 experts, top-8, intermediate 768, bf16, ~15% of the Top-K
pairs kept).  Consecutive steps rotate over several copies of the expert
weights so that no step finds its weights in the 256 MB last-level cache.

Prints ONE JSON line.  `roofline` describes the dominant kernel (gate/up
GEMM): algorithmic bytes per launch / its mean duration measured with HIP
events on the launch stream (`stage_us`: event to event; `kernel_us`: the same
minus the bubble the event pairs add, see measure_point); `roofline.traffic` is the
HBM bytes per launch that rocprofv3's FETCH_SIZE / WRITE_SIZE counters read for that kernel on
that workload, carried from profiles/traffic.json while the kernel's sources are unchanged
(measured_traffic).  `cpu_baseline` is the plain CPU oracle timed on the host cores.
`points` holds the other workload points (decode batch sizes, the prefill grid, whole blocks
with shared experts, the Mixtral-shaped and the large layer) measured the same way, each
with its own `roofline`.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0   # dense bf16


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=int(os.environ.get("WORLD_SIZE", "1")))
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="qwen3_decode")
    ap.add_argument("--tokens", type=int, default=None)
    ap.add_argument("--keep", type=float, default=None)
    ap.add_argument("--weight-sets", type=int, default=4)
    ap.add_argument("--no-points", action="store_true", help="skip the extra workload points")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--packed", action="store_true",
                    help="(the default where the shape allows it) run from expert weights repacked "
                         "once, outside the timed region, by beam_pack_weights")
    ap.add_argument("--plain", action="store_true",
                    help="run from row-major expert weights instead")
    ap.add_argument("--stack-layers", type=int, default=48,
                    help="depth of the decode stack replayed under one HIP graph (0 = skip)")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MIB",
                    help="also run a plain device copy of this many MiB a few times (a kernel of "
                         "known traffic, to calibrate rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def measure_point(cfg, d, g, weight_sets, steps, warmup, torch, beam, hp, packed=False):
    """Time `steps` forwards of one workload point; returns a dict of results.
    packed: the weight sets are in matrix-core fragment order (beam_pack_weights)."""
    import numpy as np
    s = hp.shape_of(cfg, packed=packed)
    S = cfg.S     # shared-expert blocks (App. A.3 workloads): the block entry point runs
    nb = beam.beam_block_workspace_bytes(s, S)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    out = hp.out_tensor(cfg)
    mids = torch.empty((cfg.T, cfg.K + S), dtype=torch.int32, device="cuda")
    npairs = torch.zeros((1,), dtype=torch.int32, device="cuda")
    stream = hp.stream_ptr()
    nsets = len(weight_sets)
    gate, res = g.get("w_sh_gate"), g.get("residual")

    def step(i, want_ids=False):
        wgu, wd = weight_sets[i % nsets]
        beam.beam_moe_block_forward(s, S, g["x"], g["w_router"], g["b_router"], g["w_mask"],
                                    g["b_mask"], wgu, wd, gate, res, out, None, None,
                                    mids if want_ids else None, npairs if want_ids else None,
                                    ws, nb, stream)

    step(0, want_ids=True)
    torch.cuda.synchronize()
    m = mids.cpu().numpy()
    P = int(npairs.item())                     # kept routed pairs + T*S shared slots
    U = int(np.unique(m[m >= 0]).size)         # experts touched, shared blocks included
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms = elapsed * 1e3 / steps

    # per-stage durations, HIP events on the launch stream (same weight rotation)
    nprof = max(10, min(steps, 50))
    acc = [0.0] * beam.binding.BEAM_NUM_STAGES
    for i in range(nprof):
        wgu, wd = weight_sets[i % nsets]
        _, st = beam.beam_moe_block_forward_timed(s, S, g["x"], g["w_router"], g["b_router"],
                                                  g["w_mask"], g["b_mask"], wgu, wd, gate, res,
                                                  out, ws, nb, stream)
        acc = [a + b for a, b in zip(acc, st)]
    stage_us = {n: 1e3 * a / nprof for n, a in zip(beam.binding.STAGE_NAMES, acc)}
    # An event pair around a stage adds a bubble of 2-3 us that the untimed forward does not
    # have (the six stage figures add up to more than the wall clock per layer).  With one
    # kernel-bearing stage after the other the bubble is the same for each, so the kernel
    # durations are the stage figures minus a sixth of that excess; rocprofv3's kernel trace
    # of the same command agrees with the corrected figure to a fraction of a microsecond.
    # (Not applied on the three-kernel path of tiny batches, where stages are empty.)
    tiny = (cfg.T * (cfg.K + S) <= 24 and cfg.dtype == "bf16" and cfg.H % 512 == 0
            and cfg.I % 128 == 0)
    bubble = 0.0 if tiny else max(0.0, (sum(stage_us.values()) - ms * 1e3) / len(stage_us))
    kernel_us = {n: max(v - bubble, 0.0) for n, v in stage_us.items()}

    esz = 2 if cfg.dtype == "bf16" else 4
    H, I, N, T = cfg.H, cfg.I, cfg.N, cfg.T
    # algorithmic traffic: each touched expert's weights once (3*H*I elements:
    # 2I x H gate/up + H x I down), both routing heads, x in, out out
    # (a shared expert of width S*I counts as its S blocks in U and T*S pairs in P;
    # the residual is one more read of T*H)
    layer_bytes = U * 3 * H * I * esz + 2 * N * H * esz + (3 if res is not None else 2) * T * H * esz
    layer_flops = P * 6 * H * I + 4 * T * H * N
    gate_up_bytes = U * 2 * H * I * esz + T * H * esz
    gate_up_flops = P * 4 * H * I
    # down: the touched experts' H x I weights, the hidden rows in, the pair rows out
    ybytes = beam.beam_fused_pair_row_bits(s, S) // 8      # fp32, or half precision for large batches
    down_bytes = U * H * I * esz + P * I * esz + P * H * ybytes
    down_flops = P * 2 * H * I
    t_roof_us = max(layer_bytes / (HBM_PEAK_GBS * 1e3), layer_flops / (MFMA_BF16_PEAK_TFLOPS * 1e6))
    return {
        "workload": f"{cfg.name} T={T} keep={cfg.keep}", "T": T, "P": P, "U": U,
        "weights": "packed" if packed else "plain",
        "stage_algorithmic": {"gate_up": {"bytes": gate_up_bytes, "flops": gate_up_flops},
                              "down": {"bytes": down_bytes, "flops": down_flops}},
        # 6 stages; the grouping of more than 8192 pairs is 4 launches, the tiled logits GEMM repacks the
        # heads first, a gated shared expert adds one; up to 32 tokens Top-K and grouping are
        # one launch; tiny batches take the three-kernel path
        # ... and between decode and prefill size both families of expert GEMM kernels are
        # enqueued (the one the device does not choose leaves at once): two more
        "kernels_per_layer": (3 if tiny else 6 + (3 if T * (cfg.K + S) > 8192 else 0) + (
            1 if T > 512 and cfg.dtype == "bf16" and cfg.H % 256 == 0 else 0) - (
            1 if T <= 32 and T * (cfg.K + S) <= 512 and cfg.K + S <= 16 and cfg.N % 4 == 0
            else 0)) + (1 if gate is not None else 0) + (
            2 if (cfg.dtype == "bf16" and cfg.H % 512 == 0 and cfg.I % 128 == 0 and cfg.I < 4096
                  and max(512, 8 * (N + S)) < T * (cfg.K + S) <= 256 * (N + S)) else 0),
        "us_per_layer": ms * 1e3, "tokens_per_s": T / (ms * 1e-3), "stage_us": stage_us,
        "kernel_us": kernel_us,
        "layer_GBs": layer_bytes / (ms * 1e-3) / 1e9,
        "layer_TFLOPs": layer_flops / (ms * 1e-3) / 1e12,
        "frac_hbm": layer_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "frac_mfma": layer_flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "frac_of_roofline": t_roof_us / (ms * 1e3),
        "gate_up": {"bytes": gate_up_bytes, "flops": gate_up_flops, "us": kernel_us["gate_up"]},
        "ms_per_step": ms,
    }


def measure_ceilings(buf, torch, beam):
    """What this GPU delivers on the two rooflines (library probe kernels timed with
    events): a plain streaming read of `buf` and a bare bf16 MFMA loop."""
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    nbytes = buf.numel() * buf.element_size()

    def timed(fn, reps):
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    read = [0]

    def stream():
        read[0] = beam.beam_probe_stream_read(buf, nbytes, sink, st)[1]
    flops = [0.0]

    def mfma():
        flops[0] = beam.beam_probe_mfma(20000, sink, st)[1]
    t_s = timed(stream, 10)
    t_m = timed(mfma, 3)
    return {"stream_read_GBs": read[0] / t_s / 1e9, "stream_read_bytes": read[0],
            "mfma_bf16_TFLOPs": flops[0] / t_m / 1e12,
            "published": {"hbm_GBs": HBM_PEAK_GBS, "mfma_bf16_TFLOPs": MFMA_BF16_PEAK_TFLOPS}}


def measure_training_step(cfg, g, wgu, wd, packed, steps, torch, beam, hp):
    """Training mode (Sec. 3.3) at a prefill-sized batch: the forward evaluates every
    Top-K expert and applies the mask in the sum (staged entry points), then the
    mask router's straight-through backward (Eq. 9-12) with L_reg.  Times both."""
    T, K, N, H = cfg.T, cfg.K, cfg.N, cfg.H
    s = hp.shape_of(cfg, packed=packed)
    ws, nb = hp.workspace(s)
    i32 = dict(dtype=torch.int32, device="cuda")
    f32 = dict(dtype=torch.float32, device="cuda")
    ids, mids = torch.empty((T, K), **i32), torch.empty((T, K), **i32)
    gw, ml = torch.empty((T, K), **f32), torch.empty((T, N), **f32)
    counts, offsets = torch.empty((N,), **i32), torch.empty((N + 1,), **i32)
    perm, inv, P = torch.empty((T * K,), **i32), torch.empty((T * K,), **i32), torch.empty((1,), **i32)
    y = torch.empty((T * K, H), **f32)
    out = hp.out_tensor(cfg)
    dy = torch.randn((T, H), device="cuda").to(out.dtype)
    grad_a, grad_w = torch.empty((T, K), **f32), torch.empty((N, H), **f32)
    loss_reg = torch.empty((T,), **f32)
    st = hp.stream_ptr()

    def forward():
        beam.beam_route_mask(s, g["x"], g["w_router"], g["b_router"], g["w_mask"], g["b_mask"],
                             ids, gw, mids, None, ml, ws, nb, st)
        beam.beam_permute(s, ids, counts, offsets, perm, inv, P, ws, nb, st)
        beam.beam_expert_ffn(s, g["x"], wgu, wd, offsets, perm, P, y, ws, nb, st)
        beam.beam_combine(s, y, gw, mids, inv, out, st)

    def backward():
        beam.beam_mask_router_backward(s, g["x"], ids, gw, ml, y, offsets, perm, inv, dy, 1e-3,
                                       grad_a, grad_w, loss_reg, ws, nb, st)

    def timed(fn):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e6 / steps

    fwd_us = timed(forward)
    bwd_us = timed(backward)
    esz = 2 if cfg.dtype == "bf16" else 4
    # the backward reads every expert output row once (fp32), dL/dy and x per token
    # (re-read per slot from cache), and writes grad_a and grad_w_mask
    bwd_bytes = T * K * H * 4 + 2 * T * H * esz + T * K * 4 * 3 + N * H * 4
    return {"workload": f"{cfg.name} T={T} keep={cfg.keep}, all Top-K evaluated",
            "forward_us": fwd_us, "mask_router_backward_us": bwd_us,
            "backward_GBs": bwd_bytes / (bwd_us * 1e-6) / 1e9,
            "backward_frac_hbm": bwd_bytes / (bwd_us * 1e-6) / 1e9 / HBM_PEAK_GBS}


def measure_rules(cfg, g, weight_sets, steps, torch, beam, hp, packed=False):
    """The same layer under other activation rules (Sec. 4.1 baselines, Sec. 4.4
    ablation), same inputs and weights: us per layer and kept pairs per token.
    Layer time follows the experts touched, whatever rule chose them."""
    import math
    T, K = cfg.T, cfg.K
    s = hp.shape_of(cfg, packed=packed)
    ws, nb = hp.workspace(s)
    out = hp.out_tensor(cfg)
    npairs = torch.zeros((1,), dtype=torch.int32, device="cuda")
    stream = hp.stream_ptr()
    all_kept = torch.full((cfg.N,), 1.0e4, dtype=torch.float32, device="cuda")
    cases = [("mask tau=0.5 (the paper's rule)", s, (beam.BEAM_RULE_MASK, 0.0), g["b_mask"])]
    for tau in (0.3, 0.7):
        cases.append((f"mask tau={tau}", s, (beam.BEAM_RULE_MASK, math.log(tau / (1 - tau))),
                      g["b_mask"]))
    for phi in (0.02, 0.05, 0.1):
        cases.append((f"cumulative probability phi={phi}", s, (beam.BEAM_RULE_CUMPROB, phi),
                      g["b_mask"]))
    for k2 in (1, 2, K):
        cases.append((f"top-{k2} of the same router, nothing masked",
                      hp.shape_of(cfg.with_(K=k2), packed=packed),
                      (beam.BEAM_RULE_MASK, 0.0), all_kept))
    res = []
    for label, shape, rule, b_mask in cases:
        def step(i, want=False):
            wgu, wd = weight_sets[i % len(weight_sets)]
            beam.beam_moe_forward_rule(shape, rule, g["x"], g["w_router"], g["b_router"],
                                       g["w_mask"], b_mask, wgu, wd, out, None, None, None,
                                       npairs if want else None, ws, nb, stream)
        step(0, want=True)
        for i in range(5):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(i)
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) * 1e6 / steps
        res.append({"rule": label, "us_per_layer": us, "kept_pairs_per_token":
                    int(npairs.item()) / T})
    return res


def measure_decode_stack(cfg, n_layers, batches, torch, beam, hp, synth, packed=False):
    """A stack of n_layers masked-MoE blocks (h' = h + layer(h), App. A.3 without a
    shared expert) with their own weights, run for one decode step: eager launches
    against one HIP graph replay.  Keep rate per layer rises linearly with depth
    around the workload's mean (deeper layers keep more in decode, Sec. 4.4).
    Weights are drawn on the device (N(0, 0.02^2), bf16): this is a timing run; the
    per-layer arithmetic is what the parity tests cover."""
    dt = torch.bfloat16
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.seed_for(cfg, 99))

    def rnd(*shape, std=0.02):
        return (torch.randn(*shape, generator=gen, device="cuda", dtype=torch.float32) * std).to(dt)

    layers = []
    for l in range(n_layers):
        keep = cfg.keep * (0.4 + 1.2 * l / max(1, n_layers - 1))
        bm = torch.full((cfg.N,), synth.mask_bias_value(cfg.with_(keep=keep)),
                        dtype=torch.float32, device="cuda")
        layers.append((rnd(cfg.N, cfg.H), rnd(cfg.N, cfg.H), bm, rnd(cfg.N, 2 * cfg.I, cfg.H),
                       rnd(cfg.N, cfg.H, cfg.I)))
    res = []
    for T in batches:
        c = cfg.with_(T=T)
        # packed: the random arrays are read as fragment-ordered weights (a permutation of
        # i.i.d. draws is the same distribution, so no repacking pass is run on them)
        s = hp.shape_of(c, packed=packed)
        nb = beam.beam_block_workspace_bytes(s, 0)
        ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
        x0 = rnd(T, cfg.H, std=1.0)
        bufs = [torch.empty_like(x0), torch.empty_like(x0)]
        npairs = torch.zeros((n_layers,), dtype=torch.int32, device="cuda")

        def run_stack(count_pairs=False):
            h = x0
            for l, (wr, wm, bm, wgu, wd) in enumerate(layers):
                out = bufs[l & 1]
                beam.beam_moe_block_forward(s, 0, h, wr, None, wm, bm, wgu, wd, None, h, out,
                                            None, None, None,
                                            npairs[l:l + 1] if count_pairs else None, ws, nb,
                                            torch.cuda.current_stream().cuda_stream)
                h = out
            return h

        final = run_stack(count_pairs=True).clone()
        torch.cuda.synchronize()
        kept = npairs.cpu().numpy()
        reps = 10
        for _ in range(2):
            run_stack()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            run_stack()
        torch.cuda.synchronize()
        eager_us = (time.perf_counter() - t0) * 1e6 / reps
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            run_stack()
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                h_graph = run_stack()
        torch.cuda.synchronize()
        same = True
        for _ in range(3):                      # every replay must equal the eager result
            graph.replay()
            torch.cuda.synchronize()
            same = same and bool(torch.equal(h_graph, final))
            run_stack()                         # eager work between replays
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - t0) * 1e6 / reps
        res.append({"T": T, "layers": n_layers, "eager_us_per_step": eager_us,
                    "graph_us_per_step": graph_us, "graph_us_per_layer": graph_us / n_layers,
                    "tokens_per_s_graph": T / (graph_us * 1e-6),
                    "kept_pairs_per_token_first_last": [float(kept[0]) / T, float(kept[-1]) / T],
                    "kept_pairs_per_token_mean": float(kept.mean()) / T,
                    "graph_replays_equal_eager": same})
        del graph
    return res


def upload_layer(cfg, d, hp, synth):
    """Device buffers of a layer; with a shared expert its S blocks are appended
    to the expert arrays and the gate vector and residual come along."""
    g = hp.upload(cfg, d)
    if cfg.S > 0:
        gu, dn = synth.append_shared_blocks(cfg, d)
        g["w_gate_up"], g["w_down"] = hp.dev(gu, cfg.dtype), hp.dev(dn, cfg.dtype)
        g["w_sh_gate"] = hp.dev(d["w_sh_gate"], cfg.dtype)
        g["residual"] = hp.dev(d["residual"], cfg.dtype)
    return g


def device_weight_sets(cfg, nsets, torch, seed):
    """Expert weights drawn on the device (N(0, 0.02^2), bf16, seeded) for workload points
    whose multi-GB weights would take minutes to draw on the host.  Timing only: the
    routing inputs (x, heads, biases) still come from synth, so keep rate and skew are the
    workload's; read as packed weights a random array is the same distribution."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    n = cfg.N + cfg.S
    sets = []
    for _ in range(nsets):
        gu = (torch.randn(n, 2 * cfg.I, cfg.H, generator=gen, device="cuda") * 0.02).to(torch.bfloat16)
        dn = (torch.randn(n, cfg.H, cfg.I, generator=gen, device="cuda") * 0.02).to(torch.bfloat16)
        sets.append((gu, dn))
    return sets


def _sha16(paths):
    import hashlib
    h = hashlib.sha256()
    for p in paths:
        with open(os.path.join(ROOT, p), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` on `workload` from the tracked counter summary
    (profiles/traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, scaled by what the
    same counters read for a device copy of known size).  Counters cannot be read inside
    this process, so the figure is carried from that run, and only while the kernel's
    source files still hash to what they were when it was taken; otherwise None."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    for rec in json.load(open(path))["records"]:
        if rec["workload"] == workload and rec["kernel"] == kernel:
            try:
                same = _sha16(rec["source_files"]) == rec["source_sha16"]
            except OSError:
                same = False
            if same:
                return {"bytes": rec["fetch_bytes"] + rec["write_bytes"],
                        "source": f"profiles/traffic.json@{rec['commit']}"}
    return None


def roofline_of(pt):
    """Roofline record of the dominant kernel (gate/up) of a point: HBM bound
    when its byte time exceeds its flop time at the peaks, else MFMA bound."""
    gu = pt["gate_up"]
    sec = gu["us"] * 1e-6
    t_b = gu["bytes"] / (HBM_PEAK_GBS * 1e9)
    t_f = gu["flops"] / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    tr = measured_traffic(pt["workload"] + " " + pt["weights"], "gate_up")
    extra = {"traffic": tr["bytes"] if tr else None,
             "duration_us": gu["us"], "duration_kind": "HIP events around the stage, bubble-corrected"}
    if tr:
        extra["traffic_source"] = tr["source"]
        extra["traffic_over_algorithmic"] = tr["bytes"] / gu["bytes"]
    if t_b >= t_f:
        a = gu["bytes"] / sec / 1e9
        return {"bound": "hbm", "kernel": "gate_up", "achieved": a, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": a / HBM_PEAK_GBS, **extra}
    a = gu["flops"] / sec / 1e12
    return {"bound": "mfma", "kernel": "gate_up", "achieved": a, "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": a / MFMA_BF16_PEAK_TFLOPS, **extra}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the layer fits one MI355X and tokens are "
              "independent); --gpus N with N > 1 is not supported.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2605_14438_amd as beam
    from paper_2605_14438_amd import build as beam_build, runtime as hp, synth

    if not os.path.exists(beam_build.LIB):
        beam_build.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    cfg = synth.CONFIGS[args.workload]
    if args.tokens is not None:
        cfg = cfg.with_(T=args.tokens)
    if args.keep is not None:
        cfg = cfg.with_(keep=args.keep)

    t_gen = time.perf_counter()
    d = synth.make_layer(cfg)
    g = upload_layer(cfg, d, hp, synth)
    sets = [(g["w_gate_up"], g["w_down"])]
    for _ in range(max(1, args.weight_sets) - 1):
        sets.append((g["w_gate_up"].clone(), g["w_down"].clone()))
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    if args.copy_probe > 0:
        src = torch.empty(args.copy_probe << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    packed_sets = None

    def get_packed_sets():
        nonlocal packed_sets
        if packed_sets is None:
            packed_sets = [hp.pack_weights(cfg.with_(N=cfg.N + cfg.S), a, b) for a, b in sets]
            torch.cuda.synchronize()
        return packed_sets

    # Packed is the layout a server keeps its weights in (one-time repack, not part of the
    # layer): every kernel family reads it and the streaming kernels are 6-9 % faster from it.
    args.packed = (not args.plain) and cfg.dtype == "bf16" and cfg.H % 512 == 0 and cfg.I % 128 == 0
    main_sets = get_packed_sets() if args.packed else sets
    main_pt = measure_point(cfg, d, g, main_sets, args.steps, args.warmup, torch, beam, hp,
                            packed=args.packed)

    # the same point without the rotation: every step finds whatever part of its expert
    # weights fits the 256 MB last-level cache still there (reported beside, never as `value`)
    warm = None
    if not args.no_points and len(main_sets) > 1:
        wp = measure_point(cfg, d, g, main_sets[:1], max(20, args.steps // 4), 10, torch, beam, hp,
                           packed=args.packed)
        warm = {"us_per_layer": wp["us_per_layer"], "tokens_per_s": wp["tokens_per_s"],
                "weight_sets_rotated": 1,
                "note": "warm last-level cache: one copy of the expert weights, re-read every step"}

    points = []
    training = None
    if not args.no_points and args.workload == "qwen3_decode":
        psteps = max(20, args.steps // 4)
        for T in (1, 8, 32):
            c = cfg.with_(T=T)
            dd = synth.make_layer(c, with_experts=False)
            gg = {**hp.upload(c, dd), "w_gate_up": g["w_gate_up"], "w_down": g["w_down"]}
            points.append(measure_point(c, dd, gg, main_sets, psteps, 10, torch, beam, hp,
                                        packed=args.packed))
        pre = synth.CONFIGS["qwen3_prefill"]
        for T, keep, n in ((1024, 0.15, 30), (4096, 0.15, 30), (4096, 0.25, 30), (4096, 0.5, 20),
                           (4096, 1.0, 20), (16384, 0.15, 20), (16384, 0.25, 20),
                           (16384, 0.5, 15), (16384, 1.0, 10)):
            c = pre.with_(T=T, keep=keep)
            dd = synth.make_layer(c, with_experts=False)
            gg = {**hp.upload(c, dd), "w_gate_up": g["w_gate_up"], "w_down": g["w_down"]}
            # 20 untimed forwards first: the clock needs tens of milliseconds of load to settle
            points.append(measure_point(c, dd, gg, get_packed_sets(), n, 20, torch, beam, hp,
                                        packed=True))
        c = pre.with_(T=16384, keep=0.15)
        dd = synth.make_layer(c, with_experts=False)
        gg = hp.upload(c, dd)
        pw = get_packed_sets()[0]
        training = measure_training_step(c, gg, pw[0], pw[1], True, 10, torch, beam, hp)
        del dd, gg, pw
        # the two shared-expert model shapes (whole block: residual + routed + shared)
        if not args.packed:
            packed_sets = None       # free the repacked Qwen3 copies
        for name in ("qwen15_moe", "dsv2_lite"):
            c = synth.CONFIGS[name]
            dd = synth.make_layer(c)
            gg = upload_layer(c, dd, hp, synth)
            bsets = [(gg["w_gate_up"], gg["w_down"]),
                     (gg["w_gate_up"].clone(), gg["w_down"].clone())]
            if args.packed:
                bsets = [hp.pack_weights(c.with_(N=c.N + c.S), a, b) for a, b in bsets]
            points.append(measure_point(c, dd, gg, bsets, psteps, 10, torch, beam, hp,
                                        packed=args.packed))
            del dd, gg, bsets
        # Mixtral-shaped and large fine-grained layers: expert weights drawn on the device
        packed_sets = None               # free the repacked Qwen3 copies
        torch.cuda.empty_cache()
        for name, Ts in (("mixtral", (1, 16, 2048)), ("large", (64, 8192))):
            base = synth.CONFIGS[name]
            wsets = device_weight_sets(base, 2, torch, synth.seed_for(base, 98))
            for T in Ts:
                c = base.with_(T=T)
                for sweep in range(8):     # a single token may keep nothing: next draw then
                    dd = synth.make_layer(c, sweep=sweep, with_experts=False)
                    gg = hp.upload(c, dd)
                    pt = measure_point(c, dd, gg, wsets, 20 if T <= 64 else 10, 10, torch, beam,
                                       hp, packed=args.packed)
                    if pt["P"] > 0:
                        break
                pt["weights"] += ", drawn on the device"
                pt["input_draw"] = sweep
                points.append(pt)
                del dd, gg
            del wsets
            torch.cuda.empty_cache()
    rules = []
    if not args.no_points and args.workload == "qwen3_decode":
        rules = measure_rules(cfg, g, main_sets, max(20, args.steps // 4), torch, beam, hp,
                              args.packed)
    stack = []
    if not args.no_points and args.workload == "qwen3_decode" and args.stack_layers > 0:
        stack = measure_decode_stack(cfg, args.stack_layers, (1, 8, 64), torch, beam, hp, synth,
                                     args.packed)
    for p in points:
        p["roofline"] = roofline_of(p)
        p.pop("gate_up")

    cpu = None
    if not args.no_cpu_baseline:
        import oracle      # the oracle is timed here and nowhere else in this file
        nthreads = min(oracle.max_threads(), 16)
        Ts = min(cfg.T, 256)
        xs = d["x"][:Ts]

        def run():
            if cfg.S > 0:
                return oracle.block_forward(xs, d["w_router"], d["b_router"], d["w_mask"],
                                            d["b_mask"], d["w_gate_up"], d["w_down"], cfg.K,
                                            w_sh_gate_up=d["w_sh_gate_up"],
                                            w_sh_down=d["w_sh_down"], w_sh_gate=d["w_sh_gate"],
                                            residual=d["residual"][:Ts], nthreads=nthreads)
            return oracle.moe_forward(xs, d["w_router"], d["b_router"], d["w_mask"], d["b_mask"],
                                      d["w_gate_up"], d["w_down"], cfg.K, nthreads=nthreads)
        run()
        t0 = time.perf_counter()
        reps = 0
        while reps < 3 or (time.perf_counter() - t0 < 5.0 and reps < 50):
            run()
            reps += 1
        dt = (time.perf_counter() - t0) / reps
        cpu = {"value": Ts / dt, "unit": "tokens/s", "cores": nthreads, "kind": "oracle",
               "sample": f"first {Ts} tokens of the step, mean of {reps} runs after 1 warm-up, "
                         f"{dt * 1e3:.1f} ms each"}

    ceilings = measure_ceilings(g["w_gate_up"], torch, beam)
    main_roofline = roofline_of(main_pt)
    for rf in [main_roofline] + [p["roofline"] for p in points]:
        rf["frac_of_measured_ceiling"] = rf["achieved"] / (
            ceilings["stream_read_GBs"] if rf["bound"] == "hbm" else ceilings["mfma_bf16_TFLOPs"])
    rec = {
        "metric": "masked_moe_layer_tokens_per_s", "value": main_pt["tokens_per_s"],
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_pt["ms_per_step"], "us_per_layer": main_pt["us_per_layer"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} H={cfg.H} N={cfg.N} K={cfg.K} I={cfg.I} "
                               f"keep~{cfg.keep}" + (f" shared={cfg.S}x{cfg.I}" if cfg.S else ""),
                   "kept_pairs": main_pt["P"],
                   "experts_touched": main_pt["U"], "weight_sets_rotated": len(sets),
                   "weights": main_pt["weights"],
                   "point": main_pt["workload"] + " " + main_pt["weights"],
                   "input_setup_s": round(t_gen, 1)},
        "layer": {k: main_pt[k] for k in ("layer_GBs", "layer_TFLOPs", "frac_hbm", "frac_mfma",
                                          "frac_of_roofline", "stage_us", "kernel_us",
                                          "stage_algorithmic")},
        "roofline": main_roofline,
        "cpu_baseline": cpu,
        "warm_cache": warm,
        "points": points,
        "rules": rules,
        "decode_stack": stack,
        "training_step": training,
        "ceilings": ceilings,
    }
    print(json.dumps(rec))


if __name__ == "__main__":
    main()

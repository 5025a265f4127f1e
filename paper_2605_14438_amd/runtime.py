"""PyTorch plumbing around the C ABI: device buffers for a synthetic layer,
workspace and output allocation, the current stream handle.  PyTorch is used
for memory and streams only; nothing here computes."""
from __future__ import annotations

import numpy as np
import torch

from . import binding, synth


def dev(arr, dtype: str):
    """numpy fp32 -> device tensor in the layer dtype ("bf16" is exact: the
    values are already bf16-representable)."""
    if arr is None:
        return None
    if dtype == "bf16":
        bits = synth.bf16_bits(arr).view(np.int16)
        return torch.from_numpy(bits).cuda().view(torch.bfloat16).reshape(arr.shape)
    return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).cuda()


def dev_f32(arr):
    return None if arr is None else torch.from_numpy(np.ascontiguousarray(arr, np.float32)).cuda()


def upload(cfg, d):
    g = {k: dev(d[k], cfg.dtype) for k in ("x", "w_router", "w_mask", "w_gate_up", "w_down")
         if d.get(k) is not None}
    g["b_router"] = dev_f32(d["b_router"])
    g["b_mask"] = dev_f32(d["b_mask"])
    return g


def shape_of(cfg, T=None, packed: bool = False):
    return binding.make_shape(cfg.T if T is None else T, cfg.H, cfg.N, cfg.K, cfg.I,
                              binding.BEAM_BF16 if cfg.dtype == "bf16" else binding.BEAM_F32,
                              binding.BEAM_WEIGHTS_PACKED if packed else binding.BEAM_WEIGHTS_PLAIN)


def pack_weights(cfg, w_gate_up, w_down):
    """One-time repack of plain expert weights into matrix-core fragment order."""
    s = shape_of(cfg, packed=False)
    pg = torch.empty_like(w_gate_up)
    pd = torch.empty_like(w_down)
    binding.beam_pack_weights(s, w_gate_up, w_down, pg, pd, stream_ptr())
    return pg, pd


def workspace(shape):
    nbytes = binding.beam_workspace_bytes(shape)
    if nbytes <= 0:
        raise ValueError("unsupported shape")
    return torch.empty(nbytes, dtype=torch.uint8, device="cuda"), nbytes


def out_tensor(cfg, T=None):
    T = cfg.T if T is None else T
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    return torch.full((T, cfg.H), float("nan"), dtype=dt, device="cuda")


def stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream

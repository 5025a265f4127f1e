"""Seeded synthetic inputs for the binary-masked MoE layer (BEAM, Sec. 3.2).

This module only draws random buffers.  It contains none of the method's
arithmetic (no logits, no Top-K, no mask decision, no expert FFN), so both the
CPU oracle's tests and the HIP path can consume exactly the same numbers
without sharing any logic.

Shapes follow the paper's notation: T tokens, H = d_h hidden size, N experts,
K experts per token, I = expert intermediate size.  Weight layouts are
"output-feature major, reduction dimension contiguous":

    w_router  [N, H]      router R(x) = x W_r           (Sec. 3.2 Step 1)
    w_mask    [N, H]      mask router a = x W_m         (Eq. 5)
    w_gate_up [N, 2I, H]  rows 0..I-1 = W_gate^T, rows I..2I-1 = W_up^T   (Eq. 3)
    w_down    [N, H, I]   W_down^T                      (Eq. 3)

With a shared expert (App. A.3; S > 0) there are also, drawn last so that the
streams of the routed layer do not move:

    w_sh_gate_up [2*S*I, H], w_sh_down [H, S*I]   one GLU expert of width S*I
    w_sh_gate    [H]      gate vector of the shared expert's weight (optional)
    residual     [T, H]   the block input h before normalisation, ~ N(0, 1)

The recipe (value distributions, keep-rate calibration, popularity skew) is a
stand-in for real model activations, which need trained weights:

* hidden states ~ N(0, 1); every weight ~ N(0, 0.02^2);
* bf16 configurations round every buffer to bf16 (round-to-nearest-even)
  before anyone sees it, and hand out the exactly representable fp32 values;
* the keep rate is set with a uniform mask-head bias b = sigma_a * Phi^-1(keep)
  where sigma_a = 0.02 * sqrt(H) is the standard deviation of a mask logit of
  a random token.  The mask logit of a random W_m is independent of the routing
  rank, which is what the paper observes for trained masks (Sec. 4.4, position
  wise masking), so the kept count of a token is ~ Binomial(K, keep) and
  tokens with no kept expert are common at low keep rates;
* "zipf" router skew adds b_r[e] = -s * ln(rank_e) with a random rank
  permutation, which concentrates the routed pairs on a few experts;
* "beta" keep mode draws a per-token keep probability rho_t ~ Beta(a, b) and
  realises it inside the paper's parametrisation (a bias cannot depend on the
  token) by reserving hidden feature 0: W_m[:, 0] = 1 and
  x[t, 0] = sigma_a * Phi^-1(rho_t).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from statistics import NormalDist
from typing import Dict, Optional

import numpy as np

_INIT_STD = 0.02
_BASE_SEED = 14438 * 100


@dataclass(frozen=True)
class LayerConfig:
    """One synthetic workload point."""

    name: str
    index: int          # position in the benchmark's config list (seed stream)
    T: int
    H: int
    N: int
    K: int
    I: int
    dtype: str          # "f32" or "bf16": dtype of x, all weights and the output
    keep: float         # target fraction of Top-K pairs kept by the mask
    router_skew: str = "none"   # "none" | "zipf"
    zipf_s: float = 1.1
    keep_mode: str = "uniform"  # "uniform" | "beta"
    beta_a: float = 2.0
    beta_b: float = 8.0
    S: int = 0                  # shared expert of width S*I (0 = none)
    shared_gate: bool = False   # draw a gate vector for the shared expert's weight

    def with_(self, **kw) -> "LayerConfig":
        return replace(self, **kw)


# The benchmark's named workloads.  T and keep are the defaults; sweeps
# override them with LayerConfig.with_().
CONFIGS: Dict[str, LayerConfig] = {
    "tiny": LayerConfig("tiny", 0, T=64, H=256, N=8, K=2, I=512, dtype="f32", keep=0.5),
    "qwen3_decode": LayerConfig("qwen3_decode", 1, T=64, H=2048, N=128, K=8, I=768,
                                dtype="bf16", keep=0.15),
    "qwen3_prefill": LayerConfig("qwen3_prefill", 2, T=4096, H=2048, N=128, K=8, I=768,
                                 dtype="bf16", keep=0.15, router_skew="zipf"),
    "mixtral": LayerConfig("mixtral", 3, T=16, H=4096, N=8, K=2, I=14336,
                           dtype="bf16", keep=0.6),
    "large": LayerConfig("large", 4, T=64, H=4096, N=128, K=8, I=1536,
                         dtype="bf16", keep=0.2, keep_mode="beta"),
    # The two shared-expert models of the paper's evaluation (App. A.5): 60 routed
    # experts, 4 per token, 4 shared (gated); 64 routed, 6 per token, 2 shared.
    "qwen15_moe": LayerConfig("qwen15_moe", 5, T=64, H=2560, N=60, K=4, I=1408,
                              dtype="bf16", keep=0.25, S=4, shared_gate=True),
    "dsv2_lite": LayerConfig("dsv2_lite", 6, T=64, H=2048, N=64, K=6, I=1408,
                             dtype="bf16", keep=0.25, S=2),
}


def seed_for(cfg: LayerConfig, sweep: int = 0) -> int:
    return _BASE_SEED + cfg.index * 10 + sweep


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(a: np.ndarray) -> np.ndarray:
    """fp32 array -> nearest bf16 value, returned as fp32 (exactly representable)."""
    return bf16_bits_to_f32(bf16_bits(a))


def _normal(rng: np.random.Generator, shape, std: float, chunk: int = 1 << 24) -> np.ndarray:
    """N(0, std^2) in fp32, filled in chunks so the fp64 temporaries stay small."""
    out = np.empty(shape, dtype=np.float32)
    flat = out.reshape(-1)
    for lo in range(0, flat.size, chunk):
        hi = min(lo + chunk, flat.size)
        rng.standard_normal(hi - lo, dtype=np.float32, out=flat[lo:hi])
    if std != 1.0:
        flat *= np.float32(std)
    return out


def mask_logit_sigma(cfg: LayerConfig) -> float:
    """Std of a mask logit of a random token: |x| ~ sqrt(H), weights N(0, 0.02^2)."""
    return _INIT_STD * math.sqrt(cfg.H)


def mask_bias_value(cfg: LayerConfig) -> float:
    if cfg.keep >= 1.0:
        return 1.0e4
    if cfg.keep <= 0.0:
        return -1.0e4
    return mask_logit_sigma(cfg) * NormalDist().inv_cdf(cfg.keep)


def make_layer(cfg: LayerConfig, sweep: int = 0, with_experts: bool = True) -> Dict[str, Optional[np.ndarray]]:
    """Draw every buffer of one layer.  Draw order is fixed: x, W_r, W_m, rank
    permutation / per-token keep draws, then W_gate_up and W_down.

    Returns fp32 numpy arrays (bf16 configs: values already rounded to bf16)
    plus "b_router" / "b_mask" (fp32 [N] or None).
    """
    rng = np.random.Generator(np.random.PCG64(seed_for(cfg, sweep)))
    T, H, N, I = cfg.T, cfg.H, cfg.N, cfg.I
    x = _normal(rng, (T, H), 1.0)
    w_router = _normal(rng, (N, H), _INIT_STD)
    w_mask = _normal(rng, (N, H), _INIT_STD)

    b_router = None
    if cfg.router_skew == "zipf":
        rank = rng.permutation(N) + 1
        b_router = (-cfg.zipf_s * np.log(rank.astype(np.float64))).astype(np.float32)

    b_mask = None
    if cfg.keep_mode == "beta":
        rho = rng.beta(cfg.beta_a, cfg.beta_b, size=T)
        rho = np.clip(rho, 1e-6, 1.0 - 1e-6)
        nd = NormalDist()
        s = np.array([nd.inv_cdf(float(p)) for p in rho]) * mask_logit_sigma(cfg)
        x[:, 0] = s.astype(np.float32)
        w_mask[:, 0] = 1.0
    else:
        b = mask_bias_value(cfg)
        if b != 0.0:
            b_mask = np.full((N,), b, dtype=np.float32)

    out: Dict[str, Optional[np.ndarray]] = {"b_router": b_router, "b_mask": b_mask}
    if with_experts:
        w_gate_up = _normal(rng, (N, 2 * I, H), _INIT_STD)
        w_down = _normal(rng, (N, H, I), _INIT_STD)
    else:
        w_gate_up = w_down = None

    if cfg.dtype == "bf16":
        x = bf16_round(x)
        w_router = bf16_round(w_router)
        w_mask = bf16_round(w_mask)
        if with_experts:
            w_gate_up = bf16_round(w_gate_up)
            w_down = bf16_round(w_down)
    out.update(x=x, w_router=w_router, w_mask=w_mask, w_gate_up=w_gate_up, w_down=w_down)
    if cfg.S > 0:
        rnd = bf16_round if cfg.dtype == "bf16" else (lambda a: a)
        if with_experts:
            out["w_sh_gate_up"] = rnd(_normal(rng, (2 * cfg.S * I, H), _INIT_STD))
            out["w_sh_down"] = rnd(_normal(rng, (H, cfg.S * I), _INIT_STD))
        out["w_sh_gate"] = rnd(_normal(rng, (H,), _INIT_STD)) if cfg.shared_gate else None
        out["residual"] = rnd(_normal(rng, (T, H), 1.0))
    return out


def append_shared_blocks(cfg: LayerConfig, data: Dict[str, Optional[np.ndarray]]):
    """Expert arrays with the shared expert cut into S column blocks of width I
    and appended as experts N .. N+S-1 (a copy; the layout the library's block
    entry point takes).  Returns (w_gate_up [N+S,2I,H], w_down [N+S,H,I])."""
    S, I, H = cfg.S, cfg.I, cfg.H
    sgu, sd = data["w_sh_gate_up"], data["w_sh_down"]
    gu = np.empty((cfg.N + S, 2 * I, H), dtype=np.float32)
    dn = np.empty((cfg.N + S, H, I), dtype=np.float32)
    gu[:cfg.N] = data["w_gate_up"]
    dn[:cfg.N] = data["w_down"]
    for j in range(S):
        gu[cfg.N + j, :I] = sgu[j * I:(j + 1) * I]
        gu[cfg.N + j, I:] = sgu[S * I + j * I:S * I + (j + 1) * I]
        dn[cfg.N + j] = sd[:, j * I:(j + 1) * I]
    return gu, dn


def redraw_rows(cfg: LayerConfig, data: Dict[str, Optional[np.ndarray]], rows: np.ndarray,
                sweep: int = 0, attempt: int = 1) -> None:
    """Replace the hidden rows `rows` of data["x"] in place with fresh N(0,1)
    draws from a side stream of the same seed.  Used by parity tests to redraw
    tokens whose routing or mask decision sits inside the fp32 rounding guard
    band (the caller decides which rows; this function only draws)."""
    rows = np.asarray(rows, dtype=np.int64)
    if rows.size == 0:
        return
    rng = np.random.Generator(np.random.PCG64([seed_for(cfg, sweep), 7919, attempt]))
    fresh = _normal(rng, (rows.size, cfg.H), 1.0)
    if cfg.keep_mode == "beta":
        fresh[:, 0] = data["x"][rows, 0]
    if cfg.dtype == "bf16":
        fresh = bf16_round(fresh)
    data["x"][rows] = fresh

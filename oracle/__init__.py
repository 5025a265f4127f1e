"""Python face of the CPU oracle (oracle/beam_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module.

`build()` compiles the C file with gcc; the functions below marshal numpy
arrays into it.  All arithmetic lives in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "beam_oracle.c")
_LIB = os.path.join(_HERE, "libbeam_oracle.so")
_lib: Optional[ctypes.CDLL] = None

_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int32)


def build(force: bool = True) -> str:
    """Compile the oracle (-O2, OpenMP over tokens, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        lib.beam_oracle_max_threads.restype = ctypes.c_int
        lib.beam_oracle_logits.restype = None
        lib.beam_oracle_route_mask.restype = None
        lib.beam_oracle_permute.restype = None
        lib.beam_oracle_expert_ffn.restype = None
        lib.beam_oracle_pair_outputs.restype = ctypes.c_int64
        lib.beam_oracle_moe_forward.restype = ctypes.c_int64
        lib.beam_oracle_block_forward.restype = ctypes.c_int64
        lib.beam_oracle_route_rule.restype = None
        lib.beam_oracle_train_step.restype = None
        lib.beam_oracle_moe_forward_rule.restype = ctypes.c_int64
        _lib = lib
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a: Optional[np.ndarray], typ):
    if a is None:
        return typ()
    return a.ctypes.data_as(typ)


def max_threads() -> int:
    return int(_load().beam_oracle_max_threads())


def logits(x, w, bias=None) -> np.ndarray:
    """[T,H] x [N,H] (+bias) -> [T,N] fp32 (fp64 sums)."""
    x = _f32(x)
    w = _f32(w)
    b = None if bias is None else _f32(bias)
    T, H = x.shape
    N = w.shape[0]
    assert w.shape[1] == H
    out = np.empty((T, N), dtype=np.float32)
    _load().beam_oracle_logits(T, H, N, _ptr(x, _f32p), _ptr(w, _f32p), _ptr(b, _f32p),
                               _ptr(out, _f32p))
    return out


def route_mask(router_logits, mask_logits, K: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """-> (topk_ids [T,K] i32, topk_weights [T,K] f64, masked_ids [T,K] i32)."""
    r = _f32(router_logits)
    a = _f32(mask_logits)
    T, N = r.shape
    assert a.shape == (T, N) and 1 <= K <= N
    ids = np.empty((T, K), dtype=np.int32)
    g = np.empty((T, K), dtype=np.float64)
    msk = np.empty((T, K), dtype=np.int32)
    _load().beam_oracle_route_mask(T, N, K, _ptr(r, _f32p), _ptr(a, _f32p), _ptr(ids, _i32p),
                                   _ptr(g, _f64p), _ptr(msk, _i32p))
    return ids, g, msk


def permute(masked_ids, N: int):
    """-> (counts [N], offsets [N+1], perm [TK], inv_perm [TK], num_pairs)."""
    m = np.ascontiguousarray(masked_ids, dtype=np.int32).reshape(-1)
    TK = m.size
    counts = np.empty((N,), dtype=np.int32)
    offsets = np.empty((N + 1,), dtype=np.int32)
    perm = np.empty((TK,), dtype=np.int32)
    inv = np.empty((TK,), dtype=np.int32)
    P = ctypes.c_int32(0)
    _load().beam_oracle_permute(TK, N, _ptr(m, _i32p), _ptr(counts, _i32p), _ptr(offsets, _i32p),
                                _ptr(perm, _i32p), _ptr(inv, _i32p), ctypes.byref(P))
    return counts, offsets, perm, inv, int(P.value)


def expert_ffn(x_row, w_gate_up_e, w_down_e) -> np.ndarray:
    """One expert on one token: x [H], w_gate_up_e [2I,H], w_down_e [H,I] -> y [H] f64."""
    x = _f32(x_row)
    wgu = _f32(w_gate_up_e)
    wd = _f32(w_down_e)
    H = x.shape[0]
    I = wd.shape[1]
    assert wgu.shape == (2 * I, H) and wd.shape == (H, I)
    y = np.empty((H,), dtype=np.float64)
    _load().beam_oracle_expert_ffn(H, I, _ptr(x, _f32p), _ptr(wgu, _f32p), _ptr(wd, _f32p),
                                   _ptr(y, _f64p))
    return y


def pair_outputs(x, w_gate_up, w_down, masked_ids, nthreads: int = 0):
    """E_e(x_t) per kept slot -> (y_slots [T*K,H] f64, evaluations)."""
    x = _f32(x)
    wgu = _f32(w_gate_up)
    wd = _f32(w_down)
    m = np.ascontiguousarray(masked_ids, dtype=np.int32)
    T, H = x.shape
    N, H2, I = wd.shape
    K = m.shape[1]
    assert H2 == H and wgu.shape == (N, 2 * I, H) and m.shape[0] == T
    y = np.empty((T * K, H), dtype=np.float64)
    n = _load().beam_oracle_pair_outputs(T, H, N, K, I, _ptr(x, _f32p), _ptr(wgu, _f32p),
                                         _ptr(wd, _f32p), _ptr(m, _i32p), _ptr(y, _f64p),
                                         int(nthreads))
    return y, int(n)


def moe_forward(x, w_router, b_router, w_mask, b_mask, w_gate_up, w_down, K: int,
                nthreads: int = 0):
    """Whole layer -> dict(out [T,H] f64, topk_ids, topk_weights, masked_ids, pair_evals)."""
    x = _f32(x)
    wr = _f32(w_router)
    wm = _f32(w_mask)
    br = None if b_router is None else _f32(b_router)
    bm = None if b_mask is None else _f32(b_mask)
    wgu = _f32(w_gate_up)
    wd = _f32(w_down)
    T, H = x.shape
    N, H2, I = wd.shape
    assert H2 == H and wr.shape == (N, H) and wm.shape == (N, H) and wgu.shape == (N, 2 * I, H)
    assert 1 <= K <= N
    out = np.empty((T, H), dtype=np.float64)
    ids = np.empty((T, K), dtype=np.int32)
    g = np.empty((T, K), dtype=np.float64)
    msk = np.empty((T, K), dtype=np.int32)
    n = _load().beam_oracle_moe_forward(
        T, H, N, K, I, _ptr(x, _f32p), _ptr(wr, _f32p), _ptr(br, _f32p), _ptr(wm, _f32p),
        _ptr(bm, _f32p), _ptr(wgu, _f32p), _ptr(wd, _f32p), _ptr(out, _f64p), _ptr(ids, _i32p),
        _ptr(g, _f64p), _ptr(msk, _i32p), int(nthreads))
    return {"out": out, "topk_ids": ids, "topk_weights": g, "masked_ids": msk,
            "pair_evals": int(n)}


RULE_THRESHOLD = 0    # param = theta = ln(tau / (1 - tau)): keep iff a >= theta
RULE_CUMPROB = 1      # param = phi: activate ranks until the cumulative softmax-over-N exceeds phi


def route_rule(router_logits, mask_logits, K: int, kind: int, param: float):
    """route_mask under another activation rule -> (topk_ids, topk_weights, masked_ids)."""
    r = _f32(router_logits)
    a = _f32(mask_logits)
    T, N = r.shape
    assert a.shape == (T, N) and 1 <= K <= N
    ids = np.empty((T, K), dtype=np.int32)
    g = np.empty((T, K), dtype=np.float64)
    msk = np.empty((T, K), dtype=np.int32)
    _load().beam_oracle_route_rule(T, N, K, _ptr(r, _f32p), _ptr(a, _f32p), int(kind),
                                   ctypes.c_float(param), _ptr(ids, _i32p), _ptr(g, _f64p),
                                   _ptr(msk, _i32p))
    return ids, g, msk


def moe_forward_rule(x, w_router, b_router, w_mask, b_mask, w_gate_up, w_down, K: int,
                     kind: int, param: float, nthreads: int = 0):
    """moe_forward under another activation rule."""
    x = _f32(x)
    wr = _f32(w_router)
    wm = _f32(w_mask)
    br = None if b_router is None else _f32(b_router)
    bm = None if b_mask is None else _f32(b_mask)
    wgu = _f32(w_gate_up)
    wd = _f32(w_down)
    T, H = x.shape
    N, H2, I = wd.shape
    assert H2 == H and wr.shape == (N, H) and wm.shape == (N, H) and wgu.shape == (N, 2 * I, H)
    assert 1 <= K <= N
    out = np.empty((T, H), dtype=np.float64)
    ids = np.empty((T, K), dtype=np.int32)
    g = np.empty((T, K), dtype=np.float64)
    msk = np.empty((T, K), dtype=np.int32)
    n = _load().beam_oracle_moe_forward_rule(
        T, H, N, K, I, _ptr(x, _f32p), _ptr(wr, _f32p), _ptr(br, _f32p), _ptr(wm, _f32p),
        _ptr(bm, _f32p), _ptr(wgu, _f32p), _ptr(wd, _f32p), int(kind), ctypes.c_float(param),
        _ptr(out, _f64p), _ptr(ids, _i32p), _ptr(g, _f64p), _ptr(msk, _i32p), int(nthreads))
    return {"out": out, "topk_ids": ids, "topk_weights": g, "masked_ids": msk,
            "pair_evals": int(n)}


def block_forward(x, w_router, b_router, w_mask, b_mask, w_gate_up, w_down, K: int,
                  w_sh_gate_up=None, w_sh_down=None, w_sh_gate=None, residual=None,
                  nthreads: int = 0):
    """Whole block with shared expert and residual (App. A.3) -> dict like moe_forward
    plus g_shared [T] f64.  w_sh_gate_up [2*I_sh,H], w_sh_down [H,I_sh] (both or neither)."""
    x = _f32(x)
    wr = _f32(w_router)
    wm = _f32(w_mask)
    br = None if b_router is None else _f32(b_router)
    bm = None if b_mask is None else _f32(b_mask)
    wgu = _f32(w_gate_up)
    wd = _f32(w_down)
    T, H = x.shape
    N, H2, I = wd.shape
    assert H2 == H and wr.shape == (N, H) and wm.shape == (N, H) and wgu.shape == (N, 2 * I, H)
    assert 1 <= K <= N
    assert (w_sh_gate_up is None) == (w_sh_down is None)
    I_sh = 0
    sgu = sd = sg = res = None
    if w_sh_down is not None:
        sgu = _f32(w_sh_gate_up)
        sd = _f32(w_sh_down)
        I_sh = sd.shape[1]
        assert sd.shape == (H, I_sh) and sgu.shape == (2 * I_sh, H)
    if w_sh_gate is not None:
        sg = _f32(w_sh_gate)
        assert sg.shape == (H,)
    if residual is not None:
        res = _f32(residual)
        assert res.shape == (T, H)
    out = np.empty((T, H), dtype=np.float64)
    ids = np.empty((T, K), dtype=np.int32)
    g = np.empty((T, K), dtype=np.float64)
    msk = np.empty((T, K), dtype=np.int32)
    gsh = np.empty((T,), dtype=np.float64)
    n = _load().beam_oracle_block_forward(
        T, H, N, K, I, _ptr(x, _f32p), _ptr(wr, _f32p), _ptr(br, _f32p), _ptr(wm, _f32p),
        _ptr(bm, _f32p), _ptr(wgu, _f32p), _ptr(wd, _f32p), I_sh, _ptr(sgu, _f32p),
        _ptr(sd, _f32p), _ptr(sg, _f32p), _ptr(res, _f32p), _ptr(out, _f64p), _ptr(ids, _i32p),
        _ptr(g, _f64p), _ptr(msk, _i32p), _ptr(gsh, _f64p), int(nthreads))
    return {"out": out, "topk_ids": ids, "topk_weights": g, "masked_ids": msk,
            "g_shared": gsh, "pair_evals": int(n)}


def train_step(x, w_router, b_router, w_mask, b_mask, w_gate_up, w_down, K: int, grad_out,
               reg_coeff: float):
    """Training-mode forward and the mask router's backward (Sec. 3.3, Eq. 9-12) ->
    dict(out [T,H], grad_a [T,K], grad_w_mask [N,H], loss_reg [T], topk_ids, masked_ids)."""
    x = _f32(x)
    wr = _f32(w_router)
    wm = _f32(w_mask)
    br = None if b_router is None else _f32(b_router)
    bm = None if b_mask is None else _f32(b_mask)
    wgu = _f32(w_gate_up)
    wd = _f32(w_down)
    dy = _f32(grad_out)
    T, H = x.shape
    N, H2, I = wd.shape
    assert H2 == H and wr.shape == (N, H) and wm.shape == (N, H) and wgu.shape == (N, 2 * I, H)
    assert dy.shape == (T, H) and 1 <= K <= N
    out = np.empty((T, H), dtype=np.float64)
    ga = np.empty((T, K), dtype=np.float64)
    gw = np.empty((N, H), dtype=np.float64)
    lr = np.empty((T,), dtype=np.float64)
    ids = np.empty((T, K), dtype=np.int32)
    msk = np.empty((T, K), dtype=np.int32)
    _load().beam_oracle_train_step(
        T, H, N, K, I, _ptr(x, _f32p), _ptr(wr, _f32p), _ptr(br, _f32p), _ptr(wm, _f32p),
        _ptr(bm, _f32p), _ptr(wgu, _f32p), _ptr(wd, _f32p), _ptr(dy, _f32p),
        ctypes.c_double(reg_coeff), _ptr(out, _f64p), _ptr(ga, _f64p), _ptr(gw, _f64p),
        _ptr(lr, _f64p), _ptr(ids, _i32p), _ptr(msk, _i32p))
    return {"out": out, "grad_a": ga, "grad_w_mask": gw, "loss_reg": lr, "topk_ids": ids,
            "masked_ids": msk}


def decision_margin(router_logits, mask_logits, K: int) -> np.ndarray:
    """Per token: the smallest gap any integer decision of the layer rests on.

    Those decisions are the K+1 leading ranks of the router logits (adjacent
    gaps between ranks 1..K+1 decide both membership and slot order) and the
    sign of the mask pre-activation of the K selected experts.  A token whose
    margin is far above fp32 summation noise has indices that any correct
    fp32 evaluation must reproduce bit for bit.
    """
    r = np.asarray(router_logits, dtype=np.float64)
    a = np.asarray(mask_logits, dtype=np.float64)
    T, N = r.shape
    order = np.argsort(-r, axis=1, kind="stable")
    lead = np.take_along_axis(r, order[:, : min(K + 1, N)], axis=1)
    gaps = lead[:, :-1] - lead[:, 1:] if lead.shape[1] > 1 else np.full((T, 1), np.inf)
    a_sel = np.abs(np.take_along_axis(a, order[:, :K], axis=1))
    return np.minimum(gaps.min(axis=1), a_sel.min(axis=1))

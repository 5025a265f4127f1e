"""Thin ctypes binding of libbeam.so: same names and argument order as
include/beam.h.  Argument marshalling only; every step of the layer runs in
the HIP kernels.  Pointers may be given as torch tensors (their data_ptr() is
taken; the caller keeps them alive and on the right device), as ints, or as
None for the optional ones.

There is no fallback: if the library has not been built, importing the
functions raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbeam.so")

BEAM_OK = 0
BEAM_ERR_INVALID_ARG = 1
BEAM_ERR_UNSUPPORTED = 2
BEAM_ERR_WORKSPACE = 3
BEAM_ERR_HIP = 4
BEAM_F32 = 0
BEAM_BF16 = 1
BEAM_WEIGHTS_PLAIN = 0
BEAM_WEIGHTS_PACKED = 1

EXPORTS = ("beam_abi_version", "beam_status_string", "beam_workspace_bytes", "beam_route_mask",
           "beam_permute", "beam_expert_ffn", "beam_combine", "beam_moe_forward",
           "beam_moe_forward_timed", "beam_pack_weights", "beam_block_workspace_bytes",
           "beam_moe_block_forward", "beam_moe_block_forward_timed", "beam_route_rule",
           "beam_moe_forward_rule", "beam_mask_router_backward", "beam_probe_stream_read",
           "beam_probe_mfma", "beam_workspace_logits_region",
           "beam_moe_forward_noalloc", "beam_fused_pair_row_bits")
BEAM_NOALLOC_WORKSPACE_BYTES = 32 << 20
BEAM_RULE_MASK = 0
BEAM_RULE_CUMPROB = 1
BEAM_NUM_STAGES = 6
STAGE_NAMES = ("logits", "topk_mask", "permute", "gate_up", "down", "combine")


class beam_shape(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("H", ctypes.c_int32), ("N", ctypes.c_int32),
                ("K", ctypes.c_int32), ("I", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("weight_layout", ctypes.c_int32)]


class beam_rule(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("param", ctypes.c_float)]


class BeamError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn}: {beam_status_string(status)} (status {status})")


_lib: Optional[ctypes.CDLL] = None


def load() -> ctypes.CDLL:
    """dlopen the in-tree library; raises if it was never built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with "
                "`python -m paper_2605_14438_amd.build` (there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        sp = ctypes.POINTER(beam_shape)
        lib.beam_abi_version.restype = ctypes.c_int32
        lib.beam_abi_version.argtypes = []
        lib.beam_status_string.restype = ctypes.c_char_p
        lib.beam_status_string.argtypes = [ctypes.c_int]
        lib.beam_workspace_bytes.restype = sz
        lib.beam_workspace_bytes.argtypes = [sp]
        lib.beam_route_mask.restype = ctypes.c_int
        lib.beam_route_mask.argtypes = [sp] + [vp] * 11 + [sz, vp]
        lib.beam_permute.restype = ctypes.c_int
        lib.beam_permute.argtypes = [sp] + [vp] * 7 + [sz, vp]
        lib.beam_expert_ffn.restype = ctypes.c_int
        lib.beam_expert_ffn.argtypes = [sp] + [vp] * 8 + [sz, vp]
        lib.beam_combine.restype = ctypes.c_int
        lib.beam_combine.argtypes = [sp] + [vp] * 6
        lib.beam_moe_forward.restype = ctypes.c_int
        lib.beam_moe_forward.argtypes = [sp] + [vp] * 13 + [sz, vp]
        lib.beam_moe_forward_noalloc.restype = ctypes.c_int
        lib.beam_moe_forward_noalloc.argtypes = [sp] + [vp] * 9
        rp = ctypes.POINTER(beam_rule)
        lib.beam_route_rule.restype = ctypes.c_int
        lib.beam_route_rule.argtypes = [sp, rp] + [vp] * 11 + [sz, vp]
        lib.beam_moe_forward_rule.restype = ctypes.c_int
        lib.beam_moe_forward_rule.argtypes = [sp, rp] + [vp] * 13 + [sz, vp]
        lib.beam_mask_router_backward.restype = ctypes.c_int
        lib.beam_mask_router_backward.argtypes = [sp] + [vp] * 9 + [ctypes.c_float] + [vp] * 4 + [
            sz, vp]
        lib.beam_probe_stream_read.restype = ctypes.c_int
        lib.beam_probe_stream_read.argtypes = [vp, sz, vp, vp, ctypes.POINTER(sz)]
        lib.beam_probe_mfma.restype = ctypes.c_int
        lib.beam_probe_mfma.argtypes = [ctypes.c_int32, vp, vp, ctypes.POINTER(ctypes.c_double)]
        lib.beam_block_workspace_bytes.restype = sz
        lib.beam_block_workspace_bytes.argtypes = [sp, ctypes.c_int32]
        lib.beam_workspace_logits_region.restype = ctypes.c_int
        lib.beam_workspace_logits_region.argtypes = [sp, ctypes.c_int32, ctypes.POINTER(sz),
                                                     ctypes.POINTER(sz),
                                                     ctypes.POINTER(ctypes.c_int32)]
        lib.beam_fused_pair_row_bits.restype = ctypes.c_int32
        lib.beam_fused_pair_row_bits.argtypes = [sp, ctypes.c_int32]
        lib.beam_moe_block_forward.restype = ctypes.c_int
        lib.beam_moe_block_forward.argtypes = [sp, ctypes.c_int32] + [vp] * 15 + [sz, vp]
        lib.beam_moe_block_forward_timed.restype = ctypes.c_int
        lib.beam_moe_block_forward_timed.argtypes = [sp, ctypes.c_int32] + [vp] * 11 + [
            sz, vp, ctypes.POINTER(ctypes.c_float)]
        lib.beam_pack_weights.restype = ctypes.c_int
        lib.beam_pack_weights.argtypes = [sp] + [vp] * 5
        lib.beam_moe_forward_timed.restype = ctypes.c_int
        lib.beam_moe_forward_timed.argtypes = [sp] + [vp] * 9 + [sz, vp,
                                                                 ctypes.POINTER(ctypes.c_float)]
        _lib = lib
    return _lib


def _p(a) -> Optional[int]:
    if a is None:
        return None
    if isinstance(a, int):
        return a
    return a.data_ptr()


def _shape(s) -> beam_shape:
    if isinstance(s, beam_shape):
        return s
    return beam_shape(*s)


def make_shape(T: int, H: int, N: int, K: int, I: int, dtype: int,
               weight_layout: int = BEAM_WEIGHTS_PLAIN) -> beam_shape:
    return beam_shape(T, H, N, K, I, dtype, weight_layout)


def _check(fn: str, status: int, check: bool) -> int:
    if check and status != BEAM_OK:
        raise BeamError(fn, status)
    return status


def beam_abi_version() -> int:
    return int(load().beam_abi_version())


def beam_status_string(status: int) -> str:
    return load().beam_status_string(int(status)).decode()


def beam_workspace_bytes(shape) -> int:
    s = _shape(shape)
    return int(load().beam_workspace_bytes(ctypes.byref(s)))


def beam_pack_weights(shape, w_gate_up, w_down, w_gate_up_packed, w_down_packed, hip_stream=None,
                      check: bool = True) -> int:
    s = _shape(shape)
    st = load().beam_pack_weights(ctypes.byref(s), _p(w_gate_up), _p(w_down),
                                  _p(w_gate_up_packed), _p(w_down_packed), _p(hip_stream))
    return _check("beam_pack_weights", st, check)


def beam_route_mask(shape, x, w_router, router_bias, w_mask, mask_bias, topk_ids, topk_weights,
                    masked_ids, router_logits_dbg, mask_logits_dbg, workspace, workspace_bytes,
                    hip_stream=None, check: bool = True) -> int:
    s = _shape(shape)
    st = load().beam_route_mask(ctypes.byref(s), _p(x), _p(w_router), _p(router_bias), _p(w_mask),
                                _p(mask_bias), _p(topk_ids), _p(topk_weights), _p(masked_ids),
                                _p(router_logits_dbg), _p(mask_logits_dbg), _p(workspace),
                                int(workspace_bytes), _p(hip_stream))
    return _check("beam_route_mask", st, check)


def beam_permute(shape, masked_ids, expert_counts, expert_offsets, perm, inv_perm, num_pairs,
                 workspace, workspace_bytes, hip_stream=None, check: bool = True) -> int:
    s = _shape(shape)
    st = load().beam_permute(ctypes.byref(s), _p(masked_ids), _p(expert_counts),
                             _p(expert_offsets), _p(perm), _p(inv_perm), _p(num_pairs),
                             _p(workspace), int(workspace_bytes), _p(hip_stream))
    return _check("beam_permute", st, check)


def beam_expert_ffn(shape, x, w_gate_up, w_down, expert_offsets, perm, num_pairs, y_pairs,
                    workspace, workspace_bytes, hip_stream=None, check: bool = True) -> int:
    s = _shape(shape)
    st = load().beam_expert_ffn(ctypes.byref(s), _p(x), _p(w_gate_up), _p(w_down),
                                _p(expert_offsets), _p(perm), _p(num_pairs), _p(y_pairs),
                                _p(workspace), int(workspace_bytes), _p(hip_stream))
    return _check("beam_expert_ffn", st, check)


def beam_combine(shape, y_pairs, topk_weights, masked_ids, inv_perm, out, hip_stream=None,
                 check: bool = True) -> int:
    s = _shape(shape)
    st = load().beam_combine(ctypes.byref(s), _p(y_pairs), _p(topk_weights), _p(masked_ids),
                             _p(inv_perm), _p(out), _p(hip_stream))
    return _check("beam_combine", st, check)


def beam_moe_forward(shape, x, w_router, router_bias, w_mask, mask_bias, w_gate_up, w_down, out,
                     topk_ids_opt, topk_weights_opt, masked_ids_opt, num_pairs_opt, workspace,
                     workspace_bytes, hip_stream=None, check: bool = True) -> int:
    s = _shape(shape)
    st = load().beam_moe_forward(ctypes.byref(s), _p(x), _p(w_router), _p(router_bias),
                                 _p(w_mask), _p(mask_bias), _p(w_gate_up), _p(w_down), _p(out),
                                 _p(topk_ids_opt), _p(topk_weights_opt), _p(masked_ids_opt),
                                 _p(num_pairs_opt), _p(workspace), int(workspace_bytes),
                                 _p(hip_stream))
    return _check("beam_moe_forward", st, check)


def beam_moe_forward_noalloc(shape, x, w_router, router_bias, w_mask, mask_bias, w_gate_up, w_down,
                             out, hip_stream=None, check: bool = True) -> int:
    s = _shape(shape)
    st = load().beam_moe_forward_noalloc(ctypes.byref(s), _p(x), _p(w_router), _p(router_bias),
                                         _p(w_mask), _p(mask_bias), _p(w_gate_up), _p(w_down),
                                         _p(out), _p(hip_stream))
    return _check("beam_moe_forward_noalloc", st, check)


def beam_block_workspace_bytes(shape, num_shared: int) -> int:
    s = _shape(shape)
    return int(load().beam_block_workspace_bytes(ctypes.byref(s), int(num_shared)))


def beam_workspace_logits_region(shape, num_shared: int, check: bool = True):
    """Returns (status, byte offset, bytes, parts) of the logits region of the workspace."""
    s = _shape(shape)
    off, nb, parts = ctypes.c_size_t(0), ctypes.c_size_t(0), ctypes.c_int32(0)
    st = load().beam_workspace_logits_region(ctypes.byref(s), int(num_shared), ctypes.byref(off),
                                             ctypes.byref(nb), ctypes.byref(parts))
    return _check("beam_workspace_logits_region", st, check), off.value, nb.value, parts.value


def beam_fused_pair_row_bits(shape, num_shared: int = 0) -> int:
    """32 or 16: width of the pair rows inside the fused entry points; 0 = unsupported shape."""
    s = _shape(shape)
    return int(load().beam_fused_pair_row_bits(ctypes.byref(s), int(num_shared)))


def beam_moe_block_forward(shape, num_shared, x, w_router, router_bias, w_mask, mask_bias,
                           w_gate_up, w_down, w_shared_gate, residual, out, topk_ids_opt,
                           topk_weights_opt, masked_ids_opt, num_pairs_opt, workspace,
                           workspace_bytes, hip_stream=None, check: bool = True) -> int:
    s = _shape(shape)
    st = load().beam_moe_block_forward(ctypes.byref(s), int(num_shared), _p(x), _p(w_router),
                                       _p(router_bias), _p(w_mask), _p(mask_bias),
                                       _p(w_gate_up), _p(w_down), _p(w_shared_gate),
                                       _p(residual), _p(out), _p(topk_ids_opt),
                                       _p(topk_weights_opt), _p(masked_ids_opt),
                                       _p(num_pairs_opt), _p(workspace), int(workspace_bytes),
                                       _p(hip_stream))
    return _check("beam_moe_block_forward", st, check)


def beam_moe_forward_timed(shape, x, w_router, router_bias, w_mask, mask_bias, w_gate_up, w_down,
                           out, workspace, workspace_bytes, hip_stream=None, check: bool = True):
    """-> (status, [ms per stage]); synchronises the stream (measurement aid)."""
    s = _shape(shape)
    ms = (ctypes.c_float * BEAM_NUM_STAGES)()
    st = load().beam_moe_forward_timed(ctypes.byref(s), _p(x), _p(w_router), _p(router_bias),
                                       _p(w_mask), _p(mask_bias), _p(w_gate_up), _p(w_down),
                                       _p(out), _p(workspace), int(workspace_bytes),
                                       _p(hip_stream), ms)
    return _check("beam_moe_forward_timed", st, check), [float(v) for v in ms]


def beam_moe_block_forward_timed(shape, num_shared, x, w_router, router_bias, w_mask, mask_bias,
                                 w_gate_up, w_down, w_shared_gate, residual, out, workspace,
                                 workspace_bytes, hip_stream=None, check: bool = True):
    """-> (status, [ms per stage]); synchronises the stream (measurement aid)."""
    s = _shape(shape)
    ms = (ctypes.c_float * BEAM_NUM_STAGES)()
    st = load().beam_moe_block_forward_timed(
        ctypes.byref(s), int(num_shared), _p(x), _p(w_router), _p(router_bias), _p(w_mask),
        _p(mask_bias), _p(w_gate_up), _p(w_down), _p(w_shared_gate), _p(residual), _p(out),
        _p(workspace), int(workspace_bytes), _p(hip_stream), ms)
    return _check("beam_moe_block_forward_timed", st, check), [float(v) for v in ms]


def _rule(rule):
    """None, a beam_rule, or a (kind, param) pair -> ctypes argument."""
    if rule is None:
        return None
    if not isinstance(rule, beam_rule):
        rule = beam_rule(int(rule[0]), float(rule[1]))
    return ctypes.byref(rule)


def beam_route_rule(shape, rule, x, w_router, router_bias, w_mask, mask_bias, topk_ids,
                    topk_weights, masked_ids, router_logits_dbg, mask_logits_dbg, workspace,
                    workspace_bytes, hip_stream=None, check: bool = True) -> int:
    s = _shape(shape)
    st = load().beam_route_rule(ctypes.byref(s), _rule(rule), _p(x), _p(w_router),
                                _p(router_bias), _p(w_mask), _p(mask_bias), _p(topk_ids),
                                _p(topk_weights), _p(masked_ids), _p(router_logits_dbg),
                                _p(mask_logits_dbg), _p(workspace), int(workspace_bytes),
                                _p(hip_stream))
    return _check("beam_route_rule", st, check)


def beam_moe_forward_rule(shape, rule, x, w_router, router_bias, w_mask, mask_bias, w_gate_up,
                          w_down, out, topk_ids_opt, topk_weights_opt, masked_ids_opt,
                          num_pairs_opt, workspace, workspace_bytes, hip_stream=None,
                          check: bool = True) -> int:
    s = _shape(shape)
    st = load().beam_moe_forward_rule(ctypes.byref(s), _rule(rule), _p(x), _p(w_router),
                                      _p(router_bias), _p(w_mask), _p(mask_bias), _p(w_gate_up),
                                      _p(w_down), _p(out), _p(topk_ids_opt),
                                      _p(topk_weights_opt), _p(masked_ids_opt),
                                      _p(num_pairs_opt), _p(workspace), int(workspace_bytes),
                                      _p(hip_stream))
    return _check("beam_moe_forward_rule", st, check)


def beam_mask_router_backward(shape, x, topk_ids, topk_weights, mask_logits, y_pairs,
                              expert_offsets, perm, inv_perm, grad_out, reg_coeff, grad_a,
                              grad_w_mask, loss_reg, workspace, workspace_bytes, hip_stream=None,
                              check: bool = True) -> int:
    s = _shape(shape)
    st = load().beam_mask_router_backward(
        ctypes.byref(s), _p(x), _p(topk_ids), _p(topk_weights), _p(mask_logits), _p(y_pairs),
        _p(expert_offsets), _p(perm), _p(inv_perm), _p(grad_out), ctypes.c_float(reg_coeff),
        _p(grad_a), _p(grad_w_mask), _p(loss_reg), _p(workspace), int(workspace_bytes),
        _p(hip_stream))
    return _check("beam_mask_router_backward", st, check)


def beam_probe_stream_read(buf, nbytes, sink, hip_stream=None, check: bool = True):
    """-> (status, bytes the probe kernel reads); measurement aid."""
    n = ctypes.c_size_t(0)
    st = load().beam_probe_stream_read(_p(buf), int(nbytes), _p(sink), _p(hip_stream),
                                       ctypes.byref(n))
    return _check("beam_probe_stream_read", st, check), int(n.value)


def beam_probe_mfma(iters, sink, hip_stream=None, check: bool = True):
    """-> (status, flops the probe kernel performs); measurement aid."""
    f = ctypes.c_double(0.0)
    st = load().beam_probe_mfma(int(iters), _p(sink), _p(hip_stream), ctypes.byref(f))
    return _check("beam_probe_mfma", st, check), float(f.value)

"""Host side of the C ABI: runs without a GPU.  The library must load, export
every function include/beam.h declares, size its workspace sanely and reject
bad arguments before anything is enqueued (no compute calls here)."""
import ctypes
import os
import re

import pytest

import paper_2605_14438_amd as beam
from paper_2605_14438_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if build.is_stale():
        build.build()
    return binding.load()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "beam.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(beam_[a-z_]+)\s*\(", text)))


def test_header_functions_are_exported(lib):
    names = _declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    raw = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        getattr(raw, n)          # raises AttributeError if the symbol is missing


def test_binding_exposes_the_same_names():
    for n in binding.EXPORTS:
        assert callable(getattr(beam, n)), n


def test_status_strings(lib):
    seen = {beam.beam_status_string(c) for c in range(5)}
    assert len(seen) == 5 and all(seen)
    assert beam.beam_abi_version() >= 1


def test_workspace_bytes(lib):
    s = beam.make_shape(64, 2048, 128, 8, 768, beam.BEAM_BF16)
    small = beam.beam_workspace_bytes(s)
    big = beam.beam_workspace_bytes(beam.make_shape(16384, 2048, 128, 8, 768, beam.BEAM_BF16))
    assert 0 < small < big
    # dominated by y_pairs [T*K,H] fp32 and hidden [T*K,I]
    assert big >= 16384 * 8 * (2048 * 4 + 768 * 2)
    assert big < 1.3 * 16384 * 8 * (2048 * 4 + 768 * 2)
    assert beam.beam_workspace_bytes(beam.make_shape(0, 256, 8, 2, 512, beam.BEAM_F32)) > 0
    # invalid / unsupported shapes -> 0
    assert beam.beam_workspace_bytes(beam.make_shape(4, 256, 8, 9, 512, beam.BEAM_F32)) == 0
    assert beam.beam_workspace_bytes(beam.make_shape(4, 256, 512, 2, 512, beam.BEAM_F32)) == 0


def test_workspace_covers_the_split_reductions(lib):
    """Shapes whose fused layer cuts a reduction into parts need one array per part:
    the down projection of few experts with a long reduction (four [T*K,H] arrays) and
    the prefill logits GEMM with fewer items than CUs (up to four [T,2N] arrays)."""
    T, H, N, K, I = 512, 4096, 8, 2, 14336                    # Mixtral-shaped, packed
    s = beam.make_shape(T, H, N, K, I, beam.BEAM_BF16, binding.BEAM_WEIGHTS_PACKED)
    assert beam.beam_workspace_bytes(s) >= 4 * T * K * H * 4 + T * K * I * 2
    # four times the tokens: more than 512 down-GEMM items possible, the reduction stays whole
    s4 = beam.make_shape(4 * T, H, N, K, I, beam.BEAM_BF16, binding.BEAM_WEIGHTS_PACKED)
    assert beam.beam_workspace_bytes(s4) < 2 * (4 * T) * K * (H * 4 + I * 2)
    q = beam.make_shape(1024, 2048, 128, 8, 768, beam.BEAM_BF16)   # 16 logits items -> 4 parts
    assert beam.beam_workspace_bytes(q) >= 4 * 1024 * 256 * 4 + 1024 * 8 * (2048 * 4 + 768 * 2)


def _logits_parts(T, H, N):
    """Parts the prefill logits product cuts its reduction into, as documented for the
    kernel: 64-row tiles x 256-column tiles are its items; the parts double (up to 4)
    while twice the items still fit 256 compute units and the 128-wide reduction steps
    divide evenly."""
    if T <= 512 or H % 256:
        return 1
    items = -(-T // 64) * -(-2 * N // 256)
    k = 1
    while k < 4 and items * k * 2 <= 256 and (H // 128) % (2 * k) == 0:
        k *= 2
    return k


def test_logits_region_holds_the_parts_of_the_routed_shape(lib):
    """The block entry point sizes the workspace for N + S experts, but the logits product
    and Top-K run on the N routed experts and cut the reduction by THEIR column count:
    the region must hold that many [T, 2N] arrays, for every (N, S, T)."""
    worst = 0
    for H in (2048, 512):
        for N in (8, 60, 64, 120, 126, 127, 128, 200):
            for S in (0, 1, 2, 4, 10):
                if N + S > 256:
                    continue
                for T in (513, 1024, 2048, 2049, 4096, 4097, 6000, 8192, 8193, 16384):
                    s = beam.make_shape(T, H, N, 4, 256, beam.BEAM_BF16)
                    st, off, nbytes, parts = beam.beam_workspace_logits_region(s, S)
                    assert st == binding.BEAM_OK and off % 256 == 0
                    need = _logits_parts(T, H, N)
                    worst = max(worst, need)
                    assert parts >= need and parts >= _logits_parts(T, H, N + S)
                    assert nbytes >= need * T * 2 * N * 4, (H, N, S, T)
                    assert off + nbytes <= beam.beam_block_workspace_bytes(s, S)
    assert worst == 4
    # the case that used to overflow: 4 parts of [4096, 256] fp32 where N + S gave room for 2
    s = beam.make_shape(4096, 2048, 128, 8, 768, beam.BEAM_BF16)
    _, _, nbytes, parts = beam.beam_workspace_logits_region(s, 1)
    assert parts == 4 and nbytes >= 4 * 4096 * 256 * 4
    assert beam.beam_workspace_logits_region(s, 200, check=False)[0] == binding.BEAM_ERR_UNSUPPORTED
    bad = beam.make_shape(4, 256, 8, 9, 512, beam.BEAM_F32)
    assert beam.beam_workspace_logits_region(bad, 0, check=False)[0] == binding.BEAM_ERR_INVALID_ARG


def test_fused_pair_row_bits_follow_the_documented_rule(lib):
    """Half-precision pair rows inside the fused layer exactly where the header says: bf16, the
    tiled GEMM on the host's word (256 rows per expert or more in the worst case), a whole
    down reduction, and T*K*H fp32 rows that fill the 256 MiB last-level cache or more."""
    mk = beam.make_shape
    q = dict(H=2048, N=128, K=8, I=768)
    def bits(T, S=0, dtype=beam.BEAM_BF16, layout=beam.BEAM_WEIGHTS_PACKED, **kw):
        d = {**q, **kw}
        return beam.beam_fused_pair_row_bits(mk(T, d["H"], d["N"], d["K"], d["I"], dtype, layout), S)
    assert bits(16384) == 16 and bits(4096) == 16           # 4096 * 8 * 2048 * 4 B = 256 MiB
    assert bits(4095) == 32
    assert bits(64) == 32 and bits(1) == 32
    assert bits(16384, layout=beam.BEAM_WEIGHTS_PLAIN) == 16
    assert bits(16384, dtype=beam.BEAM_F32, layout=beam.BEAM_WEIGHTS_PLAIN) == 32
    assert bits(4000, S=1) == 16                            # 9 slots per token with a shared block
    assert bits(8192, H=4096, I=1536) == 16 and bits(2048, H=4096, I=1536) == 32
    # few experts with a long reduction: the fused layer splits the down reduction, fp32 parts
    assert bits(2048, H=4096, N=8, K=2, I=14336) == 32
    assert bits(16384, H=320, N=60, K=4, I=136, layout=beam.BEAM_WEIGHTS_PLAIN) == 32   # generic kernels
    assert bits(4, K=9, N=8) == 0 and bits(16384, S=200) == 0                           # invalid shapes


def test_residual_must_not_overlap_the_output(lib):
    s = beam.make_shape(4, 256, 8, 2, 512, beam.BEAM_F32)
    ok, big = 0x100000, 1 << 40
    nbytes = 4 * 256 * 4

    def block(res, out):
        return beam.beam_moe_block_forward(s, 0, ok, ok, None, ok, None, ok, ok, None, res, out,
                                           None, None, None, None, ok, big, check=False)
    out = 0x200000
    assert block(out, out) == binding.BEAM_ERR_INVALID_ARG
    assert block(out + nbytes - 16, out) == binding.BEAM_ERR_INVALID_ARG
    assert block(out - nbytes + 16, out) == binding.BEAM_ERR_INVALID_ARG


@pytest.mark.parametrize("shape,code", [
    ((-1, 256, 8, 2, 512, 0), binding.BEAM_ERR_INVALID_ARG),
    ((4, 256, 8, 0, 512, 0), binding.BEAM_ERR_INVALID_ARG),
    ((4, 256, 8, 9, 512, 0), binding.BEAM_ERR_INVALID_ARG),
    ((4, 256, 8, 2, 512, 7), binding.BEAM_ERR_INVALID_ARG),
    ((4, 256, 8, 2, 512, 1, 5), binding.BEAM_ERR_INVALID_ARG),       # unknown weight layout
    ((4, 256, 8, 2, 512, 0, 1), binding.BEAM_ERR_UNSUPPORTED),       # packed needs bf16
    ((4, 320, 8, 2, 512, 1, 1), binding.BEAM_ERR_UNSUPPORTED),       # packed needs H % 256 == 0
    ((4, 250, 8, 2, 512, 0), binding.BEAM_ERR_UNSUPPORTED),
    ((4, 256, 300, 2, 512, 0), binding.BEAM_ERR_UNSUPPORTED),
    ((4, 256, 8, 2, 511, 1), binding.BEAM_ERR_UNSUPPORTED),
    ((1 << 22, 256, 8, 4, 512, 1), binding.BEAM_ERR_UNSUPPORTED),
])
def test_bad_shapes_are_rejected_on_the_host(lib, shape, code):
    s = beam.make_shape(*shape)
    fake = 0x1000      # never dereferenced: shape checks come first
    assert beam.beam_route_mask(s, fake, fake, None, fake, None, fake, fake, fake, None, None,
                                fake, 1 << 40, check=False) == code
    assert beam.beam_permute(s, fake, fake, fake, fake, fake, fake, fake, 1 << 40,
                             check=False) == code
    assert beam.beam_expert_ffn(s, fake, fake, fake, fake, fake, fake, fake, fake, 1 << 40,
                                check=False) == code
    assert beam.beam_combine(s, fake, fake, fake, fake, fake, check=False) == code
    assert beam.beam_moe_forward(s, fake, fake, None, fake, None, fake, fake, fake, None, None,
                                 None, None, fake, 1 << 40, check=False) == code


def test_null_misaligned_and_small_workspace(lib):
    s = beam.make_shape(4, 256, 8, 2, 512, beam.BEAM_F32)
    need = beam.beam_workspace_bytes(s)
    ok = 0x1000
    # NULL required pointer
    assert beam.beam_moe_forward(s, None, ok, None, ok, None, ok, ok, ok, None, None, None, None,
                                 ok, need, check=False) == binding.BEAM_ERR_INVALID_ARG
    assert beam.beam_route_mask(s, ok, ok, None, ok, None, None, ok, ok, None, None, ok, need,
                                check=False) == binding.BEAM_ERR_INVALID_ARG
    assert beam.beam_combine(s, ok, ok, ok, ok, None, check=False) == binding.BEAM_ERR_INVALID_ARG
    # misaligned x
    assert beam.beam_moe_forward(s, ok + 4, ok, None, ok, None, ok, ok, ok, None, None, None,
                                 None, ok, need, check=False) == binding.BEAM_ERR_INVALID_ARG
    # workspace one byte short / missing
    assert beam.beam_moe_forward(s, ok, ok, None, ok, None, ok, ok, ok, None, None, None, None,
                                 ok, need - 1, check=False) == binding.BEAM_ERR_WORKSPACE
    assert beam.beam_permute(s, ok, ok, ok, ok, ok, ok, ok, need - 1,
                             check=False) == binding.BEAM_ERR_WORKSPACE
    assert beam.beam_expert_ffn(s, ok, ok, ok, ok, ok, ok, ok, None, need,
                                check=False) == binding.BEAM_ERR_INVALID_ARG
    with pytest.raises(beam.BeamError):
        beam.beam_combine(s, None, ok, ok, ok, ok)


def test_pack_weights_argument_checks(lib):
    ok = 0x1000
    s = beam.make_shape(0, 256, 8, 2, 512, beam.BEAM_BF16)
    assert beam.beam_pack_weights(s, ok, ok, None, ok + 0x100, check=False) == \
        binding.BEAM_ERR_INVALID_ARG
    assert beam.beam_pack_weights(s, ok, ok, ok, ok, check=False) == binding.BEAM_ERR_INVALID_ARG
    s32 = beam.make_shape(0, 256, 8, 2, 512, beam.BEAM_F32)
    assert beam.beam_pack_weights(s32, ok, ok, ok + 0x100, ok + 0x200, check=False) == \
        binding.BEAM_ERR_UNSUPPORTED
    assert beam.beam_abi_version() == 3


def test_zero_tokens_is_ok_without_launch(lib):
    s = beam.make_shape(0, 256, 8, 2, 512, beam.BEAM_F32)
    need = beam.beam_workspace_bytes(s)
    ok = 0x1000
    assert beam.beam_moe_forward(s, ok, ok, None, ok, None, ok, ok, ok, None, None, None, None,
                                 ok, need, check=False) == binding.BEAM_OK
    assert beam.beam_route_mask(s, ok, ok, None, ok, None, ok, ok, ok, None, None, ok, need,
                                check=False) == binding.BEAM_OK
    assert beam.beam_combine(s, ok, ok, ok, ok, ok, check=False) == binding.BEAM_OK


def test_newer_entry_points_check_arguments_on_the_host(lib):
    """Block (App. A.3), activation-rule and mask-router-backward entry points: every
    check happens before anything is enqueued, so fake pointers are never touched."""
    ok = 0x1000
    bad, unsup, short = (binding.BEAM_ERR_INVALID_ARG, binding.BEAM_ERR_UNSUPPORTED,
                         binding.BEAM_ERR_WORKSPACE)
    s = beam.make_shape(4, 256, 8, 2, 512, beam.BEAM_F32)
    s0 = beam.make_shape(0, 256, 8, 2, 512, beam.BEAM_F32)
    big = 1 << 40

    def block(shape, S, gate=None, res=None, ws_bytes=big, x=ok):
        return beam.beam_moe_block_forward(shape, S, x, ok, None, ok, None, ok, ok, gate, res, ok,
                                           None, None, None, None, ok, ws_bytes, check=False)
    assert beam.beam_block_workspace_bytes(s, 0) == beam.beam_workspace_bytes(s)
    assert beam.beam_block_workspace_bytes(s, 3) > beam.beam_workspace_bytes(s)
    assert beam.beam_block_workspace_bytes(s, -1) == 0
    assert beam.beam_block_workspace_bytes(s, 249) == 0          # N + S > 256
    assert block(s, -1) == bad
    assert block(s, 249) == unsup
    assert block(s, 0, gate=ok) == bad                           # gate vector without a shared expert
    assert block(s, 2, gate=ok + 2) == bad and block(s, 2, res=ok + 2) == bad    # misaligned
    assert block(s, 2, ws_bytes=beam.beam_block_workspace_bytes(s, 2) - 1) == short
    assert block(s, 2, x=None) == bad
    assert block(s0, 2, gate=ok, res=ok) == binding.BEAM_OK      # T = 0: nothing to do

    def fwd_rule(rule, shape=s0, w_mask=ok):
        return beam.beam_moe_forward_rule(shape, rule, ok, ok, None, w_mask, None, ok, ok, ok, None,
                                          None, None, None, ok, big, check=False)
    assert fwd_rule(None) == bad
    assert fwd_rule((5, 0.0)) == bad and fwd_rule((binding.BEAM_RULE_MASK, float("nan"))) == bad
    assert fwd_rule((binding.BEAM_RULE_MASK, 0.0), w_mask=None) == bad
    assert fwd_rule((binding.BEAM_RULE_CUMPROB, 0.3), w_mask=None) == binding.BEAM_OK
    assert fwd_rule((binding.BEAM_RULE_MASK, -1.5)) == binding.BEAM_OK

    def backward(shape=s, grad_out=ok, reg=0.1, ws_bytes=big, grad_w=ok):
        return beam.beam_mask_router_backward(shape, ok, ok, ok, ok, ok, ok, ok, ok, grad_out, reg,
                                              ok, grad_w, ok, ok, ws_bytes, check=False)
    assert backward(grad_out=None) == bad
    assert backward(reg=float("nan")) == bad
    assert backward(grad_w=ok + 4) == bad
    assert backward(ws_bytes=16) == short
    assert backward(shape=s0) == binding.BEAM_OK
    assert backward(shape=beam.make_shape(4, 256, 8, 9, 512, beam.BEAM_F32)) == bad   # K > N


def test_probe_entry_points_check_arguments_on_the_host(lib):
    ok = 0x1000
    bad = binding.BEAM_ERR_INVALID_ARG
    assert beam.beam_probe_stream_read(None, 1 << 27, ok, check=False)[0] == bad
    assert beam.beam_probe_stream_read(ok, 1 << 27, None, check=False)[0] == bad
    assert beam.beam_probe_stream_read(ok + 4, 1 << 27, ok, check=False)[0] == bad    # misaligned
    assert beam.beam_probe_stream_read(ok, (1 << 26) - 1, ok, check=False)[0] == bad  # too small to time
    assert beam.beam_probe_mfma(0, ok, check=False)[0] == bad
    assert beam.beam_probe_mfma(10, None, check=False)[0] == bad


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2605_14438_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "beam_oracle" not in text, f

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


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2605_14438_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "beam_oracle" not in text, f

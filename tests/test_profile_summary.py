"""The profile summariser's host logic: which kernel belongs to which expert GEMM stage, which
source files a stage's traffic record is keyed by, and how the counter scale is taken from the
copies of known size in a counter run."""
import pytest

from paper_2605_14438_amd import profile_summary as ps


@pytest.mark.parametrize("name,stage", [
    ("void beam::ffn_tile_kernel<1, 4, 2, true, true>(unsigned short const*, int)", "gate_up"),
    ("void beam::ffn_tile_kernel<1, 4, 2, false, true>(unsigned short const*, int)", "down"),
    ("void beam::ffn_tile_kernel<1, 8, 1, true, true>(unsigned short const*)", "gate_up"),
    ("beam::gate_up_stream_packed_kernel(unsigned short const*)", "gate_up"),
    ("void beam::gate_up_slot_packed_kernel<0>(unsigned short const*)", "gate_up"),
    ("beam::down_stream_packed_kernel(unsigned short const*)", "down"),
    ("void beam::down_stream_kernel<2>(unsigned short const*)", "down"),
    ("void beam::down_combine_token_packed_kernel<0>(unsigned short const*)", "down"),
    ("void beam::combine_wave_kernel<unsigned short, 8>(float const*)", None),
    ("void beam::topk_mask_kernel<0>(float const*)", None),
    ("beam::logits_tile_kernel(unsigned short const*)", None),
    ("__amd_rocclr_copyBuffer", None),
])
def test_stage_of(name, stage):
    assert ps.stage_of(name) == stage


def test_sources_follow_the_kernel_family():
    common = "paper_2605_14438_amd/csrc/common.hpp"
    assert ps.sources_of(["beam::gate_up_stream_packed_kernel(x)"]) == [
        common, "paper_2605_14438_amd/csrc/ffn_stream.hip"]
    assert ps.sources_of(["void beam::ffn_tile_kernel<1, 4, 2, true, true>(x)"]) == [
        common, "paper_2605_14438_amd/csrc/ffn_tiled.hip"]
    # a device-chosen launch enqueues both families: both files key the record
    both = ps.sources_of(["beam::gate_up_stream_packed_kernel(x)",
                          "void beam::ffn_tile_kernel<1, 8, 1, true, true>(x)"])
    assert both == [common, "paper_2605_14438_amd/csrc/ffn_stream.hip",
                    "paper_2605_14438_amd/csrc/ffn_tiled.hip"]
    assert len(ps.sha16(both)) == 16


def test_copy_scale_uses_the_largest_copies_only():
    # five probe copies of 1 GiB read as half their size (the counter's unit on this GPU), among
    # smaller housekeeping copies
    copies = [524300.0, 524299.0, 524301.5, 524300.5, 524299.5, 1024.0, 393216.0, 16.0]
    scale, raw = ps.copy_scale(copies, 1048576.0, "FETCH_SIZE")
    assert abs(raw - 524300.1) < 1.0 and abs(scale - 2.0) < 1e-4
    with pytest.raises(SystemExit):
        ps.copy_scale([], 1048576.0, "FETCH_SIZE")

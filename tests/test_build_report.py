"""The compiler's own resource report for the device code (CPU only: hipcc cross-compiles without a GPU): no kernel
of the library may use scratch memory -- a register spill in a KV-streaming kernel costs it the very loads it is
built to keep in flight -- and the streaming kernels must fit two waves per SIMD (256 registers per lane)."""
import pytest

from paper_2602_07223_amd import build


@pytest.fixture(scope="module")
def usage():
    u = build.kernel_resource_usage()
    assert u, "the compiler printed no resource report"
    return u


def test_no_kernel_spills_registers(usage):
    spilled = {k: v["scratch_bytes_per_lane"] for k, v in usage.items() if v.get("scratch_bytes_per_lane", 0) != 0}
    assert not spilled, f"kernels with scratch (bytes per lane): {spilled}"


def test_streaming_kernels_fit_two_waves_per_simd(usage):
    streaming = {k: v for k, v in usage.items() if "attn_split_kernel" in k or "attn_pair_kernel" in k or "attn_draft16_kernel" in k}
    assert len(streaming) >= 32                      # every instantiation the launch code can pick is in the report
    for name, v in streaming.items():
        assert v["vgprs"] + v.get("agprs", 0) <= 256, (name, v)
        assert v["occupancy"] >= 2, (name, v)

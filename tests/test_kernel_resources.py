"""Build-time check of the registers the compiler gives the block kernels (CPU only: hipcc cross-compiles).

The headline kernel keeps 128 state registers per lane and runs two waves per SIMD, so it sits at the
256-register limit: a change that pushes values into scratch memory inside the token loop would cost time on
every block without failing any numerical test.  The compiler's own resource remarks are parsed here."""
import os
import re

import pytest

from paper_2605_11196_amd import build

CSRC = os.path.join(os.path.dirname(os.path.abspath(build.__file__)), "csrc")


@pytest.fixture(scope="module")
def chunk_usage():
    use = build.resource_usage(os.path.join(CSRC, "vla_chunk.hip"))
    out = {}
    for name, r in use.items():
        m = re.search(r"chunk_kernel<(\d+), (\d+), (\d+), ([\w ]+), (true|false)>", name)
        if m:
            out[(int(m.group(1)), int(m.group(2)), "bf16" if "short" in m.group(4) else "f32",
                 m.group(5) == "true")] = r
    return out


def test_every_block_kernel_instantiation_is_reported(chunk_usage):
    for d in (16, 32, 64, 96, 128):
        for io in ("bf16", "f32"):
            for fmap in (False, True):
                assert (d, d, io, fmap) in chunk_usage


@pytest.mark.parametrize("d", [16, 32, 64, 96, 128])
def test_bf16_block_kernels_use_no_scratch_and_keep_two_waves_per_simd(chunk_usage, d):
    """bf16 I/O is what the large-batch and long-context workloads run."""
    for fmap in (False, True):
        r = chunk_usage[(d, d, "bf16", fmap)]
        assert r["ScratchSize"] == 0 and r["VGPRSpill"] == 0, r
        assert r["VGPRs"] + r.get("AGPRs", 0) <= 256 and r["Occupancy"] >= 2, r


def test_float32_io_kernels_stay_within_their_known_spills(chunk_usage):
    """With float32 I/O the staged rows take twice the registers: at d = 128 the compiler keeps two addresses in
    scratch (reloaded, never stored, inside the loop); nothing else spills."""
    for d in (16, 32, 64, 96):
        for fmap in (False, True):
            assert chunk_usage[(d, d, "f32", fmap)]["ScratchSize"] == 0
    for fmap in (False, True):
        r = chunk_usage[(128, 128, "f32", fmap)]
        assert r["ScratchSize"] <= 12 and r["VGPRSpill"] <= 2 and r["Occupancy"] >= 2, r


def test_headline_kernel_fits_two_workgroups_per_compute_unit(chunk_usage):
    r = chunk_usage[(128, 128, "bf16", False)]
    assert 2 * r["LDSSize"] <= 160 * 1024

"""Host-side check of the register allocation of the kernels that count their loads.

The M <= 16 stream kernels, the paper-literal tile kernel and the 256 x 256 tile kernel issue their loads from assembly
and wait for them with exact `vmcnt` counts.  A register spill would add scratch loads and
stores that the counts do not know about, so the build must not spill in these kernels (and
the gfx950 code objects of those files must not contain scratch accesses at all).
"""
import os
import re
import shutil
import subprocess

import pytest

from paper_2309_16119_amd import build

SRC = os.path.join(build.CSRC, "smallm.hip")


def _hipcc():
    for cand in ("/opt/rocm/bin/hipcc", shutil.which("hipcc")):
        if cand and os.path.exists(cand):
            return cand
    return None


@pytest.mark.skipif(_hipcc() is None, reason="hipcc not available")
def test_stream_kernels_do_not_spill(tmp_path):
    out = tmp_path / "smallm.s"
    cmd = [_hipcc(), *build.HIPCC_FLAGS, "-S", "--cuda-device-only", SRC, "-o", str(out)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    text = out.read_text()
    names = re.findall(r"^\s*\.name:\s+(\S+)", text, flags=re.M)
    spills = re.findall(r"^\s*\.vgpr_spill_count:\s+(\d+)", text, flags=re.M)
    sgpr_spills = re.findall(r"^\s*\.sgpr_spill_count:\s+(\d+)", text, flags=re.M)
    kernels = [n for n in names if "smallm_" in n]
    assert len(kernels) >= 11, kernels          # 6 forward, 3 backward, 2 finish kernels
    assert len(spills) == len(names)
    for name, v, s in zip(names, spills, sgpr_spills):
        assert int(v) == 0 and int(s) == 0, "%s spills (%s vector, %s scalar registers)" % (name, v, s)
    assert "scratch_load" not in text and "scratch_store" not in text
    # two forward workgroups (stream + projection) must fit one compute unit: at most 128 registers
    counts = dict(zip(names, re.findall(r"^\s*\.vgpr_count:\s+(\d+)", text, flags=re.M)))
    for name, c in counts.items():
        if "smallm_fwd_kernel" in name:
            assert int(c) <= 128, (name, c)


@pytest.mark.skipif(_hipcc() is None, reason="hipcc not available")
def test_f16_tile_kernels_do_not_spill(tmp_path):
    out = tmp_path / "f16_path.s"
    cmd = [_hipcc(), *build.HIPCC_FLAGS, "-S", "--cuda-device-only", os.path.join(build.CSRC, "f16_path.hip"), "-o", str(out)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    text = out.read_text()
    names = re.findall(r"^\s*\.name:\s+(\S+)", text, flags=re.M)
    spills = re.findall(r"^\s*\.vgpr_spill_count:\s+(\d+)", text, flags=re.M)
    assert sum("f16_gemm_kernel" in n for n in names) == 12       # 3 bit widths x forward / backward x 2 tile heights
    for name, v in zip(names, spills):
        assert int(v) == 0, "%s spills %s vector registers" % (name, v)
    assert "scratch_load" not in text and "scratch_store" not in text


@pytest.mark.skipif(_hipcc() is None, reason="hipcc not available")
def test_large_m_tile_kernel_does_not_spill(tmp_path):
    """The 256 x 256 kernel waits for its assembly-issued loads by count and keeps staged registers
    untouched while their loads are in flight: no spills, no scratch accesses."""
    out = tmp_path / "gemm_big.s"
    cmd = [_hipcc(), *build.HIPCC_FLAGS, "-S", "--cuda-device-only", os.path.join(build.CSRC, "gemm_big.hip"), "-o", str(out)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    text = out.read_text()
    names = re.findall(r"^\s*\.name:\s+(\S+)", text, flags=re.M)
    spills = re.findall(r"^\s*\.vgpr_spill_count:\s+(\d+)", text, flags=re.M)
    # 3 bit widths x forward / backward x bfloat16 / binary16 x 256- / 128-row tiles
    assert sum("gemm_big_kernel" in n for n in names) == 24
    for name, v in zip(names, spills):
        assert int(v) == 0, "%s spills %s vector registers" % (name, v)
    assert "scratch_load" not in text and "scratch_store" not in text


@pytest.mark.skipif(_hipcc() is None, reason="hipcc not available")
def test_producer_consumer_tile_kernel_does_not_spill(tmp_path):
    """The 128 x 64 producer / consumer kernel counts its assembly-issued loads in both roles."""
    out = tmp_path / "gemm_mid.s"
    cmd = [_hipcc(), *build.HIPCC_FLAGS, "-S", "--cuda-device-only", os.path.join(build.CSRC, "gemm_mid.hip"), "-o", str(out)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    text = out.read_text()
    names = re.findall(r"^\s*\.name:\s+(\S+)", text, flags=re.M)
    spills = re.findall(r"^\s*\.vgpr_spill_count:\s+(\d+)", text, flags=re.M)
    assert sum("gemm_mid_kernel" in n for n in names) == 12       # 3 bit widths x forward / backward x bfloat16 / binary16
    for name, v in zip(names, spills):
        assert int(v) == 0, "%s spills %s vector registers" % (name, v)
    assert "scratch_load" not in text and "scratch_store" not in text

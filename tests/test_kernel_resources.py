"""What the compiler made of the decode kernels (CPU only: hipcc cross-compiles for gfx950).

A kernel whose tile registers end up in scratch memory, or that no longer fits two waves per SIMD,
still computes the right thing and silently loses half its bandwidth, so the resource remarks of
the compiler are checked: the decode kernels (range pass, its probe, split pass) and the 8-wave
causal kernel use no scratch memory and spill no vector registers, and keep at least two waves
per SIMD.
"""
import os
import re
import shutil
import subprocess

import pytest

from paper_2508_11553_amd import build as sd_build

CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2508_11553_amd", "csrc")


def resource_remarks(source, tmp_path):
    flags = [f for f in sd_build.FLAGS if f not in ("-shared", "-fPIC")]
    r = subprocess.run([sd_build.HIPCC, *flags, "--cuda-device-only", "-c", os.path.join(CSRC, source), "-o",
                        str(tmp_path / "dev.o"), "-Rpass-analysis=kernel-resource-usage"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    out, name = {}, None
    for line in r.stderr.splitlines():
        m = re.search(r"remark: .*Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            out[name] = {}
            continue
        m = re.search(r"remark: \s*([A-Za-z ]+?)(?: \[[^\]]*\])?: (\d+)", line)
        if m and name:
            out[name][m.group(1).strip()] = int(m.group(2))
    return out


@pytest.mark.skipif(shutil.which(sd_build.HIPCC) is None and not os.path.exists(sd_build.HIPCC), reason="needs hipcc")
@pytest.mark.parametrize("source,kernels,least", [("attn_range.hip", "range_kernel", 3), ("attn_split.hip", "split_kernel", 3),
                                                   ("attn_prefill.hip", "prefill_wide_kernel", 1)])
def test_decode_kernels_keep_their_tiles_in_registers(source, kernels, least, tmp_path):
    remarks = {k: v for k, v in resource_remarks(source, tmp_path).items() if kernels in k}
    assert len(remarks) >= least, list(remarks)
    for name, res in remarks.items():
        assert res["ScratchSize"] == 0, (name, res)
        assert res["VGPRs Spill"] == 0, (name, res)
        assert res["Occupancy"] >= 2, (name, res)

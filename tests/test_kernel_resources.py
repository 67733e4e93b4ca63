"""Register budgets that the measured kernel rates depend on, read from the compiler's resource remarks (no GPU needed).

k_pack_keys is written to fit three wavefronts per SIMD (at most 170 VGPRs on gfx950); a few more registers leave two and
the sweep runs 40 % slower, which no parity test would notice."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_key_sweep_keeps_three_wavefronts_per_simd(tmp_path):
    from paper_2009_13003_amd import build
    flags = [f for f in build.FLAGS if f != "-shared"]
    src = os.path.join(build.CSRC, "lc_encode.hip")
    res = subprocess.run(["hipcc"] + flags + ["--cuda-device-only", "-Rpass-analysis=kernel-resource-usage", "-c", "-o",
                                              str(tmp_path / "enc.o"), src], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    blocks = re.split(r"remark: Function Name: ", res.stderr)
    found = {}
    for b in blocks[1:]:
        name = b.split()[0]
        occ = re.search(r"Occupancy \[waves/SIMD\]: (\d+)", b)
        vgpr = re.search(r"VGPRs: (\d+)", b)
        if occ and vgpr:
            found[name] = (int(vgpr.group(1)), int(occ.group(1)))
    keys = [v for k, v in found.items() if "k_pack_keys" in k]
    assert keys, sorted(found)
    assert all(occ >= 3 for _, occ in keys), keys

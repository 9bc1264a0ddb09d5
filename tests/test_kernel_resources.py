"""Compile-time guard for the contraction kernels: the DistMult / ComplEx / Dot instantiations must not
spill registers (a spill inside the tile loop once halved the wide-row kernel's speed without failing any
numerical test).  Uses hipcc's resource-usage remarks; no GPU needed."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not (os.path.exists(HIPCC) or shutil.which("hipcc")), reason="hipcc not available")
def test_dot_product_contraction_kernels_do_not_spill(tmp_path):
    src = os.path.join(ROOT, "paper_2101_08358_amd", "csrc", "mar_flash.hip")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Rpass-analysis=kernel-resource-usage", "-c", src, "-o", str(tmp_path / "flash.o")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    blocks = re.split(r"remark: Function Name: ", r.stderr)[1:]
    seen = 0
    for b in blocks:
        name = b.split()[0]
        if "k_flash" not in name or not name.endswith("ELi0EEv9FlashArgs"):      # last template argument: TransE = 1
            continue
        seen += 1
        spill = int(re.search(r"VGPRs Spill: (\d+)", b).group(1))
        scratch = int(re.search(r"ScratchSize \[bytes/lane\]: (\d+)", b).group(1))
        assert spill == 0 and scratch == 0, (name, spill, scratch)
    assert seen >= 10


@pytest.mark.skipif(not (os.path.exists(HIPCC) or shutil.which("hipcc")), reason="hipcc not available")
def test_split_precision_kernels_do_not_spill(tmp_path):
    src = os.path.join(ROOT, "paper_2101_08358_amd", "csrc", "mar_split.hip")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Rpass-analysis=kernel-resource-usage", "-c", src, "-o", str(tmp_path / "split.o")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    blocks = re.split(r"remark: Function Name: ", r.stderr)[1:]
    seen = 0
    for b in blocks:
        name = b.split()[0]
        if "k_split" not in name:
            continue
        seen += 1
        spill = int(re.search(r"VGPRs Spill: (\d+)", b).group(1))
        scratch = int(re.search(r"ScratchSize \[bytes/lane\]: (\d+)", b).group(1))
        assert spill == 0 and scratch == 0, (name, spill, scratch)
    assert seen >= 12

"""The compiled kernels' resources, read from the compiler's own report (no GPU needed): no kernel
may spill registers or use scratch memory (the runtime would allocate scratch for a queue at the
kernel's first launch, behind the back of the entry point that promises to allocate nothing),
none may contain a packed-fp32 VALU instruction, and the MFMA shrink must leave room for two
workgroups per compute unit."""
import os
import re
import shutil
import subprocess

import pytest

from paper_2311_03285_amd import build as hip_build

pytestmark = pytest.mark.skipif(shutil.which(hip_build.HIPCC) is None and not os.path.exists(hip_build.HIPCC),
                                reason="no hipcc")


@pytest.fixture(scope="module")
def report(tmp_path_factory):
    d = tmp_path_factory.mktemp("res")
    src = os.path.join(hip_build.CSRC, "kernels.hip")
    asm = str(d / "kernels.s")
    r = subprocess.run([hip_build.HIPCC] + hip_build.FLAGS + ["-x", "hip", "--cuda-device-only", "-S", src, "-o", asm,
                                                              "-Rpass-analysis=kernel-resource-usage"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    kernels = {}
    name = None
    for line in r.stderr.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            kernels[name] = {}
            continue
        m = re.search(r"remark:\s+([A-Za-z ]+?)(?: \[[^\]]*\])?: (\d+)", line)
        if m and name:
            kernels[name][m.group(1).strip()] = int(m.group(2))
    return kernels, open(asm).read()


def test_no_kernel_spills_or_uses_scratch(report):
    kernels, _ = report
    ours = {k: v for k, v in kernels.items() if "slora" in k}
    assert len(ours) >= 10, sorted(kernels)
    for k, v in ours.items():
        assert v.get("ScratchSize", 0) == 0, (k, v)
        assert v.get("VGPRs Spill", 0) == 0 and v.get("SGPRs Spill", 0) == 0, (k, v)


def test_mfma_shrink_fits_two_workgroups_per_compute_unit(report):
    kernels, _ = report
    ms = {k: v for k, v in kernels.items() if "shrink_mfma_kernel" in k}
    assert len(ms) == 2
    for k, v in ms.items():
        assert v["VGPRs"] + v.get("AGPRs", 0) <= 256, (k, v)   # 512 registers per SIMD lane, 4 wavefronts per workgroup


def test_no_packed_fp32_instructions(report):
    _, asm = report
    assert not re.search(r"\bv_pk_(add|mul|fma)_f32\b", asm)

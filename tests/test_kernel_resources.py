"""CPU-only: no GEMM kernel spills registers.

The DMA GEMM kernels keep 128 accumulators and two sets of operand fragments per lane and sit at (or just under) the 256
registers two wavefronts per SIMD can have.  A spill there costs far more than its few instructions: scratch reloads count
in the same in-order vector-memory counter as the global-to-LDS copies, so waiting for one waits for every copy issued before
it.  The compiler reports each kernel's scratch size; this test compiles the GEMM source for the device only and checks it."""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

from paper_2603_22370_amd import build as fbuild


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="needs hipcc")
def test_no_gemm_kernel_uses_scratch_memory():
    src = os.path.join(fbuild.CSRC, "faar_gemm.hip")
    with tempfile.TemporaryDirectory() as tmp:
        cmd = [fbuild.hipcc(), *fbuild.HIPCC_FLAGS, "--cuda-device-only", "-Rpass-analysis=kernel-resource-usage",
               "-c", src, "-o", os.path.join(tmp, "gemm.o")]
        r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    kernels = {}
    for block in re.split(r"remark: Function Name: ", r.stderr)[1:]:
        name = block.split()[0]
        scratch = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", block)
        vgprs = re.search(r" VGPRs: (\d+)", block)
        if scratch and vgprs:
            kernels[name] = (int(scratch.group(1)), int(vgprs.group(1)))
    dma = {k: v for k, v in kernels.items() if "k_gemm_dma" in k}
    assert len(dma) >= 30, len(dma)                      # every tile shape x epilogue instantiation was seen
    assert any("Dma64CfgILi192ELi256" in k for k in dma) and any("Dma64CfgILi256ELi192" in k for k in dma)
    spilling = {k: v for k, v in dma.items() if v[0] != 0}
    assert not spilling, spilling
    assert max(v[1] for v in dma.values()) <= 256

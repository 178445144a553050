"""No kernel of the library spills registers to scratch memory.

The step kernels are written to the register budget of their occupancy (128 registers per lane at
16 wavefronts per workgroup for the resident kernel, 256 or 512 for the streaming ones); a helper
that grows by a few registers tips them over without any error, and the spill traffic then costs
several per cent of throughput.  The compiler reports the figures; this test reads them.
"""
import os
import re
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _resource_report(src, flags, hipcc, csrc):
    with tempfile.TemporaryDirectory() as tmp:
        cmd = [hipcc, *flags, "--cuda-device-only", "-Rpass-analysis=kernel-resource-usage", "-c",
               os.path.join(csrc, src), "-o", os.path.join(tmp, "dev.o")]
        out = subprocess.run(cmd, check=True, capture_output=True, text=True, timeout=600).stderr
    kernels, name = {}, None
    for line in out.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            kernels[name] = {}
            continue
        m = re.search(r"remark:\s+(VGPRs Spill|ScratchSize \[bytes/lane\]): (\d+)", line)
        if m and name:
            kernels[name][m.group(1)] = int(m.group(2))
    return kernels


def test_no_kernel_spills_registers():
    from paper_1810_08313_amd import build
    hipcc = build.HIPCC if os.path.exists(build.HIPCC) else shutil.which("hipcc")
    if not hipcc:
        pytest.skip("hipcc not available")
    sources = [s for s in build.SOURCES if s != "lc_api.hip"]   # lc_api.hip holds host code only
    with ThreadPoolExecutor(max_workers=len(sources)) as ex:
        reports = list(ex.map(lambda s: _resource_report(s, build.FLAGS, hipcc, build.CSRC), sources))
    seen = 0
    for src, kernels in zip(sources, reports):
        assert kernels, src
        for name, r in kernels.items():
            seen += 1
            assert r.get("VGPRs Spill", 0) == 0, (src, name, r)
            assert r.get("ScratchSize [bytes/lane]", 0) == 0, (src, name, r)
    assert seen >= 40   # forward, backward, head, resident, first-layer and streaming instances

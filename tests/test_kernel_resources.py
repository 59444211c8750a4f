"""No kernel of the library may spill registers to scratch memory: a spill inside a streaming loop costs more
than any launch-shape tuning recovers (the sampling head once lost a quarter of its time that way).  Compiles the
two kernel files for gfx950 with the compiler's resource-usage remarks and checks every kernel."""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2307_02628_amd import _build

KERNEL_FILES = ["kernels_f32.hip", "kernels_bf16.hip"]


@pytest.mark.parametrize("src", KERNEL_FILES)
def test_no_kernel_spills(src):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory() as tmp:
        cmd = [hipcc, "--offload-arch=gfx950", "--cuda-device-only", "-O3", "-std=c++17",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Rpass-analysis=kernel-resource-usage",
               "-x", "hip", "-c", os.path.join(_build.CSRC, src), "-o", os.path.join(tmp, "k.o")]
        res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    name, usage = None, {}
    for line in res.stderr.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            usage[name] = {}
            continue
        m = re.search(r"remark:\s+(ScratchSize \[bytes/lane\]|VGPRs Spill|SGPRs Spill): (\d+)", line)
        if m and name:
            usage[name][m.group(1)] = int(m.group(2))
    assert len(usage) >= 10, "no resource remarks found"
    bad = {k: v for k, v in usage.items() if any(v.values())}
    assert not bad, f"kernels that spill: {bad}"

"""Host-side check of what the compiler made of the kernels: no kernel may spill more than a handful of
vector registers. The big tiles sit at the register limit (256 accumulators + 256 vector registers per
lane), and a change that pushes one of them over it still compiles and still gives the right bits,
only 10-15 % slower; this is the place where that shows."""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2512_10236_amd import _build

MAX_VGPR_SPILL = 64          # today: 0-11 everywhere, 48 in the output-streaming variant of the 256x256 resident kernel (in its first and last turns, not in the steady k loop)


@pytest.mark.parametrize("src", ["ficco_gemm.hip", "ficco_reduce.hip"])
def test_no_kernel_spills_more_than_a_few_vector_registers(src):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    with tempfile.TemporaryDirectory() as tmp:
        cmd = [hipcc] + _build.FLAGS + ["-c", os.path.join(_build.CSRC, src), "-o", os.path.join(tmp, "x.o"),
                                        "-Rpass-analysis=kernel-resource-usage"]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-2000:]
    name, seen, bad = None, 0, []
    for line in r.stdout.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"VGPRs Spill: (\d+)", line)
        if m:
            seen += 1
            if int(m.group(1)) > MAX_VGPR_SPILL:
                bad.append((name, int(m.group(1))))
    assert seen > 0, "the compiler printed no resource usage"
    assert not bad, f"kernels that spill vector registers: {bad}"

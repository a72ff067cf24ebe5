"""Host-side check of what the compiler made of the kernels (no GPU): register spills.

The decode and GEMM kernels issue some of their loads as instructions and count the loads in flight by hand; the
compiler does not know that such a load's target register is not valid yet.  If it ran out of registers there and moved
such a register to scratch memory, it would save what the register held before the load landed.  So these kernels must
not use scratch memory at all (one instance is known to park three 64-bit addresses outside its loops)."""
import concurrent.futures
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2507_01438_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# kernel name fragment -> bytes of scratch per lane it may use
ALLOWED = {
    "decode_kernelILi4ELb1ELi8ELb0ELb1E": 12,        # 8 waves, 8-bit W: addresses parked before and after the stream
    "decode_group_kernelILi4ELb1ELi8ELb0ELb1E": 12,
}


def _scratch_of(source):
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "--cuda-device-only", "-c",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-Rpass-analysis=kernel-resource-usage", "-o", os.devnull, os.path.join(CSRC, source)]
    p = subprocess.run(cmd, capture_output=True, text=True)
    assert p.returncode == 0, p.stderr[-2000:]
    out, name = {}, None
    for line in p.stderr.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and name:
            out[name] = int(m.group(1))
            name = None
    return out


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="no hipcc here")
def test_kernels_that_count_their_loads_by_hand_do_not_spill():
    with concurrent.futures.ThreadPoolExecutor(2) as ex:
        found = {}
        for part in ex.map(_scratch_of, ["gemm.hip", "decode.hip"]):
            found.update(part)
    assert any("lora_gemm_kernel" in k for k in found) and any("decode_kernel" in k for k in found)
    for name, scratch in found.items():
        limit = max([v for k, v in ALLOWED.items() if k in name] or [0])
        assert scratch <= limit, f"{name} uses {scratch} bytes of scratch memory per lane"

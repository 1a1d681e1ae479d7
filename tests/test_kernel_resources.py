"""Host-side guard on the compiled kernels: none of them may spill registers to scratch memory.

A spill does not change results, so no parity test sees it, but it multiplies a kernel's
time (a second store in one fully unrolled epilogue once tripled every launch of the 128 x 128
GEMM).  hipcc reports each kernel's scratch bytes per lane with
-Rpass-analysis=kernel-resource-usage; the sources are compiled for the device only, in
parallel, which takes well under a minute.
"""
import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

from paper_2403_00877_amd import build as hip_build

# kernels that are allowed to spill, with the reason (none)
ALLOWED = set()


def _resources(src):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in hip_build.FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [hipcc] + flags + ["--cuda-device-only", "-c", "-Rpass-analysis=kernel-resource-usage",
                             "-o", os.devnull, src]
    out = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, check=True).stdout
    found, name = {}, None
    for line in out.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and name:
            found[name] = int(m.group(1))
    return found


def test_no_kernel_spills_to_scratch():
    with ThreadPoolExecutor(max_workers=5) as pool:
        per_file = list(pool.map(_resources, hip_build.sources()))
    kernels = {}
    for d in per_file:
        kernels.update(d)
    assert len(kernels) > 50, "the compiler's resource remarks were not parsed"
    spilling = {k: v for k, v in kernels.items()
                if v > 0 and not any(re.search(a, k) for a in ALLOWED)}
    assert not spilling, spilling

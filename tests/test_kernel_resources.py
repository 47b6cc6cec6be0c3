"""Build-time check (CPU only, cross-compiles for gfx950): no kernel of the library may use private
scratch memory.  A register array that the compiler cannot keep in registers silently turns into
extra memory traffic (caught once by the hardware counters in the fused mean + line-6 kernel)."""
import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

from paper_1906_12043_amd import build as hip_build


def _assembly(src):
    cmd = [hip_build.HIPCC, *[f for f in hip_build.FLAGS if f != "-fPIC"], "-S", "--cuda-device-only",
           os.path.join(hip_build.CSRC, src), "-o", "-"]
    return subprocess.run(cmd, capture_output=True, text=True, check=True).stdout


def test_no_kernel_uses_scratch_memory_or_spills():
    sources = [s for s in hip_build.SOURCES if s != "api.hip"]
    with ThreadPoolExecutor(max_workers=4) as pool:
        texts = list(pool.map(_assembly, sources))
    seen = 0
    for src, text in zip(sources, texts):
        names = re.findall(r"\.name:\s+(\S+)", text)
        scratch = [int(v) for v in re.findall(r"\.private_segment_fixed_size:\s+(\d+)", text)]
        spills = [int(v) for v in re.findall(r"\.vgpr_spill_count:\s+(\d+)", text)]
        assert names and len(scratch) == len(spills) == len(names), src
        for name, sc, sp in zip(names, scratch, spills):
            assert sc == 0 and sp == 0, "%s: %s uses %d B scratch, %d spilled registers" % (src, name, sc, sp)
            seen += 1
    assert seen >= 20

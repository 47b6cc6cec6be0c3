"""Build-time check (CPU only, cross-compiles for gfx950): no kernel of the library may use private
scratch memory.  A register array that the compiler cannot keep in registers silently turns into
extra memory traffic (caught once by the hardware counters in the fused mean + line-6 kernel).
The figures come from the compiler's own resource-usage remarks; nothing is written to disk."""
import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

from paper_1906_12043_amd import build as hip_build


def _remarks(src):
    cmd = [hip_build.HIPCC, *[f for f in hip_build.FLAGS if f != "-fPIC"], "-Rpass-analysis=kernel-resource-usage",
           "--cuda-device-only", "-c", os.path.join(hip_build.CSRC, src), "-o", os.devnull]
    return subprocess.run(cmd, capture_output=True, text=True, check=True).stderr


def kernel_resources(src):
    """{kernel name: {remark field: integer value}} of one source file."""
    out, name = {}, None
    for line in _remarks(src).splitlines():
        m = re.search(r"remark:\s+(.*?):\s+(\S+) \[-Rpass-analysis=kernel-resource-usage\]", line)
        if not m:
            continue
        field, value = m.group(1).strip(), m.group(2)
        if field == "Function Name":
            name = value
            out[name] = {}
        elif name is not None and value.lstrip("-").isdigit():
            out[name][field] = int(value)
    return out


def test_no_kernel_uses_scratch_memory_or_spills():
    sources = [s for s in hip_build.SOURCES if s != "api.hip"]
    with ThreadPoolExecutor(max_workers=4) as pool:
        tables = list(pool.map(kernel_resources, sources))
    seen = 0
    for src, table in zip(sources, tables):
        assert table, src
        for name, res in table.items():
            # (scalar registers parked in vector-register lanes cost no memory traffic and are not counted)
            assert res["ScratchSize [bytes/lane]"] == 0 and res["VGPRs Spill"] == 0, \
                "%s: %s uses %d B scratch, %d spilled vector registers" % (
                    src, name, res["ScratchSize [bytes/lane]"], res["VGPRs Spill"])
            seen += 1
    assert seen >= 20

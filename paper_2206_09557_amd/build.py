"""Build liblutgemm.so (gfx950) in-tree with hipcc.  `python -m paper_2206_09557_amd.build`.

The device source is compiled once per kernel family (-DLUT_PART=k) in parallel, then linked with the host source."""
from __future__ import annotations

import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "liblutgemm.so")
HOST_SOURCE = os.path.join(PKG, "csrc", "lutgemm_host.cpp")
DEVICE_SOURCE = os.path.join(PKG, "csrc", "lutgemm_device.hip")
PARTS = 14   # kernel families of lutgemm_device.hip (LUT_PART = 0 .. 13)

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-pthread",
    # packed fp32 VALU forms stay off for every HIP translation unit of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-ffp-contract=off", "-Wall", "-Wno-unused-command-line-argument",
    # a unit that instantiates one kernel family leaves the others' helpers unused
    "-Wno-unused-function", "-Wno-unused-const-variable",
]


def _resource_summary(stderr_text: str):
    """(kernels, [(name, scratch bytes per lane)] of those that use scratch memory, largest LDS)
    from the compiler's kernel-resource-usage remarks."""
    kernels, name, scratch, lds = 0, None, [], 0
    for line in stderr_text.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split("[")[0].strip()
            kernels += 1
        elif "ScratchSize [bytes/lane]:" in line:
            n = int(line.split("ScratchSize [bytes/lane]:")[1].split("[")[0])
            if n:
                scratch.append((name, n))
        elif "LDS Size [bytes/block]:" in line:
            lds = max(lds, int(line.split("LDS Size [bytes/block]:")[1].split("[")[0]))
    return kernels, scratch, lds


def build_library(verbose: bool = True, jobs: int | None = None, report: bool = False) -> str:
    """Compile and link.  report=True also prints how many kernels were compiled, which of
    them use scratch memory (none should: a spill in a lookup loop costs more than any
    prefetch hides) and the largest LDS allocation."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = jobs or min(PARTS + 1, os.cpu_count() or 1, 16)
    inc = ["-I", os.path.join(ROOT, "include")]
    with tempfile.TemporaryDirectory(prefix="lutgemm_build_") as tmp:
        units = [(HOST_SOURCE, os.path.join(tmp, "host.o"), [])]
        units += [(DEVICE_SOURCE, os.path.join(tmp, f"device_{k}.o"), [f"-DLUT_PART={k}"]) for k in range(PARTS)]

        def compile_unit(unit):
            src, obj, extra = unit
            cmd = [hipcc, *HIPCC_FLAGS, *extra, *inc, "-c", "-o", obj, src]
            if report and src == DEVICE_SOURCE:
                cmd.append("-Rpass-analysis=kernel-resource-usage")
            if verbose:
                print(" ".join(cmd), flush=True)
            done = subprocess.run(cmd, check=True, stderr=subprocess.PIPE if report else None, text=True)
            return obj, (done.stderr or "")

        with ThreadPoolExecutor(max_workers=jobs) as pool:
            results = list(pool.map(compile_unit, units))
        objects = [obj for obj, _ in results]
        if report:
            kernels, scratch, lds = _resource_summary("\n".join(err for _, err in results))
            print(f"{kernels} kernels, largest LDS allocation {lds} bytes, {len(scratch)} kernels use scratch memory")
            for name, n in scratch:
                print(f"  scratch {n} bytes/lane: {name}")
        link = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-pthread", "-Wno-unused-command-line-argument",
                "-o", LIB, *objects]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True)
    return LIB


if __name__ == "__main__":
    build_library(report="--report" in sys.argv[1:])
    sys.exit(0)

"""Builds the HIP library in-tree for gfx950 (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "cbd.hip")
DEPS = [SRC, os.path.join(HERE, "csrc", "cbd_device.hpp"), os.path.join(HERE, "csrc", "cbd_lean.hpp"), os.path.join(HERE, "csrc", "cbd_team.hpp"), os.path.join(HERE, "..", "include", "cbd.h")]
LIB = os.path.join(HERE, "libcbdec.so")
LIB_PROFILE = os.path.join(HERE, "libcbdec_prof.so")   # diagnostic build: phase stamps in the lean frame code

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the kernels already combine a wave's updates into one atomic issued by one lane; the compiler's own
    # wave-level combining of atomics would only wrap each of them in more code
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    "-Wall", "-Wno-unused-result", "-pthread",
]


def build(force: bool = True, verbose: bool = False, profile: bool = False) -> str:
    """Compile libcbdec.so.  With force=False only when a source is newer than the library.
    profile=True builds libcbdec_prof.so instead: the same code with -DCBD_PROFILE, in which thread 0 of every
    workgroup stamps the phases of the lean frames (bench.py --phases reads the sums); not the product build."""
    lib = LIB_PROFILE if profile else LIB
    if not force and os.path.exists(lib) and all(os.path.getmtime(lib) >= os.path.getmtime(d) for d in DEPS):
        return lib
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *(["-DCBD_PROFILE"] if profile else []), "-o", lib + ".tmp", SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(lib + ".tmp", lib)
    return lib


def resource_usage() -> dict:
    """Compiles the device code once more with the compiler's resource remarks on and returns, per kernel,
    {"vgprs", "vgpr_spill", "scratch", "lds"} (name = demangled-ish substring of the kernel symbol)."""
    import re
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-Wall", "-Wno-unused-result")]
    with tempfile.TemporaryDirectory() as tmp:
        cmd = [hipcc, *flags, "--cuda-device-only", "-c", "-Rpass-analysis=kernel-resource-usage",
               "-o", os.path.join(tmp, "dev.o"), SRC]
        out = subprocess.run(cmd, check=True, capture_output=True, text=True).stderr
    usage, cur = {}, None
    for line in out.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", line)
        if m:
            cur = usage.setdefault(m.group(1), {})
            continue
        for key, pat in (("vgprs", r"remark:\s+VGPRs: (\d+)"), ("vgpr_spill", r"VGPRs Spill: (\d+)"),
                         ("scratch", r"ScratchSize \[bytes/lane\]: (\d+)"), ("lds", r"LDS Size \[bytes/block\]: (\d+)")):
            m = re.search(pat, line)
            if m and cur is not None:
                cur[key] = int(m.group(1))
    return usage


if __name__ == "__main__":
    print(build(force=True, verbose=True, profile="--profile" in sys.argv[1:]))

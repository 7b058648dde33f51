"""Build step of libmrfmp: three hipcc compilations side by side and a link, in-tree output next to
the sources."""
from __future__ import annotations

import os
import subprocess

CSRC = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc")
LIB_PATH = os.path.join(CSRC, "libmrfmp.so")
SOURCES = ["mrfmp.hip"]
HEADERS = ["mrfmp_device.h", "mrfmp_fwd.h", "mrfmp_bwd.h", "mrfmp_head.h", "../../include/mrfmp.h"]

# -ffp-contract=off: the only fused multiply-add is the explicit one of the message update,
#   so that floating point decisions (argmins) match a plain C evaluation order.
# packed-fp32 instructions are switched off for the test machines of machines.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-munsafe-fp-atomics",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall"]


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(verbose: bool = False) -> str:
    """Compile libmrfmp.so for gfx950 (cross-compiles without a GPU): the one source as three
    translation units (forward pass, backward pass, entry points) side by side, then link."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(CSRC, "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    jobs = []
    for part in (1, 2, 3):
        obj = os.path.join(objdir, "mrfmp_part%d.o" % part)
        cmd = [hipcc, *flags, "-DMRF_PART=%d" % part, "-c", "-o", obj, *SOURCES]
        jobs.append((obj, subprocess.Popen(cmd, cwd=CSRC, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for obj, proc in jobs:
        out, _ = proc.communicate()
        if verbose or proc.returncode != 0:
            print(out)
        failed = failed or proc.returncode != 0
    if failed:
        raise RuntimeError("hipcc failed compiling libmrfmp")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *[obj for obj, _ in jobs]]
    res = subprocess.run(cmd, cwd=CSRC, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed linking libmrfmp.so")
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))

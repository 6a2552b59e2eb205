"""Build step: compile the HIP sources under csrc/ into libqspec.so (gfx950)."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "libqspec.so")
SOURCES = [os.path.join(HERE, "csrc", "qspec_api.hip")]
# bench-only microbenchmarks (machine ceilings); a library of its own, not part of the ABI
CEIL_LIB_PATH = os.path.join(HERE, "libqspec_ceilings.so")
CEIL_SOURCES = [os.path.join(HERE, "bench_csrc", "ceilings.hip")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    # per-kernel register / spill report, read back below
    "-Rpass-analysis=kernel-resource-usage",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


# gemm_tile16w_kernel orders its waits on direct-to-LDS loads by counting the loads
# issued after them; a register spill would put stores into that sequence (stores
# complete out of order with loads), so such an instance must not be shipped.  The
# streaming kernels are held to the same rule (a spill in their loop costs more than
# the instance gains), and so is the draft-mode tiled kernel.
NO_SPILL_KERNELS = ("gemm_tile16w_kernel", "gemm_stream_kernel", "gemm_tile4w_kernel")


def spilling_kernels(report: str, names) -> list:
    """Mangled names of kernels matching `names` whose resource remarks show VGPR spills."""
    bad, current = [], None
    for line in report.splitlines():
        m = re.search(r"remark: +Function Name: (\S+)", line)
        if m:
            current = m.group(1)
            continue
        m = re.search(r"remark: +VGPRs Spill: (\d+)", line)
        if m and current and int(m.group(1)) > 0 and any(n in current for n in names):
            bad.append(current)
    return bad


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = True) -> str:
    """Always recompiles; returns the path of the shared library."""
    cmd = [hipcc(), *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(HERE, "csrc"), "-o", LIB_PATH, *SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops" not in l and "-Rpass-analysis=kernel-resource-usage" not in l)
    if verbose and out.strip():
        print(out, flush=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    spilled = spilling_kernels(res.stdout, NO_SPILL_KERNELS)
    if spilled:
        raise RuntimeError("kernels that must not spill registers do: " + ", ".join(spilled))
    cmd = [hipcc(), *HIPCC_FLAGS, "-I", os.path.join(HERE, "csrc"), "-o", CEIL_LIB_PATH, *CEIL_SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    return LIB_PATH


if __name__ == "__main__":
    build()
    sys.exit(0)

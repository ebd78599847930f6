"""Build the HIP library (libls_attn.so) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libls_attn.so")
PROBE_SRC = os.path.join(HERE, "csrc_probe", "ls_probe.hip")
PROBE_LIB_PATH = os.path.join(HERE, "libls_probe.so")   # bench-only measurement helpers

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.hpp")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    return any(os.path.getmtime(d) > t for d in deps)


RESOURCE_REPORT = os.path.join(HERE, "libls_attn.resources.txt")


def build_library(force: bool = True, extra_flags=()) -> str:
    """Compile every csrc/*.hip into one shared library.  Returns its path.  The compiler's
    per-kernel resource remarks (registers, scratch, spills) are kept next to the library:
    the cached-key kernel counts its own outstanding loads, which a register spill would upset."""
    if not force and not is_stale():
        return LIB_PATH
    cmd = [HIPCC, *FLAGS, *extra_flags, "-Rpass-analysis=kernel-resource-usage", "-o", LIB_PATH, *sources()]
    done = subprocess.run(cmd, check=False, stderr=subprocess.PIPE, text=True)
    remarks = [ln for ln in done.stderr.splitlines() if "[-Rpass-analysis=kernel-resource-usage]" in ln]
    other = [ln for ln in done.stderr.splitlines() if "[-Rpass-analysis=kernel-resource-usage]" not in ln
             and "packed-fp32-ops" not in ln]
    if other:
        print("\n".join(other), file=sys.stderr)
    if done.returncode != 0:
        raise subprocess.CalledProcessError(done.returncode, cmd)
    with open(RESOURCE_REPORT, "w") as f:
        f.write("\n".join(remarks) + "\n")
    return LIB_PATH


def kernel_resources(report: str = RESOURCE_REPORT) -> dict:
    """{kernel name: {"VGPRs": n, "AGPRs": n, "ScratchSize": n, "SGPRs Spill": n, "VGPRs Spill": n, ...}}"""
    import re
    out, cur = {}, None
    for ln in open(report):
        m = re.search(r"remark: Function Name: (\S+)", ln)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z ]+?)(?: \[[^\]]*\])?: (\d+)", ln)
        if m and cur is not None:
            cur[m.group(1).strip()] = int(m.group(2))
    return out


def build_probe_library() -> str:
    """Compile the benchmark's measurement helpers into a shared library of their own."""
    subprocess.run([HIPCC, *FLAGS, "-o", PROBE_LIB_PATH, PROBE_SRC], check=True)
    return PROBE_LIB_PATH


if __name__ == "__main__":
    print(build_library())
    print(build_probe_library())

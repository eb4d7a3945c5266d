"""Builds libeeverify.so (HIP, gfx950 only) next to the sources."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libeeverify.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unused-value", "-Wno-unused-result",
]


def sources():
    return [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith((".hip", ".hpp"))] + [
        os.path.join(os.path.dirname(_HERE), "include", "ee.h")]


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile the library; with force=False only when a source is newer."""
    if not force and os.path.exists(LIB_PATH):
        if os.path.getmtime(LIB_PATH) >= max(os.path.getmtime(s) for s in sources()):
            return LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-Rpass-analysis=kernel-resource-usage", "-o", LIB_PATH,
           os.path.join(CSRC, "ee_runtime.hip")]
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    report = check_resources(r.stdout)
    noise = ("remark:", "packed-fp32-ops", "      |", "[-Rpass-analysis")
    for line in r.stdout.splitlines():
        if r.returncode != 0 or (verbose and not any(n in line for n in noise)):
            print(line)
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, cmd)
    for line in report:
        print(line)
    return LIB_PATH


def check_resources(compiler_output: str):
    """Kernels of the pass must not use scratch memory (register spills or stack arrays):
    measured on MI355X, a few hundred bytes of scratch per lane add tens of microseconds to
    every launch of these 256-workgroup kernels.  Returns warning lines."""
    import re
    name, out = None, []
    for line in compiler_output.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and name and int(m.group(1)) > 0 and any(k in name for k in ("ee_gemm_kernel", "att_kernel", "misc_kernel", "sample_kernel")):
            out.append(f"WARNING: {name} uses {m.group(1)} bytes of scratch per lane (expect slow launches)")
    return out


if __name__ == "__main__":
    build(verbose=True)

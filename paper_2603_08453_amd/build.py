"""Builds liblychee.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import re
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblychee.so")
SOURCES = ["lc_api.hip", "lc_retrieve.hip", "lc_decode.hip", "lc_build.hip", "lc_chunker.hip", "lc_bench.hip"]


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if c and os.path.exists(c):
            return c
    raise RuntimeError("hipcc not found")


def build(verbose: bool = True) -> str:
    """Compile every HIP source for gfx950 and link the shared library."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    cmd += ["-Rpass-analysis=kernel-resource-usage"]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    cmd += ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    kernels = kernel_resources(proc.stderr)
    rest = [ln for ln in proc.stderr.splitlines()
            if "kernel-resource-usage" not in ln and "packed-fp32-ops" not in ln and not _REMARK_ECHO.match(ln)]
    if rest and (verbose or proc.returncode != 0):
        print("\n".join(rest), file=sys.stderr, flush=True)
    if proc.returncode != 0:
        raise subprocess.CalledProcessError(proc.returncode, cmd)
    # No kernel may use scratch memory (register spills): the 1024-thread kernels are written to fit
    # their 128 registers per lane, and a spill there is a regression to be fixed, not shipped.
    spilled = {k: v for k, v in kernels.items() if v.get("scratch", 0) > 0}
    if spilled:
        if os.path.exists(LIB):
            os.remove(LIB)
        raise RuntimeError("kernels that spill registers to scratch memory: " +
                           ", ".join(f"{k} ({v['scratch']} B/lane)" for k, v in sorted(spilled.items())))
    if verbose and kernels:
        print(f"{len(kernels)} kernels, at most {max(v.get('vgprs', 0) for v in kernels.values())} VGPRs, none uses scratch memory",
              flush=True)
    return LIB


_REMARK_ECHO = re.compile(r"^\s*(\d+\s*\|.*|\|\s*\^.*)$")     # the source line and caret clang prints under a remark


def kernel_resources(remarks: str) -> dict:
    """Per kernel {"vgprs", "scratch"} from clang's kernel-resource-usage remarks."""
    out, cur = {}, None
    for ln in remarks.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", ln)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        if cur is None:
            continue
        m = re.search(r"remark:\s+VGPRs: (\d+)", ln)
        if m:
            cur["vgprs"] = int(m.group(1))
        m = re.search(r"remark:\s+ScratchSize \[bytes/lane\]: (\d+)", ln)
        if m:
            cur["scratch"] = int(m.group(1))
    return out


if __name__ == "__main__":
    build()
    print("built", LIB)

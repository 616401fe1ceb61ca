"""Build librsdgc.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import re
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librsdgc.so")
SOURCES = ["rsdgc_plan.cpp", "rsdgc_kernels.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall"]


def build_library(verbose: bool = False, extra_flags=()) -> str:
    """Compiles the library.  The compiler's per-kernel resource remarks are read back: the NSI
    kernels are sized to run without register spills (the main pass at 96 VGPRs under an
    occupancy hint), and a spill there costs tens of percent silently -- so it is reported."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, "-Rpass-analysis=kernel-resource-usage", *extra_flags]
    for s in SOURCES:
        path = os.path.join(CSRC, s)
        cmd += (["-x", "hip", path] if s.endswith(".cpp") else [path])
    cmd += ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    remarks, other, after_remark = [], [], False
    for line in proc.stderr.splitlines():
        if "[-Rpass-analysis=kernel-resource-usage]" in line:
            remarks.append(line)
            after_remark = True
        elif after_remark and re.match(r"^\s*\d*\s*\|", line):
            pass                                   # the source line and caret that follow a remark
        else:
            other.append(line)
            after_remark = False
    if other:
        print("\n".join(other), flush=True)
    if proc.returncode != 0:
        raise subprocess.CalledProcessError(proc.returncode, cmd)
    for name, scratch in spilling_kernels(remarks):
        print(f"warning: kernel {name} spills registers ({scratch} bytes of scratch per lane)", flush=True)
    return LIB


def spilling_kernels(remarks):
    """(mangled name, scratch bytes per lane) of the NSI kernels that use scratch memory, from
    the lines of -Rpass-analysis=kernel-resource-usage."""
    out, name = [], None
    for line in remarks:
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            continue
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and name and "k_nsi" in name and int(m.group(1)) > 0 and (name, int(m.group(1))) not in out:
            out.append((name, int(m.group(1))))
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))

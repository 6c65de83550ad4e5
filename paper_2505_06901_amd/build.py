"""Builds libecco.so (HIP kernels for gfx950 + the CPU fit) in-tree with hipcc."""
from __future__ import annotations

import os
import re
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libecco.so")
PROBE = os.path.join(HERE, "probe_lds")  # stand-alone measurement program (csrc/probe_lds.hip), not part of the library
SOURCES = ["ecco_fit.cpp", "ecco_model.cpp", "ecco_pb_model.cpp", "ecco_kernels.hip", "ecco_act.hip", "ecco_pb_kernels.hip"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


# Kernels that may park a few scalar registers in vector-register lanes.  Only the grouped-query attention kernel
# for two models with long codes does (2 registers) and passes its tests; every other kernel stays clear, so that
# a change which starts to spill is noticed when it is made.
_SGPR_SPILL_TOLERATED = ("kv_attend_gqa_kernelILb1ELb1E",)


def _check_kernel_resources(remarks: str, verbose: bool) -> None:
    """Every kernel must keep its working set in registers: a kernel that spills to scratch memory is
    far off its design point (the decode loops are sized for 1024-thread workgroups, 128 VGPRs), so
    a register spill is a build error rather than a silent slowdown."""
    name, found = None, 0
    for line in remarks.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            continue
        m = re.search(r"remark:\s+ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and name:
            found += 1
            if verbose:
                print("  %s: scratch %s bytes/lane" % (name, m.group(1)))
            if int(m.group(1)) != 0 and not os.environ.get("ECCO_ALLOW_SCRATCH"):
                raise RuntimeError("kernel %s spills %s bytes/lane to scratch memory" % (name, m.group(1)))
        m = re.search(r"remark:\s+(SGPRs|VGPRs) Spill: (\d+)", line)
        if m and name:
            if verbose and int(m.group(2)):
                print("  %s: %s spilled: %s" % (name, m.group(1), m.group(2)))
            tolerated = m.group(1) == "SGPRs" and any(k in name for k in _SGPR_SPILL_TOLERATED)
            if int(m.group(2)) != 0 and not tolerated and not os.environ.get("ECCO_ALLOW_SCRATCH"):
                raise RuntimeError("kernel %s spills %s %s" % (name, m.group(2), m.group(1)))
    if found == 0:
        raise RuntimeError("no kernel resource remarks found: cannot verify register use")


def build(verbose: bool = False) -> str:
    """Compiles every source for gfx950 and links libecco.so; always recompiles."""
    objs = []
    common = ["-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
              "-Wall", "-Wno-unused-function"]
    for src in SOURCES:
        path = os.path.join(CSRC, src)
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        if src.endswith(".hip"):
            cmd = [_hipcc(), "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                   "-Rpass-analysis=kernel-resource-usage", *common, "-c", path, "-o", obj]
        else:
            cmd = [_hipcc(), "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", *common, "-c", path, "-o", obj]
        if verbose:
            print(" ".join(cmd))
        proc = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
        if proc.returncode != 0:
            raise RuntimeError("compiling %s failed:\n%s" % (src, proc.stderr))
        if src.endswith(".hip"):
            _check_kernel_resources(proc.stderr, verbose)
        objs.append(obj)
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB, "-lpthread"]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    # the LDS / decode-loop probe: a program of its own, so that its figures can be reproduced without the library
    cmd = [_hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           os.path.join(CSRC, "probe_lds.hip"), "-o", PROBE]
    if verbose:
        print(" ".join(cmd))
    proc = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    if proc.returncode != 0:
        raise RuntimeError("compiling probe_lds.hip failed:\n%s" % proc.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))

"""Builds libecco.so (HIP kernels for gfx950 + the CPU fit) in-tree with hipcc."""
from __future__ import annotations

import os
import re
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libecco.so")
PROBES = ["probe_lds", "probe_last_vgpr"]  # stand-alone measurement programs (csrc/<name>.hip), not part of the library
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


def _check_kernel_resources(remarks: str, verbose: bool) -> dict:
    """Every kernel must keep its working set in registers: a kernel that spills to scratch memory is
    far off its design point (the decode loops are sized for 1024-thread workgroups, 128 VGPRs), so
    a register spill is a build error rather than a silent slowdown."""
    name, found, vgprs = None, 0, {}
    for line in remarks.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            continue
        m = re.search(r"remark:\s+VGPRs: (\d+)", line)
        if m and name:
            vgprs[name] = int(m.group(1))
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
    return vgprs


# On the MI355X boxes this library was developed on, a 64-bit shift (v_lshlrev_b64, v_lshrrev_b64, v_ashrrev_i64) whose
# shift amount sits in the LAST vector register of the wavefront's allocation returns wrong results in a fifth of its
# executions as soon as a SIMD holds more than one wavefront (csrc/probe_last_vgpr.hip measures it; the amount is
# apparently fetched as a register pair, and the pair's second half lies outside the allocation).  The compiler does
# not avoid that register, and the decode loops shift their 64-bit windows by table entries in whatever register the
# allocator picked, so a kernel whose register count is an exact multiple of the allocation unit (8) can be hit.
# Every kernel's generated code is therefore checked, and a hit is a build error.
_VGPR_ALLOC_UNIT = 8
_SHIFT64 = re.compile(r"^\s*(v_(?:lshlrev_b64|lshrrev_b64|ashrrev_i64)(?:_e64)?)\s+v\[\d+:\d+\],\s*v(\d+)\b")


def last_register_shifts(asm: str) -> list:
    """(kernel, instruction) for every 64-bit shift in the assembly text `asm` (hipcc -S output for gfx950) whose shift
    amount is the last register of its kernel's allocation."""
    bodies, counts, cur, pending = {}, {}, None, None
    for line in asm.splitlines():
        code = line.split(";")[0]
        m = re.match(r"^([A-Za-z_$.][\w$.]*):", code)
        if m and not m.group(1).startswith(".L"):
            cur = m.group(1)
            bodies[cur] = []
            continue
        m = re.match(r"\s*\.amdhsa_kernel\s+(\S+)", code)
        if m:
            pending, cur = m.group(1), None
            continue
        m = re.match(r"\s*\.amdhsa_next_free_vgpr\s+(\d+)", code)
        if m and pending:
            counts[pending] = int(m.group(1))
            pending = None
            continue
        if cur is not None:
            bodies[cur].append(code)
            if "s_endpgm" in code:
                cur = None
    hits = []
    for name, n in counts.items():
        last = (n + _VGPR_ALLOC_UNIT - 1) // _VGPR_ALLOC_UNIT * _VGPR_ALLOC_UNIT - 1
        for code in bodies.get(name, []):
            m = _SHIFT64.match(code)
            if m and int(m.group(2)) == last:
                hits.append((name, code.strip()))
    return hits


def kernel_register_counts(asm: str) -> dict:
    """kernel -> .amdhsa_next_free_vgpr of the assembly text `asm`."""
    counts, pending = {}, None
    for line in asm.splitlines():
        m = re.match(r"\s*\.amdhsa_kernel\s+(\S+)", line)
        if m:
            pending = m.group(1)
        m = re.match(r"\s*\.amdhsa_next_free_vgpr\s+(\d+)", line)
        if m and pending:
            counts[pending], pending = int(m.group(1)), None
    return counts


def _check_last_register_shift(path: str, flags: list, compiled_vgprs: dict, verbose: bool) -> None:
    proc = subprocess.run([_hipcc(), "--offload-arch=gfx950", *flags, "-S", "--cuda-device-only", path, "-o", "-"],
                          stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    if proc.returncode != 0:
        raise RuntimeError("generating assembly for %s failed:\n%s" % (path, proc.stderr))
    if ".amdhsa_kernel" not in proc.stdout:
        raise RuntimeError("no kernel found in the assembly of %s: cannot check its shifts" % path)
    # the assembly must be that of the object just compiled: same kernels, same register counts
    if kernel_register_counts(proc.stdout) != compiled_vgprs:
        raise RuntimeError("the assembly generated for %s does not match the compiled object (kernels or register counts differ)" % path)
    hits = last_register_shifts(proc.stdout)
    if verbose:
        print("  %s: %d 64-bit shifts by the last allocated register" % (os.path.basename(path), len(hits)))
    if hits and not os.environ.get("ECCO_ALLOW_LAST_REGISTER_SHIFT"):
        raise RuntimeError("64-bit shifts whose amount is the last register of the kernel's allocation (wrong results on "
                           "MI355X; change the kernel's register count, e.g. by reserving one more register):\n" +
                           "\n".join("  %s: %s" % h for h in hits))


def build(verbose: bool = False) -> str:
    """Compiles every source for gfx950 and links libecco.so; always recompiles."""
    objs = []
    common = ["-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
              "-Wall", "-Wno-unused-function"]
    for src in SOURCES:
        path = os.path.join(CSRC, src)
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        device_flags = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *common]
        if src.endswith(".hip"):
            cmd = [_hipcc(), "--offload-arch=gfx950", "-Rpass-analysis=kernel-resource-usage", *device_flags, "-c", path, "-o", obj]
        else:
            cmd = [_hipcc(), "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", *common, "-c", path, "-o", obj]
        if verbose:
            print(" ".join(cmd))
        proc = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
        if proc.returncode != 0:
            raise RuntimeError("compiling %s failed:\n%s" % (src, proc.stderr))
        if src.endswith(".hip"):
            compiled_vgprs = _check_kernel_resources(proc.stderr, verbose)
            _check_last_register_shift(path, device_flags, compiled_vgprs, verbose)
        objs.append(obj)
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB, "-lpthread"]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    # the measurement programs (LDS access patterns and the decode loop; the last-register shift check): programs of
    # their own, so that their figures can be reproduced without the library
    for name in PROBES:
        cmd = [_hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               os.path.join(CSRC, name + ".hip"), "-o", os.path.join(HERE, name)]
        if verbose:
            print(" ".join(cmd))
        proc = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
        if proc.returncode != 0:
            raise RuntimeError("compiling %s.hip failed:\n%s" % (name, proc.stderr))
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))

"""Compile the HIP sources under csrc/ for gfx950 into paper_2402_17764_amd/libbitnet_hip.so.

hipcc cross-compiles without a GPU.  Objects go to paper_2402_17764_amd/_build/ (not committed);
the shared library sits next to this file so that it travels with the tree.
"""
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libbitnet_hip.so")

SOURCES = ["api.hip", "quant_weights.hip", "quant_acts.hip", "linear_ref.hip", "linear_gemv.hip", "linear_skinny.hip", "linear_gemm.hip", "trit5.hip", "static_scratch.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                       # every rounding step of the quantizers is explicit
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter", "-Wno-unknown-attributes",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


# Kernels that count the vector-memory loads in flight (explicit s_waitcnt vmcnt(n)): a register spill would
# add scratch loads to that count, so the build fails if the compiler gives any of them scratch memory.
NO_SCRATCH = {"linear_skinny.hip": ("linear_skinny_2bit", "linear_skinny_ws_2bit")}


def _check_no_scratch(src, stderr):
    """stderr holds -Rpass-analysis=kernel-resource-usage remarks: 'Function Name: <mangled>' ... 'ScratchSize ...: n'."""
    name, bad = None, []
    for line in stderr.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split()[0]
        elif "ScratchSize" in line and name and any(k in name for k in NO_SCRATCH[src]):
            if int(line.split("]:")[1].split()[0]) != 0:
                bad.append(name)
    if bad:
        raise RuntimeError("%s: kernels that count loads in flight must not spill: %s" % (src, ", ".join(bad)))


def _check_issue_order(src):
    """linear_skinny_2bit waits for a step's LDS copies with a count of the younger loads (s_waitcnt vmcnt(n)), which
    holds only if each step's copies are issued before the weight loads that follow them in the source.  Scheduling
    fences in the kernel pin that; this reads the generated ISA and fails the build if a compiler ever ignores them:
    between barriers a wave must issue kC = 4 kMT / kW copies ("buffer_load ... lds") and then kR weight loads, and
    the prologue kD such groups."""
    asm = os.path.join(BUILD, os.path.splitext(src)[0] + ".s")
    cmd = [HIPCC, *FLAGS, "--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", asm]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc -S failed on %s:\n%s" % (src, r.stderr))
    cur, segs, checked = None, [""], 0
    for line in open(asm):
        m = re.match(r"^_ZN6bitnet18linear_skinny_2bitILi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)E\S*:", line)
        if m:
            cur, segs = [int(v) for v in m.groups()], [""]
            continue
        if cur is None:
            continue
        if "buffer_load_dwordx4" in line:
            segs[-1] += "L" if re.search(r"\blds\b", line) else "W"
        elif "s_barrier" in line:
            segs.append("")
        elif "s_endpgm" in line:
            kMT, kR, kW, kS, kD, kLx = cur
            unit = "L" * (4 * kMT // kW) + "W" * kR
            loops = [g for g in segs[1:] if g]
            if segs[0] != unit * kD or not loops or any(g != unit for g in loops):
                raise RuntimeError("%s: linear_skinny_2bit<%s>: loads are not issued in source order (%s), the counted "
                                   "waits would be wrong" % (src, ", ".join(map(str, cur)), " | ".join(segs)))
            cur, checked = None, checked + 1
    if checked == 0:
        raise RuntimeError("%s: no linear_skinny_2bit kernel found in the ISA: issue order unchecked" % src)


def _compile(src):
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    if src in NO_SCRATCH:
        cmd.append("-Rpass-analysis=kernel-resource-usage")
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    lines = [l for l in r.stderr.splitlines() if noise not in l]
    if src in NO_SCRATCH:                      # drop the resource remarks and the source excerpts printed under them
        lines = [l for l in lines if "remark:" not in l and not re.match(r"^\s*\d*\s*\|", l)]
    err = "\n".join(lines)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
    if src in NO_SCRATCH:
        _check_no_scratch(src, r.stderr)
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_library(verbose: bool = False) -> str:
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as ex:
        order = ex.submit(_check_issue_order, "linear_skinny.hip")
        objs = list(ex.map(_compile, SOURCES))
        order.result()
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp])
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build_library(verbose=True)

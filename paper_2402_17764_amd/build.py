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


def skinny_instantiations(source_text):
    """The linear_skinny_2bit<kMT, kR, kW, kS, kD, kLx> instantiations that the launcher dispatches: every
    `SKINNY(a, b, c, d, e, f)` use in the source."""
    return sorted({tuple(int(v) for v in m.groups())
                   for m in re.finditer(r"\bSKINNY\((\d+), (\d+), (\d+), (\d+), (\d+), (\d+)\)", source_text)})


def check_issue_order(asm_text, expected):
    """linear_skinny_2bit waits for a step's LDS copies with a count of the younger loads (s_waitcnt vmcnt(n)), which
    holds only if each step's copies are issued before the weight loads that follow them in the source.  Scheduling
    fences in the kernel pin that; this reads the device assembly the object is assembled from and raises if a
    compiler ever ignores them: between barriers a wave must issue kC = 4 kMT / kW copies ("buffer_load ... lds") and
    then kR weight loads, and the prologue kD such groups.  Every instantiation in `expected` must be present and pass;
    an instantiation in the assembly that is not expected is an error too (it would ship unchecked by the dispatch
    tests).  Returns the instantiations checked."""
    cur, segs, checked = None, [""], []
    for line in asm_text.splitlines():
        m = re.match(r"^_ZN6bitnet18linear_skinny_2bitILi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)E\S*:", line)
        if m:
            cur, segs = tuple(int(v) for v in m.groups()), [""]
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
                raise RuntimeError("linear_skinny_2bit<%s>: loads are not issued in source order (%s), the counted "
                                   "waits would be wrong" % (", ".join(map(str, cur)), " | ".join(segs)))
            checked.append(cur)
            cur = None
    if cur is not None:
        raise RuntimeError("linear_skinny_2bit<%s>: the kernel's end was not found in the assembly" % ", ".join(map(str, cur)))
    missing = sorted(set(expected) - set(checked))
    extra = sorted(set(checked) - set(expected))
    if missing or extra or len(checked) != len(set(checked)):
        raise RuntimeError("linear_skinny_2bit: issue order unchecked for %s; not dispatched but built: %s" % (missing, extra))
    return checked


def _check_issue_order(src):
    """Runs check_issue_order on the assembly that -save-temps left next to the object: the very text the device
    code of the shipped object was assembled from."""
    asm = os.path.join(BUILD, os.path.splitext(src)[0] + "-hip-amdgcn-amd-amdhsa-gfx950.s")
    expected = skinny_instantiations(open(os.path.join(CSRC, src)).read())
    if not expected:
        raise RuntimeError("%s: no SKINNY(...) dispatch found: the issue-order check has nothing to go by" % src)
    check_issue_order(open(asm).read(), expected)


# Host code with the undefined-behaviour sanitizer compiled in as traps (no runtime library to load): signed overflow,
# bad shifts, out-of-range enum and integer conversions, misaligned and null accesses in the validation and dispatch
# code end the process.  The device code is built as usual; only host-side calls are meant to run against this build.
SANITIZE_HOST = ["-Xarch_host", "-fsanitize=undefined,integer", "-Xarch_host", "-fsanitize-trap=all", "-Xarch_host",
                 "-fno-sanitize=unsigned-integer-overflow,unsigned-shift-base,implicit-conversion"]


def _compile_sanitized(src, out_dir):
    obj = os.path.join(out_dir, os.path.splitext(src)[0] + ".o")
    flags = [f for f in FLAGS if f != "-O3"] + ["-O1", *SANITIZE_HOST]
    r = subprocess.run([HIPCC, *flags, "-c", os.path.join(CSRC, src), "-o", obj], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc (host-sanitized) failed on %s:\n%s" % (src, r.stderr))
    return obj


def build_library_sanitized() -> str:
    """libbitnet_hip_ubsan.so under _build/ubsan: for the CPU test that runs the host-side tests against it."""
    out_dir = os.path.join(BUILD, "ubsan")
    os.makedirs(out_dir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile_sanitized(s, out_dir), SOURCES))
    lib = os.path.join(out_dir, "libbitnet_hip_ubsan.so")
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", lib])
    return lib


def _compile(src):
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    if src in NO_SCRATCH:
        cmd += ["-Rpass-analysis=kernel-resource-usage", "-save-temps=obj"]      # the device assembly stays next to the object
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
        _check_issue_order(src)
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_library(verbose: bool = False) -> str:
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp])
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


def build_floors(verbose: bool = False) -> str:
    """libbitnet_floors.so: the read-only and the MFMA-only kernel that bench.py and read_floor.py time next to the product
    (no part of the BitLinear library)."""
    lib = os.path.join(HERE, "libbitnet_floors.so")
    tmp = lib + ".tmp.%d" % os.getpid()
    r = subprocess.run([HIPCC, *FLAGS, "-shared", os.path.join(CSRC, "floors.hip"), os.path.join(CSRC, "prefill_ladder.hip"), "-o", tmp],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on floors.hip / prefill_ladder.hip:\n" + r.stderr)
    os.replace(tmp, lib)
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    build_library(verbose=True)
    build_floors(verbose=True)

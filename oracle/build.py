"""Compile the CPU oracle (test infrastructure) into oracle/libbitnet_oracle.so with gcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "bitnet_oracle.c")
HDR = os.path.join(HERE, "bitnet_oracle.h")
LIB = os.path.join(HERE, "libbitnet_oracle.so")

# -ffp-contract=off: no fused multiply-add may replace a rounding step the paper's arithmetic has.
CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
          "-Wall", "-Wextra"]


def build_oracle_sanitized(out_dir: str) -> str:
    """The same source with gcc's undefined-behaviour checks compiled in as traps (no sanitizer runtime to load):
    signed overflow, shifts, out-of-range conversions, misaligned or null accesses end the process.  For the test that
    runs the oracle's pins against this build."""
    os.makedirs(out_dir, exist_ok=True)
    lib = os.path.join(out_dir, "libbitnet_oracle_ubsan.so")
    flags = [f for f in CFLAGS if f != "-O2"] + ["-O1", "-g", "-fsanitize=undefined", "-fsanitize-undefined-trap-on-error",
                                                 "-fno-sanitize-recover=all"]
    subprocess.check_call(["gcc", *flags, SRC, "-o", lib, "-lm"])
    return lib


def build_oracle(force: bool = False) -> str:
    newest_src = max(os.path.getmtime(SRC), os.path.getmtime(HDR))
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < newest_src:
        tmp = LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, SRC, "-o", tmp, "-lm"])
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_oracle(force=True))

"""The host code of the HIP library (argument validation, launch selection, the launch descriptions) and the C oracle,
each built with the undefined-behaviour sanitizer as traps, under the tests that exercise them without a GPU: a signed
overflow, an out-of-range enum or conversion, a bad shift or a misaligned access anywhere on those paths ends the child
process, and this test fails."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run_tests(files, env_extra):
    env = dict(os.environ, **env_extra)
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *files]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, "exit %d\n%s\n%s" % (r.returncode, r.stdout[-3000:], r.stderr[-2000:])
    return r.stdout


def test_host_dispatch_and_validation_under_ubsan():
    from paper_2402_17764_amd.build import build_library_sanitized
    lib = build_library_sanitized()
    out = _run_tests(["tests/test_abi_cpu.py", "tests/test_dispatch_cpu.py", "tests/test_decode_bounds_cpu.py"],
                     {"BITNET_HIP_LIBRARY": lib})
    assert " passed" in out


def test_oracle_pins_under_ubsan():
    from oracle.build import build_oracle_sanitized
    lib = build_oracle_sanitized(os.path.join(ROOT, "oracle", "_build"))
    out = _run_tests(["tests/test_oracle_pins.py", "tests/test_oracle_block_pins.py"], {"BITNET_ORACLE_LIBRARY": lib})
    assert " passed" in out

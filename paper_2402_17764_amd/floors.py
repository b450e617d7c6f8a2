"""Loader of libbitnet_floors.so (csrc/floors.hip, csrc/prefill_ladder.hip): a read-only kernel, an MFMA-only kernel and the
prefill K loop built up ingredient by ingredient -- the yardsticks that bench.py, read_floor.py and prefill_ladder.py time
next to the product kernels.  Measurement aids; no part of the BitLinear library."""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libbitnet_floors.so")

READ_SHAPES = [(b, u) for b in (256, 512, 1024) for u in (2, 4, 8)]     # workgroups of 512 threads x loads in flight per thread


def load():
    """built by paper_2402_17764_amd.build (and by __graft_entry__.build()); built here if it is missing"""
    if not os.path.exists(LIB):
        from paper_2402_17764_amd.build import build_floors
        build_floors()
    lib = ctypes.CDLL(LIB)
    lib.read_only_launch.argtypes = [ctypes.c_void_p, ctypes.c_longlong, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    lib.mfma_only_launch.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_longlong, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                     ctypes.c_void_p]
    lib.prefill_ladder_launch.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_longlong, ctypes.c_int, ctypes.c_int,
                                          ctypes.c_void_p, ctypes.c_longlong, ctypes.c_void_p, ctypes.c_void_p]
    lib.l2_read_launch.argtypes = [ctypes.c_void_p, ctypes.c_longlong, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    return lib

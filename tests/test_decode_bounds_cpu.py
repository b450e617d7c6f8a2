"""Every byte the M <= 16 decode kernel touches stays inside its buffers, for every launch the benchmark makes and for
ragged shapes: a host replica of the kernel's address arithmetic (tests/decode_addr_replica.py) enumerates all
workgroups, lanes and K items of a launch, with the instantiation and the launch geometry taken from the library's own
launch description."""
import pytest

from decode_addr_replica import ceil_div, decode_launch_spans
from paper_2402_17764_amd import binding as B

_ENTRY = {"LINEAR": B.ENTRY_LINEAR, "LINEAR_FUSED": B.ENTRY_LINEAR_FUSED, "RMSNORM_LINEAR_FUSED": B.ENTRY_RMSNORM_LINEAR_FUSED,
          "SWIGLU_LINEAR_FUSED": B.ENTRY_SWIGLU_LINEAR_FUSED, "FFN_GATE_UP": B.ENTRY_FFN_GATE_UP,
          "FFN_GATE_UP_NORM": B.ENTRY_FFN_GATE_UP_NORM}


def _check(entry, dtype, M, N, K, gstride=0, out_bytes=2):
    d = B.entry_describe(_ENTRY[entry], M, N, K, x_dtype=B.BF16 if dtype != "f32" else B.F32)
    if d["kernel"] not in ("decode", "decode_pair"):
        return None
    kR, kS, kW, kD, xmode = d["params"]
    sp, sizes, lds, grid = decode_launch_spans(kR, kS, kW, kD, xmode, d["kernel"] == "decode_pair", M, N, K,
                                               out_bytes=out_bytes, gstride=gstride)
    assert (grid, 1) == d["grid"] and lds == d["lds"] and d["block"] == 64 * kS * kW, (entry, M, N, K, d, lds, grid)
    for name, span in sp.items():
        assert span.within(sizes[name]), (entry, dtype, M, N, K, d, name, span.lo, span.hi, sizes[name])
    # the stream is read completely: the weight loads reach the last byte of the packed matrix
    assert sp["packed"].lo == 0 and sp["packed"].hi == sizes["packed"]
    return d


def test_every_decode_launch_of_the_benchmark_stays_in_bounds():
    import bench
    seen = set()
    for (leg, entry, dtype, M, N, K) in bench.launch_inventory():
        d = _check(entry, dtype, M, N, K)
        if d:
            seen.add((d["kernel"], tuple(d["params"])))
    assert len(seen) >= 8


def test_ragged_decode_launches_stay_in_bounds():
    import parity_shapes as P
    for (M, N, K) in P.GEMV_SHAPES:
        if K % 16 == 0 and M <= 8:
            for ob in (2, 4):
                _check("LINEAR", "int8", M, N, K, gstride=M % 2, out_bytes=ob)
    for dtype in ("bf16", "f32"):
        for (M, N, K) in P.FUSED_SHAPES:
            _check("LINEAR_FUSED", dtype, M, N, K, gstride=1)
        for (M, N, K) in P.NORM_FUSED_SHAPES:
            _check("RMSNORM_LINEAR_FUSED", dtype, M, N, K)
        for (M, N, F) in P.SWIGLU_FUSED_SHAPES:
            _check("SWIGLU_LINEAR_FUSED", dtype, M, N, F)
        for (M, F, K) in P.FFN_GATE_UP_SHAPES:
            _check("FFN_GATE_UP", dtype, M, F, K, gstride=1)
            _check("FFN_GATE_UP_NORM", dtype, M, F, K)


def test_the_replica_catches_a_planted_overrun():
    """the check itself: a launch whose LDS allocation is one fold slot short, and one with a row block too many"""
    sp, sizes, lds, grid = decode_launch_spans(1, 4, 1, 4, 0, False, 1, 3200, 3200)
    assert sp["lds"].within(sizes["lds"]) and not sp["lds"].within(sizes["lds"] - 16)
    sp, sizes, _, _ = decode_launch_spans(1, 4, 1, 4, 0, False, 1, 3200, 3200)
    assert not sp["packed"].within(sizes["packed"] - 16) and not sp["y"].within(sizes["y"] - 2)

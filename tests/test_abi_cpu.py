"""CPU-side checks of the C ABI: the shared library loads, exports every function that
include/bitnet.h declares, and rejects bad arguments on the host before anything is launched
(no GPU is touched: every call below returns from validation)."""
import ctypes
import os
import re

import pytest

from paper_2402_17764_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "bitnet.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bitnet_[a-z0-9_]+)\s*\(", text)))


def test_header_functions_are_exported():
    lib = binding.load()
    names = _declared_functions()
    assert len(names) >= 10
    for n in names:
        assert hasattr(lib, n), "missing export: " + n
    assert sorted(binding.SYMBOLS) == names


def test_version_and_status_strings():
    lib = binding.load()
    assert binding.version() >= 100
    seen = set()
    for s in range(0, 9):
        msg = lib.bitnet_status_string(s).decode()
        assert msg and msg not in seen
        seen.add(msg)
    assert lib.bitnet_status_string(99).decode() == "unknown status"


def test_packed_bytes_follow_the_documented_layouts():
    assert binding.packed_bytes(4096, 1536, binding.PACK_2BIT) == 4096 * 1536 // 4
    assert binding.packed_bytes(17, 65, binding.PACK_2BIT) == 32 * 128 // 4
    assert binding.packed_bytes(1, 1, binding.PACK_2BIT) == 16 * 64 // 4
    assert binding.packed_bytes(3200, 3200, binding.PACK_TRIT5) == 3200 * 3200 // 5
    assert binding.packed_bytes(16, 321, binding.PACK_TRIT5) == 16 * 640 // 5
    assert binding.quantize_weights_workspace(57344, 8192) >= 4096
    with pytest.raises(binding.BitnetError) as e:
        binding.packed_bytes(0, 5)
    assert e.value.status == 2
    with pytest.raises(binding.BitnetError) as e:
        binding.packed_bytes(4, 4, 7)
    assert e.value.status == 4
    with pytest.raises(binding.BitnetError) as e:
        binding.packed_bytes(4, 1 << 19)          # K beyond the int32 accumulator limit
    assert e.value.status == 2


def test_host_validation_rejects_before_launch():
    lib = binding.load()
    vp = ctypes.c_void_p
    a = vp(0x1000)            # never dereferenced: validation fails first
    odd = vp(0x1001)
    NULL = vp(0)
    # NULL pointers
    assert lib.bitnet_quantize_acts(NULL, 0, 1, 16, a, a, NULL) == 1
    assert lib.bitnet_quantize_weights(a, 0, 4, 4, 0, NULL, a, a, 1 << 20, NULL) == 1
    assert lib.bitnet_linear(a, a, a, NULL, 1, 16, 64, 0, a, 0, NULL) == 1
    assert lib.bitnet_unpack_weights(a, 4, 4, 0, NULL, NULL) == 1
    assert lib.bitnet_rmsnorm_quantize(NULL, 0, NULL, 0.0, 1, 16, a, a, NULL) == 1
    i64 = ctypes.c_int64
    seg_ok = (i64 * 2)(32, 16)
    seg_ragged = (i64 * 2)(24, 24)       # a segment that is not the last must own whole 16-row blocks
    seg_short = (i64 * 2)(32, 8)
    assert lib.bitnet_quantize_weights_segmented(a, 0, 48, 64, 2, seg_ok, 0, a, a, NULL, 1 << 20, NULL) == 1
    assert lib.bitnet_quantize_weights_segmented(a, 0, 48, 64, 2, seg_ragged, 0, a, a, a, 1 << 20, NULL) == 2
    assert lib.bitnet_quantize_weights_segmented(a, 0, 48, 64, 2, seg_short, 0, a, a, a, 1 << 20, NULL) == 2
    assert lib.bitnet_quantize_weights_segmented(a, 0, 48, 64, 0, seg_ok, 0, a, a, a, 1 << 20, NULL) == 2
    assert lib.bitnet_quantize_weights_segmented(a, 0, 48, 64, 2, seg_ok, 1, a, a, a, 1 << 20, NULL) == 4
    assert lib.bitnet_quantize_weights_segmented(a, 0, 48, 64, 2, seg_ok, 0, a, a, a, 8, NULL) == 6
    assert lib.bitnet_linear_segmented(a, a, a, a, 1, 48, 64, 1, a, 0, 0, NULL) == 4          # 5-trit: no segment scales
    assert lib.bitnet_linear_segmented(a, a, a, NULL, 1, 48, 64, 0, a, 0, 0, NULL) == 1
    assert lib.bitnet_swiglu_quantize(a, 0, 1, 16, NULL, a, NULL) == 1
    assert lib.bitnet_rmsnorm_linear_fused(a, 0, NULL, 1e-6, a, NULL, 1, 16, 64, 0, a, 0, NULL) == 1
    assert lib.bitnet_rmsnorm_linear_fused(a, 0, NULL, -1.0, a, a, 1, 16, 64, 0, a, 0, NULL) == 2
    assert lib.bitnet_rmsnorm_linear_fused(a, 2, NULL, 1e-6, a, a, 1, 16, 64, 0, a, 0, NULL) == 3
    assert lib.bitnet_rmsnorm_linear_fused(a, 0, NULL, 1e-6, a, a, 1, 16, 64, 1, a, 0, NULL) == 4
    assert lib.bitnet_rmsnorm_linear_fused(a, 0, vp(0x1004), 1e-6, a, a, 1, 16, 64, 0, a, 0, NULL) == 5   # gain: 16-byte aligned
    assert lib.bitnet_rmsnorm_linear_fused(a, 0, NULL, 1e-6, a, a, 17, 16, 64, 0, a, 0, NULL) == 8
    assert lib.bitnet_rmsnorm_linear_fused_segmented(a, 0, NULL, 1e-6, a, a, 17, 16, 64, 0, a, 0, NULL) == 8
    assert lib.bitnet_swiglu_linear_fused(NULL, 0, a, a, 1, 16, 64, 0, a, 0, NULL) == 1
    assert lib.bitnet_swiglu_linear_fused(a, 0, a, a, 1, 16, 0, 0, a, 0, NULL) == 2
    assert lib.bitnet_swiglu_linear_fused(a, 2, a, a, 1, 16, 64, 0, a, 0, NULL) == 3
    assert lib.bitnet_swiglu_linear_fused(a, 0, a, a, 1, 16, 64, 1, a, 0, NULL) == 4
    assert lib.bitnet_swiglu_linear_fused(a, 0, odd, a, 1, 16, 64, 0, a, 0, NULL) == 5
    assert lib.bitnet_swiglu_linear_fused(a, 0, a, a, 17, 16, 64, 0, a, 0, NULL) == 8
    szp = ctypes.c_size_t(7)
    assert lib.bitnet_linear_workspace(128, 4096, 11008, None) == 1
    assert lib.bitnet_linear_workspace(520, 2048, 11008, ctypes.byref(szp)) == 0 and szp.value == 8 * 520 * 2048 * 4
    assert lib.bitnet_linear_workspace(128, 4096, 11008, ctypes.byref(szp)) == 0 and szp.value == 0   # batched decode serves it
    assert lib.bitnet_linear_workspace(64, 4096, 11008, ctypes.byref(szp)) == 0 and szp.value == 0
    assert lib.bitnet_linear_workspace(2048, 27648, 5120, ctypes.byref(szp)) == 0 and szp.value == 0
    assert lib.bitnet_linear_workspace(0, 4096, 11008, ctypes.byref(szp)) == 2
    assert lib.bitnet_linear_ws(a, a, a, NULL, 0, 128, 256, 512, 0, a, 0, 0, a, 1 << 20, NULL) == 1
    assert lib.bitnet_linear_ws(a, a, a, a, 0, 128, 256, 512, 0, a, 0, 0, odd, 1 << 20, NULL) == 5
    assert lib.bitnet_linear_ws(a, a, a, a, 0, 128, 256, 512, 0, a, 0, 0x203, a, 1 << 20, NULL) == 8        # 3 splits: no such variant
    assert lib.bitnet_linear_ws(a, a, a, a, 0, 128, 256, 512, 0, a, 0, 0x204, a, 1 << 20, NULL) == 6        # 2 K steps, 4 splits
    assert lib.bitnet_linear_ws(a, a, a, a, 0, 128, 256, 512, 0, a, 0, 0x202, a, 1024, NULL) == 6           # buffer too small
    assert lib.bitnet_linear_ws(a, a, a, a, 0, 128, 256, 512, 1, a, 0, 0x202, a, 1 << 20, NULL) == 8        # 5-trit format
    assert lib.bitnet_ffn_gate_up_fused(a, 0, 0, NULL, 0.0, a, NULL, 0, 1, 16, 64, 0, a, 0, NULL) == 1
    assert lib.bitnet_ffn_gate_up_fused(a, 0, 0, NULL, 0.0, a, a, 0, 1, 24, 64, 0, a, 0, NULL) == 2          # F % 16
    assert lib.bitnet_ffn_gate_up_fused(a, 0, 1, NULL, -1.0, a, a, 0, 1, 16, 64, 0, a, 0, NULL) == 2         # eps < 0 with norm
    assert lib.bitnet_ffn_gate_up_fused(a, 0, 0, NULL, -1.0, a, a, 0, 17, 16, 64, 0, a, 0, NULL) == 8        # eps ignored without
    assert lib.bitnet_ffn_gate_up_fused(a, 0, 0, NULL, 0.0, a, a, 0, 1, 16, 64, 0, a, 2, NULL) == 3          # I32 out
    assert lib.bitnet_ffn_gate_up_fused(a, 0, 0, NULL, 0.0, a, a, 0, 1, 16, 64, 1, a, 0, NULL) == 4
    assert lib.bitnet_ffn_gate_up_fused(a, 0, 1, vp(0x1004), 0.0, a, a, 0, 1, 16, 64, 0, a, 0, NULL) == 5
    # sharded weight quantization
    assert lib.bitnet_abs_sum(a, 0, 16, 64, NULL, a, 1 << 20, NULL) == 1
    assert lib.bitnet_abs_sum(a, 0, 0, 64, a, a, 1 << 20, NULL) == 2
    assert lib.bitnet_abs_sum(a, 2, 16, 64, a, a, 1 << 20, NULL) == 3
    assert lib.bitnet_abs_sum(a, 0, 16, 64, vp(0x1004), a, 1 << 20, NULL) == 5
    assert lib.bitnet_abs_sum(a, 0, 16, 64, a, a, 8, NULL) == 6
    assert lib.bitnet_quantize_weights_sharded(a, 0, 16, 64, 0, NULL, 1, 16, a, a, NULL) == 1
    assert lib.bitnet_quantize_weights_sharded(a, 0, 16, 64, 0, a, 0, 16, a, a, NULL) == 2        # no shares
    assert lib.bitnet_quantize_weights_sharded(a, 0, 16, 64, 0, a, 257, 16, a, a, NULL) == 2      # more than it folds
    assert lib.bitnet_quantize_weights_sharded(a, 0, 16, 64, 0, a, 2, 8, a, a, NULL) == 2         # whole smaller than the shard
    assert lib.bitnet_quantize_weights_sharded(a, 2, 16, 64, 0, a, 2, 32, a, a, NULL) == 3
    assert lib.bitnet_quantize_weights_sharded(a, 0, 16, 64, 5, a, 2, 32, a, a, NULL) == 4
    assert lib.bitnet_quantize_weights_sharded(a, 0, 16, 64, 0, vp(0x1004), 2, 32, a, a, NULL) == 5
    # the entry point that allocates nothing validates like bitnet_quantize_weights, before it touches a device
    assert lib.bitnet_quantize_weights_static(NULL, 0, 16, 64, 0, a, a, NULL) == 1
    assert lib.bitnet_quantize_weights_static(a, 0, 0, 64, 0, a, a, NULL) == 2
    assert lib.bitnet_quantize_weights_static(a, 2, 16, 64, 0, a, a, NULL) == 3
    assert lib.bitnet_quantize_weights_static(a, 0, 16, 64, 7, a, a, NULL) == 4
    assert lib.bitnet_quantize_weights_static(a, 0, 16, 64, 0, odd, a, NULL) == 5
    # launch descriptions of the fused entry points
    buf = ctypes.create_string_buffer(128)
    assert lib.bitnet_entry_describe(1, 1, 1, 4096, 4096, 0, 0, None, 128) == 1
    assert lib.bitnet_entry_describe(9, 1, 1, 4096, 4096, 0, 0, buf, 128) == 8
    assert lib.bitnet_entry_describe(1, 2, 1, 4096, 4096, 0, 0, buf, 128) == 3
    assert lib.bitnet_entry_describe(1, 1, 1, 4096, 4096, 1, 0, buf, 128) == 4                    # 2-bit format only
    assert lib.bitnet_entry_describe(1, 1, 17, 4096, 4096, 0, 0, buf, 128) == 8                   # more than 16 tokens
    assert lib.bitnet_entry_describe(4, 1, 1, 24, 4096, 0, 0, buf, 128) == 2                      # F % 16
    assert lib.bitnet_entry_describe(1, 1, 1, 4096, 4096, 0, 0, buf, 128) == 0
    assert buf.value.decode().startswith("kernel=decode params=1,4,1,4,2 grid=256x1 block=256")
    assert lib.bitnet_entry_describe(0, 0, 1, 4096, 4096, 0, 0, buf, 128) == 0 and b"params=1,4,1,4,0" in buf.value
    # shapes
    assert lib.bitnet_quantize_acts(a, 0, 0, 16, a, a, NULL) == 2
    assert lib.bitnet_rmsnorm_quantize(a, 0, NULL, 0.0, 1, 0, a, a, NULL) == 2
    assert lib.bitnet_rmsnorm_quantize(a, 0, NULL, -1.0, 1, 16, a, a, NULL) == 2     # negative eps
    assert lib.bitnet_swiglu_quantize(a, 0, 1, 0, a, a, NULL) == 2
    assert lib.bitnet_rmsnorm_quantize(a, 2, NULL, 0.0, 1, 16, a, a, NULL) == 3      # I32 is not an input type
    assert lib.bitnet_swiglu_quantize(odd, 1, 1, 16, a, a, NULL) == 5
    assert lib.bitnet_linear(a, a, a, a, 1, -3, 64, 0, a, 0, NULL) == 2
    assert lib.bitnet_linear(a, a, a, a, 1, 16, 1 << 20, 0, a, 0, NULL) == 2
    # dtypes / formats
    assert lib.bitnet_quantize_acts(a, 2, 1, 16, a, a, NULL) == 3
    assert lib.bitnet_quantize_weights(a, 5, 4, 4, 0, a, a, a, 1 << 20, NULL) == 3
    assert lib.bitnet_linear(a, a, a, a, 1, 16, 64, 0, a, 9, NULL) == 3
    assert lib.bitnet_linear(a, a, a, a, 1, 16, 64, 9, a, 0, NULL) == 4
    # alignment
    assert lib.bitnet_quantize_weights(a, 0, 4, 4, 0, odd, a, a, 1 << 20, NULL) == 5
    assert lib.bitnet_linear(a, a, odd, a, 1, 16, 64, 0, a, 0, NULL) == 5
    # workspace
    assert lib.bitnet_quantize_weights(a, 0, 4, 4, 0, a, a, a, 8, NULL) == 6
    # a forced kernel that cannot take the shape
    assert lib.bitnet_linear_variant(a, a, a, a, 257, 16, 64, 0, a, 0, binding.KERNEL_GEMV, NULL) == 8
    assert lib.bitnet_linear_variant(a, a, a, a, 100, 100000, 64, 0, a, 0, binding.KERNEL_GEMV, NULL) == 8   # too many rows
    assert lib.bitnet_linear_variant(odd, a, a, a, 1, 16, 64, 0, a, 0, binding.KERNEL_GEMV, NULL) == 8
    # fixed-tile selectors of the prefill kernel: tile codes outside the six built ones, or an operand it cannot take
    assert lib.bitnet_linear_variant(a, a, a, a, 65, 16, 64, 0, a, 0, 0x152, NULL) == 8
    assert lib.bitnet_linear_variant(a, a, a, a, 65, 16, 64, 0, a, 0, 0x143, NULL) == 8
    assert lib.bitnet_linear_variant(a, a, a, a, 65, 16, 64, 0, a, 0, 0x110, NULL) == 8
    assert lib.bitnet_linear_variant(odd, a, a, a, 65, 16, 64, 0, a, 0, binding.KERNEL_GEMM_TILES[(64, 128)], NULL) == 8
    assert lib.bitnet_linear_variant(a, a, a, a, 65, 16, 64, 0, a, 0, 77, NULL) == 8


def test_layout_decoder_roundtrip_on_a_hand_packed_tile():
    """The numpy layout decoder used by the GPU tests, checked on a tile packed by hand here."""
    import numpy as np
    from layout_ref import decode_2bit, quad_index_2bit
    rng = np.random.default_rng(3)
    for (N, K) in [(20, 70), (33, 600), (16, 256)]:
        codes = rng.integers(-1, 2, size=(N, K)).astype(np.int8)
        Np, Kq = 16 * ((N + 15) // 16), (K + 63) // 64
        words = np.zeros((Np * Kq, 4), np.uint32)
        for n in range(N):
            for k in range(K):
                c = int(codes[n, k]) & 3
                col = k % 64
                j, i, b = col // 16, (col % 16) // 4, col % 4
                words[quad_index_2bit(n, k // 64, N, K), j] |= np.uint32(c << (8 * b + 2 * i))
        got, pad_zero = decode_2bit(words.astype("<u4").tobytes(), N, K)
        assert pad_zero and np.array_equal(got, codes)
    # spot values of the index formula: 600 columns = 10 quads = two full steps and one of two quads
    assert quad_index_2bit(0, 0, 33, 600) == 0
    assert quad_index_2bit(17, 1, 33, 600) == 64 * 1 + 16 * 1 + 1          # rb 1, g 1, r 1
    assert quad_index_2bit(0, 4, 33, 600) == 64 * 3                          # step 1 starts after 3 row blocks
    assert quad_index_2bit(32, 9, 33, 600) == 64 * 3 * 2 + 16 * 2 * 2 + 16 * 1 + 0   # partial step: 2 quads per chunk


def test_trit5_layout_decoder_on_a_hand_packed_matrix():
    import numpy as np
    from layout_ref import decode_trit5
    rng = np.random.default_rng(4)
    for (N, K) in [(20, 70), (33, 700), (16, 320)]:
        codes = rng.integers(-1, 2, size=(N, K)).astype(np.int8)
        RB, steps = (N + 15) // 16, (K + 319) // 320
        buf = np.full((steps, RB, 4, 16, 16), 121, np.int32)           # 121 = five zero codes
        buf[:] = 0
        digits = np.ones((steps, RB, 4, 16, 16, 5), np.int32)          # code + 1, padding = 1
        for n in range(N):
            for k in range(K):
                s_, c = divmod(k, 320)
                g, q = divmod(c, 80)
                p_, d = (q // 4, q % 4) if q < 64 else (q - 64, 4)
                digits[s_, n // 16, g, n % 16, p_, d] = int(codes[n, k]) + 1
        buf = (digits * np.array([1, 3, 9, 27, 81])).sum(-1)
        got, pad_zero = decode_trit5(buf.astype(np.uint8).tobytes(), N, K)
        assert pad_zero and np.array_equal(got, codes)
        assert buf.size == binding.packed_bytes(N, K, binding.PACK_TRIT5)


def test_yardstick_library_loads_and_checks_its_arguments():
    """libbitnet_floors.so (the read-only, MFMA-only and K-loop-ladder kernels that bench.py and the measurement tools time
    next to the product): it loads, exports its entry points, and turns bad arguments into an error code before
    anything is launched -- no GPU is touched here."""
    from paper_2402_17764_amd import floors
    lib = floors.load()
    for name in ("read_only_launch", "mfma_only_launch", "prefill_ladder_launch", "l2_read_launch"):
        assert hasattr(lib, name)
    assert lib.read_only_launch(None, 1 << 20, None, 256, 4, None) == -3
    assert lib.read_only_launch(0x1000, 8, 0x1000, 256, 4, None) == -3
    assert lib.mfma_only_launch(None, None, 1 << 20, 512, 10, None, None) == -3
    assert lib.mfma_only_launch(0x1000, 0x1000, 1 << 20, 512, 0, 0x1000, None) == -3
    ok = (0x1000, 0x1000, 1 << 24, 512, 10, 0x1000, 256 << 20, 0x1000, None)
    assert lib.prefill_ladder_launch(5, None, *ok[1:]) == -3
    assert lib.prefill_ladder_launch(5, *ok[:6], 1 << 20, 0x1000, None) == -3          # streaming source below 64 MiB
    assert lib.prefill_ladder_launch(5, *ok[:6], 2 << 30, 0x1000, None) == -3          # ... or beyond one raw buffer
    assert lib.prefill_ladder_launch(5, *ok[:4], 0, *ok[5:]) == -3                     # no steps
    assert lib.prefill_ladder_launch(10, *ok) == -1                                    # no such rung
    assert lib.l2_read_launch(None, 2 << 20, 10, 512, 0, 0x1000, None) == -3
    assert lib.l2_read_launch(0x1000, (2 << 20) + 16, 10, 512, 1, 0x1000, None) == -3   # not a power of two
    assert lib.l2_read_launch(0x1000, 1 << 30, 10, 512, 1, 0x1000, None) == -3          # larger than the kernel's raw buffer allows

"""Host-side launch selection of bitnet_linear / bitnet_linear_ws, read back through bitnet_linear_describe (nothing is
launched, no GPU is touched).  The rules were fitted to measurements on MI355X; these tests pin the properties the
measurements established, on the projection shapes of the 3B ... 70B LLaMA family, so that a later edit of a rule
that breaks one of them fails here and not as a slow kernel on the GPU."""
import ctypes

import pytest

from paper_2402_17764_amd import binding as B

FAMILY = {"3b": (3200, 8640), "7b": (4096, 11008), "13b": (5120, 13824), "30b": (6656, 17920), "70b": (8192, 28672)}
SHAPES = []
for _fam, (_d, _f) in FAMILY.items():
    SHAPES += [(_fam + "_qkv", 3 * _d, _d), (_fam + "_o", _d, _d), (_fam + "_gate_up", 2 * _f, _d), (_fam + "_down", _d, _f)]

CUS = 256
LDS_PER_CU = 160 * 1024


def ceil_div(a, b):
    return -(-a // b)


@pytest.mark.parametrize("name,N,K", SHAPES)
def test_decode_shapes_do_not_pad_the_k_walk(name, N, K):
    """M <= 4: each of kS waves walks ceil(steps / kS) K steps padded to a multiple of the prefetch depth kD; the
    padding is masked work, so at most a quarter of the walk may be padding (K = 5120 over 4 waves at depth 4 would
    be 37 %)."""
    steps, RB = ceil_div(K, 256), ceil_div(N, 16)
    for M in (1, 2, 4, 5, 8):
        if M > 4 and RB >= 1024:            # five to eight tokens stay on this kernel only on the smaller layers
            continue
        d = B.linear_describe(M, N, K)
        assert d["kernel"] == "decode" and d["splits"] == 1
        kR, kS, kW, kD, xsrc = d["params"]
        walked = kS * ceil_div(ceil_div(steps, kS), kD) * kD
        assert steps / walked >= 0.75, (name, M, d)
        assert d["block"] == 64 * kS * kW and d["grid"] == (ceil_div(RB, kR * kW), 1)
        assert d["lds"] <= 64 * 1024
        if RB <= CUS:                       # one row block per workgroup, or CUs get none
            assert kR * kW == 1
        assert xsrc in (0, 1) and (xsrc == 0 or 128 + M * steps * 256 <= 60 * 1024)


def _one_round_rpw(RB, tiles):
    """the fewest row blocks per workgroup with which the launch is at most one workgroup per CU (None: no such form)"""
    for c in (1, 2, 4, 6, 8, 16):
        if ceil_div(RB, c) * tiles <= CUS:
            return c
    return None


@pytest.mark.parametrize("name,N,K", SHAPES)
def test_batched_decode_is_one_round_of_workgroups(name, N, K):
    """5 ... 64 tokens: activation rings within a CU's LDS; up to 4096 row blocks at most one workgroup per CU, with
    the fewest row blocks per workgroup that achieve it for the token tile taken; the tile is the smallest that holds M
    except on layers of up to 1024 row blocks, where a finer tile (several workgroups per row group, grid z) is
    taken when that moves less x_q + weight traffic through the L2s."""
    RB = ceil_div(N, 16)
    for M in (5, 8, 9, 16, 17, 32, 33, 48, 64):
        d = B.linear_describe(M, N, K)
        if M <= 8 and RB < 1024:            # the M <= 16 kernel is faster there (measured at eight tokens)
            assert d["kernel"] == "decode", (name, M, d)
            continue
        assert d["kernel"] in ("batched_decode", "batched_decode_loader") and d["splits"] == 1, (name, M, d)
        kMT, kR, kW, kS, kD, kLx = d["params"]
        full = 1 if M <= 16 else 2 if M <= 32 else 4
        assert kMT in (1, 2, 4) and kMT <= full
        if RB > 1024 or M <= 16:
            assert kMT == full
        tiles = ceil_div(M, 16 * kMT)
        assert d["lds"] == kS * (kLx + 1) * kMT * 4096 <= LDS_PER_CU
        assert d["block"] == 64 * (kS * kW + (d["kernel"] == "batched_decode_loader")) <= 1024
        rpw = kR * kW
        assert d["grid"] == (ceil_div(RB, rpw) * tiles, 1)
        if RB <= 4096:
            assert d["grid"][0] <= CUS, (name, M, d)
            assert rpw == _one_round_rpw(RB, tiles), (name, M, d)
        if RB <= 1024:
            traffic = lambda t, c: ceil_div(RB, c) * ceil_div(M, 16 * t) * (16 * t + 4 * c)
            assert traffic(kMT, rpw) <= traffic(full, _one_round_rpw(RB, 1)), (name, M, d)


def test_batched_decode_token_tiles_on_small_layers():
    """the measured cases: 7B down at 64 and 32 tokens, 13B down at 48, 70B O at 64"""
    assert B.linear_describe(64, 4096, 11008)["params"][:3] == [1, 2, 2] and B.linear_describe(64, 4096, 11008)["grid"] == (256, 1)
    assert B.linear_describe(32, 4096, 11008)["params"][:3] == [1, 1, 2]
    assert B.linear_describe(48, 5120, 13824)["params"][:3] == [1, 2, 2] and B.linear_describe(48, 5120, 13824)["grid"] == (240, 1)
    assert B.linear_describe(64, 8192, 8192)["grid"] == (256, 1)
    assert B.linear_describe(64, 22016, 4096)["params"][0] == 4          # many row blocks: one tile of 64 tokens


def test_batched_decode_never_splits_by_itself():
    """token tiles over workgroups do what split-K was for, without its second launch"""
    for (M, N, K) in [(64, 4096, 22016), (48, 8192, 28672), (64, 4096, 11008), (33, 3200, 8640)]:
        assert B.linear_describe(M, N, K, workspace_bytes=8 * M * N * 4)["splits"] == 1
        assert B.linear_workspace(M, N, K) == 0


def test_prefill_tiles_follow_the_measured_cases():
    """The cases the cost model's comment quotes, and its limits: big grids stay on the widest tile, small ones take
    narrow tiles so that CUs are not left idle, split-K only with a workspace, a long K and few tiles."""
    assert B.linear_describe(2048, 27648, 5120)["params"] == [128, 256]
    # many tiles whose count suits 256 CUs: eight waves in two row groups on one token tile (measured: 127 -> 116 us,
    # 1231 -> 1207 us); where whole rounds of such tiles fit badly (864 tiles: 200 -> 220 us) the four-wave tiles stay
    assert B.linear_describe(2048, 15360, 5120)["params"] == [128, 512]
    assert B.linear_describe(4096, 57344, 8192)["params"] == [128, 512]
    assert B.linear_describe(1024, 15360, 5120)["params"] == [128, 512]           # 240 tiles: 65 -> 62.5 us
    assert B.linear_describe(512, 27648, 5120)["params"] == [128, 256]            # 216 such tiles: too few of the CUs
    # one workgroup per CU at most: eight waves in two K groups (measured: 19.2 -> 18.1 us, 39.7 -> 37.5 us)
    assert B.linear_describe(512, 5120, 5120)["params"] == [96, 128, 2]
    assert B.linear_describe(520, 5120, 5120)["params"] == [96, 128, 2]
    assert B.linear_describe(512, 5120, 13824)["params"] == [96, 128, 2]
    assert B.linear_describe(1024, 4096, 11008)["params"] == [64, 256, 2]
    assert B.linear_describe(768, 5120, 5120)["params"] == [64, 128]              # 480 tiles: more than one round
    assert B.linear_describe(512, 5120, 5120, workspace_bytes=8 * 512 * 5120 * 4)["params"] == [96, 128, 2]
    for (M, N, K) in [(257, 3200, 3200), (300, 9600, 3200), (1024, 4096, 11008), (2048, 8192, 28672), (4096, 3200, 8640),
                      (512, 5120, 13824), (300, 8192, 28672), (2048, 15360, 5120), (4096, 8192, 28672)]:
        d = B.linear_describe(M, N, K)
        tm, tn = d["params"][:2]
        groups = d["params"][2] if len(d["params"]) == 3 else 2 if tn == 512 else 1
        assert d["kernel"] == "prefill" and d["splits"] == 1 and d["block"] == 256 * groups
        assert d["grid"] == (ceil_div(M, tm) * ceil_div(N, tn), 1)
        if tn == 512:
            assert d["grid"][0] >= 224 and d["lds"] <= LDS_PER_CU                 # (nearly) whole rounds of one workgroup per CU
        elif groups == 2:
            assert d["grid"][0] <= 256 and d["lds"] <= LDS_PER_CU                 # one round of one workgroup per CU
        else:
            assert d["lds"] <= LDS_PER_CU // 2                  # two workgroups per CU
    big = 8 * 520 * 8192 * 4
    d = B.linear_describe(520, 2048, 11008, workspace_bytes=big)
    assert d["splits"] in (2, 4, 8) and d["grid"][1] == d["splits"]
    # a long K on few tiles from 280 tokens on: the eight-wave form beats splitting through memory (measured 79 against
    # 88 us, 41.5 against 46.8 us), so the workspace goes unused there
    for (M, N, K) in [(300, 8192, 28672), (280, 6656, 17920)]:
        d = B.linear_describe(M, N, K, workspace_bytes=big)
        assert d["splits"] == 1 and d["params"] == [96, 128, 2]
    assert B.linear_describe(520, 2048, 4096, workspace_bytes=big)["splits"] == 1       # K = 4096: nothing to gain
    assert B.linear_describe(2048, 4096, 11008, workspace_bytes=8 * 2048 * 4096 * 4)["splits"] == 1
    assert B.linear_describe(520, 2048, 11008, workspace_bytes=2 * 520 * 2048 * 4)["splits"] <= 2   # what fits


def test_batched_decode_beyond_64_tokens_only_as_one_round():
    """65 ... 512 tokens (from 257 on only with K >= 5120): the decode kernels run where a launch of at most 256
    workgroups with at most eight row blocks each exists (tiles of 32 tokens while six row blocks suffice, else of
    64); everything else is prefill."""
    for (name, N, K) in SHAPES:
        RB = ceil_div(N, 16)
        for M in (65, 96, 128, 192, 256, 257, 384, 512, 513, 1024):
            d = B.linear_describe(M, N, K)
            c2 = next((c for c in (1, 2, 4, 6) if ceil_div(RB, c) * ceil_div(M, 32) <= CUS), None)
            c4 = next((c for c in (1, 2, 4, 6, 8) if ceil_div(RB, c) * ceil_div(M, 64) <= CUS), None)
            if M > 512 or (M > 256 and K < 5120) or (c2 is None and c4 is None):
                assert d["kernel"] == "prefill", (name, M, d)
                continue
            assert d["kernel"] in ("batched_decode", "batched_decode_loader"), (name, M, d)
            kMT, kR, kW = d["params"][:3]
            assert (kMT, kR * kW) == ((2, c2) if c2 else (4, c4)), (name, M, d)
            assert d["grid"] == (ceil_div(RB, kR * kW) * ceil_div(M, 16 * kMT), 1) and d["grid"][0] <= CUS
    assert B.linear_describe(128, 4096, 11008)["params"] == [2, 2, 2, 4, 2, 2]           # 7B down: 13.6 us, prefill 35.9
    assert B.linear_describe(512, 4096, 11008)["params"] == [4, 2, 4, 1, 4, 2]           # 28.3 us, prefill 36.0
    assert B.linear_describe(512, 4096, 4096)["kernel"] == "prefill"                     # short K
    assert B.linear_describe(512, 5120, 13824)["kernel"] == "prefill"                    # 320 x 8 workgroups: two rounds
    assert B.linear_describe(256, 8192, 8192)["kernel"] == "batched_decode_loader"
    assert B.linear_describe(192, 12288, 4096)["kernel"] == "prefill"
    assert B.linear_describe(96, 22016, 4096)["kernel"] == "prefill"


def test_fallbacks_and_errors():
    assert B.linear_describe(3, 100, 70)["kernel"] == "reference"                   # K not a multiple of 16
    assert B.linear_describe(100, 64, 72)["kernel"] == "reference"
    assert B.linear_describe(1, 17280, 3200, fmt=B.PACK_TRIT5)["kernel"] == "trit5_decode"
    assert B.linear_describe(100, 17280, 3200, fmt=B.PACK_TRIT5)["kernel"] == "trit5_decode"   # 16 tokens at a time
    # 5-trit weights with a workspace that holds the 2-bit copy: the repacking pass, then the 2-bit plan for the rest
    need = B.linear_workspace(2048, 27648, 5120, B.PACK_TRIT5)
    assert need >= 27648 * 5120 // 4
    d = B.linear_describe(2048, 27648, 5120, fmt=B.PACK_TRIT5, workspace_bytes=need)
    assert d["repack"] == "trit5_to_2bit" and d["kernel"] == "prefill" and d["params"] == [128, 256]
    assert B.linear_describe(2048, 27648, 5120, fmt=B.PACK_TRIT5, workspace_bytes=need - 257)["repack"] is None
    assert B.linear_describe(16, 27648, 5120, fmt=B.PACK_TRIT5, workspace_bytes=need)["kernel"] == "trit5_decode"
    assert B.linear_describe(2048, 27648, 5120)["repack"] is None
    lib = B.load()
    buf = ctypes.create_string_buffer(128)
    assert lib.bitnet_linear_describe(1, 4096, 4096, 0, 0, None, 128) == 1
    assert lib.bitnet_linear_describe(1, 4096, 4096, 0, 0, buf, 0) == 1
    assert lib.bitnet_linear_describe(0, 4096, 4096, 0, 0, buf, 128) == 2
    assert lib.bitnet_linear_describe(1, 4096, 4096, 7, 0, buf, 128) == 4
    assert lib.bitnet_linear_describe(1, 4096, 4096, 0, 0, buf, 8) == 6                # text does not fit
    assert lib.bitnet_linear_describe(1, 4096, 4096, 0, 0, buf, 128) == 0
    assert buf.value.decode().startswith("kernel=decode params=1,4,1,4,0 grid=256x1 block=256")


def test_every_launch_shape_is_within_the_hardware_limits():
    """Seeded random shapes, ragged ones included: whatever kernel a shape gets, its launch covers the output, a
    workgroup is a whole number of wavefronts up to 1024 threads, and its LDS fits a CU."""
    import random
    rng = random.Random(1758)
    kernels = set()
    for _ in range(4000):
        M = rng.choice([1, 2, 3, 4, 5, 15, 16, 17, 33, 64, 65, 100, 128, 200, 256, 257, 400, 512, 513, 1000, 2048, 5000])
        N = rng.choice([1, 15, 16, 17, 100, 1000, 3200, 4096, 8192, 12288, 22016, 57344, 128256]) + rng.choice([0, 0, 0, 1, 16, 48])
        K = rng.choice([16, 64, 256, 272, 1024, 3200, 4096, 5120, 8640, 11008, 28672, 65536]) + rng.choice([0, 0, 0, 16, 64, 7])
        ws = rng.choice([0, 0, 8 * M * N * 4])
        d = B.linear_describe(M, N, K, workspace_bytes=ws)
        kernels.add(d["kernel"])
        RB = ceil_div(N, 16)
        if d["kernel"] == "reference":
            assert K % 16 != 0, (M, N, K, d)
            continue
        assert d["block"] % 64 == 0 and 64 <= d["block"] <= 1024, (M, N, K, d)
        assert d["lds"] <= LDS_PER_CU and 1 <= d["grid"][0] < 2 ** 31 and 1 <= d["grid"][1] < 65536, (M, N, K, d)
        assert d["splits"] == d["grid"][1] and (ws or d["splits"] == 1), (M, N, K, d)
        if d["kernel"] == "decode":
            kR, kS, kW, kD, _ = d["params"]
            assert (M <= 4 or (M <= 8 and RB < 1024)) and d["grid"][0] == ceil_div(RB, kR * kW) and d["block"] == 64 * kS * kW
        elif d["kernel"].startswith("batched_decode"):
            kMT, kR, kW, kS, kD, kLx = d["params"]
            assert 4 < M <= 512 and (M > 8 or RB >= 1024) and d["grid"][0] == ceil_div(RB, kR * kW) * ceil_div(M, 16 * kMT)
        else:
            assert d["kernel"] == "prefill", (M, N, K, d)
            tm, tn = d["params"][:2]
            groups = d["params"][2] if len(d["params"]) == 3 else 2 if tn == 512 else 1
            assert d["grid"][0] == ceil_div(M, tm) * ceil_div(N, tn) and d["block"] == 256 * groups and groups in (1, 2)
            if tn == 512:                    # two row groups: one workgroup per CU, at least 7/8 of a round of them
                assert d["grid"][0] >= 224 and d["splits"] == 1 and tm == 128, (M, N, K, d)
            elif groups == 2:                # one workgroup per CU, one round, never together with a split through memory
                assert d["grid"][0] <= 256 and d["splits"] == 1 and (tm, tn) in ((96, 128), (64, 256)), (M, N, K, d)
    assert kernels == {"reference", "decode", "batched_decode", "batched_decode_loader", "prefill"}


def test_decode_shapes_on_large_layers_follow_the_measured_cases():
    """One or two tokens on layers of 1024 row blocks and more take x_q from LDS (last parameter 1): two K-split waves
    per row block where four waves split K evenly, eight single-row-block waves without a split where they cannot
    (K = 5120); from three tokens on the wide-wave forms on x_q from global memory."""
    assert B.linear_describe(1, 35840, 6656)["params"] == [1, 2, 2, 4, 1]            # 30B gate/up: 16.1 -> 14.6 us
    assert B.linear_describe(2, 57344, 8192)["params"] == [1, 2, 2, 4, 1]            # 70B gate/up: 23.0 -> 21.3 us at M = 1
    assert B.linear_describe(4, 35840, 6656)["params"] == [4, 1, 4, 3, 0]
    assert B.linear_describe(1, 22016, 4096)["params"] == [1, 2, 2, 4, 1]            # 7B gate/up
    assert B.linear_describe(1, 19968, 6656)["params"] == [1, 2, 2, 4, 1]            # 30B QKV
    assert B.linear_describe(1, 27648, 5120)["params"] == [1, 1, 8, 5, 1]            # 13B gate/up: 9.0 -> 8.2 us
    assert B.linear_describe(1, 27648, 5120)["grid"] == (216, 1)
    assert B.linear_describe(2, 27648, 5120)["params"] == [2, 1, 4, 4, 0]
    assert B.linear_describe(1, 17280, 3200)["params"] == [1, 4, 1, 4, 1]            # 3B gate/up keeps four K-split waves


# ------------------------------------------------------------------------------------------------
# every launch the benchmark times runs a kernel instantiation that a GPU parity test reaches
# ------------------------------------------------------------------------------------------------
_ENTRY = {"LINEAR": B.ENTRY_LINEAR, "LINEAR_FUSED": B.ENTRY_LINEAR_FUSED, "RMSNORM_LINEAR_FUSED": B.ENTRY_RMSNORM_LINEAR_FUSED,
          "SWIGLU_LINEAR_FUSED": B.ENTRY_SWIGLU_LINEAR_FUSED, "FFN_GATE_UP": B.ENTRY_FFN_GATE_UP,
          "FFN_GATE_UP_NORM": B.ENTRY_FFN_GATE_UP_NORM}
_DTYPE = {"bf16": B.BF16, "f32": B.F32, "int8": B.BF16}


def _form(entry, dtype, M, N, K):
    """the kernel instantiation a call gets: family + template parameters (the launch grid is not part of it)"""
    d = B.entry_describe(_ENTRY[entry], M, N, K, x_dtype=_DTYPE[dtype])
    return (d["kernel"], tuple(d["params"]), d["splits"])


def _forms_reached_by_the_gpu_parity_tests():
    """Replays the shape lists of tests/test_gpu_parity.py (each case there is compared with the oracle) through the
    same launch selection.  Returns {form: example case}."""
    import parity_shapes as P
    reached = {}

    def add(entry, dtype, M, N, K):
        reached.setdefault(_form(entry, dtype, M, N, K), (entry, dtype, M, N, K))

    for (M, N, K) in P.GEMV_SHAPES + P.GEMM_SHAPES:                  # _run_linear_case: KERNEL_AUTO is among the kernels run
        if K % 16 == 0:
            add("LINEAR", "int8", M, N, K)
    for (M, N, K, _) in P.FULL_SIZE_GEMM:
        add("LINEAR", "int8", M, N, K)
    for (_, _name, K, N, Ms) in P.FULL_SIZE_DECODE:
        for M in Ms:
            add("LINEAR", "int8", M, N, K)
            if M == 1:
                add("LINEAR_FUSED", "bf16", M, N, K)
                if N % 32 == 0 and "gate_up" in (_name,):
                    add("FFN_GATE_UP_NORM", "bf16", M, N // 2, K)
    for (_, K, N) in P.FAMILY_DECODE:
        for M in (1, 3):
            add("LINEAR", "int8", M, N, K)
            if 128 + M * ceil_div(K, 256) * 256 <= 60 * 1024:
                add("LINEAR_FUSED", "bf16", M, N, K)
    for dtype in ("f32", "bf16"):
        for (M, N, K) in P.FUSED_SHAPES:
            add("LINEAR_FUSED", dtype, M, N, K)
        for (M, N, K) in P.NORM_FUSED_SHAPES:
            add("RMSNORM_LINEAR_FUSED", dtype, M, N, K)
        for (M, N, F) in P.SWIGLU_FUSED_SHAPES:
            add("SWIGLU_LINEAR_FUSED", dtype, M, N, F)
        for (M, F, K) in P.FFN_GATE_UP_SHAPES:
            add("FFN_GATE_UP", dtype, M, F, K)
            add("FFN_GATE_UP_NORM", dtype, M, F, K)
            add("LINEAR_FUSED", dtype, M, 2 * F, K)
            add("RMSNORM_LINEAR_FUSED", dtype, M, 2 * F, K)
    # test_decoder_chain_in_a_hip_graph_matches_the_oracle: the 3B chain at its exact shapes, bf16
    add("RMSNORM_LINEAR_FUSED", "bf16", 1, 9600, 3200)
    add("RMSNORM_LINEAR_FUSED", "bf16", 1, 17280, 3200)
    add("FFN_GATE_UP_NORM", "bf16", 1, 8640, 3200)
    # test_linear_prefill_70b_full_size_sampled
    add("LINEAR", "int8", 4096, 57344, 8192)
    add("LINEAR", "int8", 4096, 8192, 28672)
    return reached


def test_every_benchmark_launch_runs_a_parity_tested_kernel_form():
    """bench.launch_inventory() lists every product launch a default benchmark run times; each must get a kernel
    instantiation (family, template parameters, split) that at least one oracle-checked GPU case gets too -- for the
    decode workloads at the exact shape."""
    import bench
    import parity_shapes as P
    reached = _forms_reached_by_the_gpu_parity_tests()
    inv = bench.launch_inventory()
    assert len(inv) >= 50
    missing = []
    for (leg, entry, dtype, M, N, K) in inv:
        if _form(entry, dtype, M, N, K) not in reached:
            missing.append((leg, entry, dtype, M, N, K, _form(entry, dtype, M, N, K)))
    assert not missing, missing
    # the two instantiations that carry the decode headlines, at their exact shapes
    fused_exact = {(M, N, K) for (M, N, K) in P.FUSED_SHAPES} | {(1, N, K) for (_, _, K, N, Ms) in P.FULL_SIZE_DECODE if 1 in Ms}
    for (leg, entry, dtype, M, N, K) in inv:
        if leg in ("headline", "decode_3b_m1"):
            assert (M, N, K) in fused_exact, (leg, M, N, K)
    assert _form("LINEAR_FUSED", "bf16", 1, 9600, 3200) == ("decode", (1, 4, 1, 4, 2), 1)      # 3B QKV / O, 7B QKV / O
    assert _form("LINEAR_FUSED", "bf16", 1, 3200, 3200) == ("decode", (1, 4, 1, 4, 2), 1)
    assert _form("LINEAR_FUSED", "bf16", 1, 57344, 8192)[0] == "decode"


def test_no_dispatch_rule_asks_for_an_instantiation_that_is_not_built():
    """Seeded random shapes through every fused entry point: the launch selection must always land on a built
    instantiation (a rule that names a launch shape without the needed activation mode returns an error status)."""
    import random
    rng = random.Random(17764)
    seen = set()
    for _ in range(3000):
        M = rng.choice([1, 1, 1, 2, 3, 4, 8, 16])
        N = 16 * rng.choice([1, 3, 16, 100, 200, 256, 257, 320, 321, 400, 512, 513, 640, 641, 768, 769, 1024, 1025, 1536, 2048, 3584, 8000])
        K = 16 * rng.choice([1, 5, 16, 17, 64, 100, 128, 200, 208, 256, 320, 384, 416, 512, 540, 688, 864, 1024, 1120, 1792])
        if 512 + M * ceil_div(K, 256) * 256 > 65536:
            continue
        for entry in ("LINEAR_FUSED", "RMSNORM_LINEAR_FUSED", "SWIGLU_LINEAR_FUSED", "FFN_GATE_UP", "FFN_GATE_UP_NORM"):
            for dtype in ("bf16", "f32"):
                d = B.entry_describe(_ENTRY[entry], M, N, K, x_dtype=_DTYPE[dtype])
                assert d["kernel"] in ("decode", "decode_pair") and d["block"] <= 1024 and d["lds"] <= 65536, (entry, M, N, K, d)
                assert d["params"][4] in ((2, 4, 6) if dtype == "bf16" else (3, 5, 7)), (entry, M, N, K, d)
                seen.add((d["kernel"], tuple(d["params"][:4])))
    assert len(seen) >= 15

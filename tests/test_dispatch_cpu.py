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
    assert B.linear_describe(4096, 57344, 8192)["params"] == [128, 256]
    assert B.linear_describe(512, 5120, 5120)["params"] == [96, 128]
    assert B.linear_describe(520, 5120, 5120)["params"] == [96, 128]
    for (M, N, K) in [(257, 3200, 3200), (300, 9600, 3200), (1024, 4096, 11008), (2048, 8192, 28672), (4096, 3200, 8640)]:
        d = B.linear_describe(M, N, K)
        tm, tn = d["params"]
        assert d["kernel"] == "prefill" and d["splits"] == 1 and d["block"] == 256
        assert d["grid"] == (ceil_div(M, tm) * ceil_div(N, tn), 1)
        assert d["lds"] <= LDS_PER_CU // 2                      # two workgroups per CU
    big = 8 * 520 * 8192 * 4
    d = B.linear_describe(520, 2048, 11008, workspace_bytes=big)
    assert d["splits"] in (2, 4, 8) and d["grid"][1] == d["splits"]
    assert B.linear_describe(300, 8192, 28672, workspace_bytes=big)["splits"] > 1
    assert B.linear_describe(280, 6656, 17920, workspace_bytes=big)["splits"] > 1
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
            tm, tn = d["params"]
            assert d["grid"][0] == ceil_div(M, tm) * ceil_div(N, tn) and d["block"] == 256
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

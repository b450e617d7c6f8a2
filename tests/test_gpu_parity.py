"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI.

Bars (BitLinear of arXiv 2402.17764, Section 2): ternary codes, gamma, int8 activations, per-token
scales and int32 accumulators are bit-exact; the rescaled output is within 1e-5 relative (fp32 out)
or 1e-2 relative (bf16 out) of the oracle's fp64 value.
"""
import json
import os
import sys

import numpy as np
import pytest

import oracle
from layout_ref import decode_2bit, decode_trit5
from parity_shapes import (FAMILY_DECODE, FFN_GATE_UP_SHAPES, FULL_SIZE_DECODE, FULL_SIZE_GEMM, FUSED_SHAPES, GEMM_SHAPES,
                           GEMV_SHAPES, NORM_FUSED_SHAPES, SWIGLU_FUSED_SHAPES)
from paper_2402_17764_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

RTOL_F32 = 1e-5
RTOL_BF16 = 1e-2
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def bf16_tensor(bits_u16):
    return torch.from_numpy(bits_u16.view(np.int16).copy()).cuda().view(torch.bfloat16)


def check_y(y_gpu, y_ref, rtol):
    y_gpu = np.asarray(y_gpu, np.float64)
    zero = y_ref == 0
    assert np.all(y_gpu[zero] == 0), "acc == 0 must give exactly 0"
    err = np.abs(y_gpu[~zero] - y_ref[~zero]) / np.abs(y_ref[~zero])
    assert err.size == 0 or err.max() <= rtol, "max rel err %.3g > %.1g" % (err.max(), rtol)


# ------------------------------------------------------------------------------------------------
# weights
# ------------------------------------------------------------------------------------------------
WEIGHT_SHAPES = [(4096, 1536), (16, 64), (1, 1), (37, 129), (100, 70), (17, 1000), (33, 2050), (250, 4100)]


@pytest.mark.parametrize("N,K", WEIGHT_SHAPES)
def test_quantize_weights_matches_oracle(gpu_lib, N, K):
    say("quantize_weights fp32 N=%d K=%d" % (N, K))
    W = synth.weights(N, K, config=0, layer=N % 7, tensor=0)
    codes_ref, gamma_ref = oracle.quantize_weights(W)
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    torch.cuda.synchronize()
    assert gamma.cpu().numpy()[0].tobytes() == np.float32(gamma_ref).tobytes(), "gamma bits differ"
    codes = gpu_lib.unpack_weights(packed, N, K).cpu().numpy()
    assert np.array_equal(codes, codes_ref)
    # the bytes follow the documented layout, and padding is zero codes
    assert packed.numel() == gpu_lib.packed_bytes(N, K)
    dec, pad_zero = decode_2bit(packed.cpu().numpy(), N, K)
    assert pad_zero and np.array_equal(dec, codes_ref)


def test_quantize_weights_bf16_input_and_unaligned_rows(gpu_lib):
    say("quantize_weights bf16 + odd K")
    for (N, K) in [(64, 256), (19, 77)]:
        Wf, bits = synth.to_bf16(synth.weights(N, K, config=0, layer=5))
        codes_ref, gamma_ref = oracle.quantize_weights(Wf)
        packed, gamma = gpu_lib.quantize_weights(bf16_tensor(bits).view(N, K))
        assert gamma.cpu().numpy()[0] == gamma_ref
        assert np.array_equal(gpu_lib.unpack_weights(packed, N, K).cpu().numpy(), codes_ref)
    # fp32 matrix whose base pointer is only 4-byte aligned
    N, K = 24, 132
    W = synth.weights(N, K, config=0, layer=6)
    buf = torch.empty(N * K + 1, dtype=torch.float32, device="cuda")
    buf[1:] = dev(W).reshape(-1)
    codes_ref, gamma_ref = oracle.quantize_weights(W)
    packed, gamma = gpu_lib.quantize_weights(buf[1:].view(N, K))
    assert gamma.cpu().numpy()[0] == gamma_ref
    assert np.array_equal(gpu_lib.unpack_weights(packed, N, K).cpu().numpy(), codes_ref)


def test_quantize_weights_vector_paths_and_partly_aligned_bases(gpu_lib):
    """The |W| sum reads 16-byte vectors (8 bf16 or 4 fp32 elements) in rounds of four per thread, the packing pass 16- or
    8-byte vectors per row and several items per workgroup: sizes that go round those loops more than once, and base
    pointers aligned for one pass but not for the other."""
    say("quantize_weights bf16 2048 x 3072 (vector paths, several rounds)")
    N, K = 2048, 3072
    Wf, bits = synth.to_bf16(synth.weights(N, K, config=0, layer=3))
    codes_ref, gamma_ref = oracle.quantize_weights(Wf)
    packed, gamma = gpu_lib.quantize_weights(bf16_tensor(bits).view(N, K))
    assert gamma.cpu().numpy()[0].tobytes() == np.float32(gamma_ref).tobytes()
    assert np.array_equal(gpu_lib.unpack_weights(packed, N, K).cpu().numpy(), codes_ref)
    say("quantize_weights bf16, base 8-byte but not 16-byte aligned")
    N, K = 40, 264
    Wf, bits = synth.to_bf16(synth.weights(N, K, config=0, layer=4))
    buf = torch.empty(N * K + 4, dtype=torch.bfloat16, device="cuda")
    buf[4:] = bf16_tensor(bits).reshape(-1)
    assert buf[4:].data_ptr() % 16 == 8
    codes_ref, gamma_ref = oracle.quantize_weights(Wf)
    packed, gamma = gpu_lib.quantize_weights(buf[4:].view(N, K))
    assert gamma.cpu().numpy()[0].tobytes() == np.float32(gamma_ref).tobytes()
    assert np.array_equal(gpu_lib.unpack_weights(packed, N, K).cpu().numpy(), codes_ref)
    say("quantize_weights fp32, base 8-byte aligned, K a multiple of 4")
    N, K = 35, 520
    W = synth.weights(N, K, config=0, layer=2)
    buf = torch.empty(N * K + 2, dtype=torch.float32, device="cuda")
    buf[2:] = dev(W).reshape(-1)
    codes_ref, gamma_ref = oracle.quantize_weights(W)
    packed, gamma = gpu_lib.quantize_weights(buf[2:].view(N, K))
    assert gamma.cpu().numpy()[0].tobytes() == np.float32(gamma_ref).tobytes()
    assert np.array_equal(gpu_lib.unpack_weights(packed, N, K).cpu().numpy(), codes_ref)


def test_quantize_weights_larger_than_the_cached_tail(gpu_lib):
    """Above 192 MB the |W| sum reads the head of W with the streaming cache policy and only the tail normally: a
    235 MB matrix takes both branches; gamma and every code against the oracle."""
    say("quantize_weights fp32 7168 x 8192 (235 MB)")
    N, K = 7168, 8192
    W = synth.weights(N, K, config=4, layer=1, tensor=0)
    codes_ref, gamma_ref = oracle.quantize_weights(W)
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    assert gamma.cpu().numpy()[0].tobytes() == np.float32(gamma_ref).tobytes(), "gamma bits differ"
    assert np.array_equal(gpu_lib.unpack_weights(packed, N, K).cpu().numpy(), codes_ref)


def test_quantize_weights_edge_values(gpu_lib):
    say("quantize_weights edge values")
    # all-zero matrix
    Z = np.zeros((20, 70), np.float32)
    packed, gamma = gpu_lib.quantize_weights(dev(Z))
    assert gamma.cpu().numpy()[0] == 0 and not packed.cpu().numpy().any()
    # exact ties of Eq. (2): gamma + eps == 2^-3, so W = q/8 reproduces the golden q list exactly
    g = json.load(open(os.path.join(GOLDEN, "rounding_ties.json")))["round_clip"]
    q = np.array(g["q"], np.float32)
    # a matrix that contains the tie values scaled by its own gamma + eps: both sides must agree bit for bit
    W = synth.weights(8, 64, config=0, layer=8)
    gam, _ = oracle.absmean_gamma(W)
    d = np.float32(np.float32(gam) + np.float32(1e-5))
    W[0, : q.size] = q * d
    codes_ref, gamma_ref = oracle.quantize_weights(W)
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    assert gamma.cpu().numpy()[0] == gamma_ref
    assert np.array_equal(gpu_lib.unpack_weights(packed, 8, 64).cpu().numpy(), codes_ref)
    # wide dynamic range: the compensated sum must not lose the small terms
    W = np.full((4, 64), 1.0, np.float32)
    W[0, 0] = 1e8
    W[3, 63] = -1e8
    codes_ref, gamma_ref = oracle.quantize_weights(W)
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    assert gamma.cpu().numpy()[0] == gamma_ref
    assert np.array_equal(gpu_lib.unpack_weights(packed, 4, 64).cpu().numpy(), codes_ref)
    # determinism: same bytes twice
    W = synth.weights(300, 700, config=0, layer=9)
    p1, g1 = gpu_lib.quantize_weights(dev(W))
    p2, g2 = gpu_lib.quantize_weights(dev(W))
    assert torch.equal(p1, p2) and torch.equal(g1, g2)


# ------------------------------------------------------------------------------------------------
# activations
# ------------------------------------------------------------------------------------------------
ACT_SHAPES = [(1, 1536), (16, 1536), (1, 1), (3, 515), (5, 28672), (70, 4096), (2, 40000), (3, 8192), (2, 13824), (3, 70000),
              (2, 131080)]


@pytest.mark.parametrize("M,K", ACT_SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_quantize_acts_matches_oracle(gpu_lib, M, K, dtype):
    say("quantize_acts %s M=%d K=%d" % (dtype, M, K))
    if dtype == "bf16":
        x, bits = synth.activations(M, K, config=0, layer=K % 11, bf16=True)
        xd = bf16_tensor(bits).view(M, K)
    else:
        x = synth.activations(M, K, config=0, layer=K % 11)
        xd = dev(x)
    xq_ref, sx_ref = oracle.quantize_acts(x)
    xq, sx = gpu_lib.quantize_acts(xd)
    assert np.array_equal(sx.cpu().numpy().view(np.uint32), sx_ref.view(np.uint32))
    assert np.array_equal(xq.cpu().numpy(), xq_ref)


def test_quantize_acts_edge_values(gpu_lib):
    say("quantize_acts edge values")
    g = json.load(open(os.path.join(GOLDEN, "rounding_ties.json")))["acts"]
    xq, sx = gpu_lib.quantize_acts(dev(np.array(g["x"], np.float32)))
    assert xq.cpu().numpy().tolist() == g["xq"] and sx.cpu().numpy().tolist() == g["sx"]
    # all-zero token, sub-floor token, one huge outlier, misaligned base pointer
    x = np.zeros((4, 64), np.float32)
    x[1, 3] = 5e-6
    x[2] = 0.001
    x[2, 5] = -1000.0
    x[3] = synth.activations(1, 64, config=0, layer=2)[0]
    xq_ref, sx_ref = oracle.quantize_acts(x)
    xq, sx = gpu_lib.quantize_acts(dev(x))
    assert np.array_equal(xq.cpu().numpy(), xq_ref) and np.array_equal(sx.cpu().numpy(), sx_ref)
    buf = torch.empty(4 * 64 + 1, dtype=torch.float32, device="cuda")
    buf[1:] = dev(x).reshape(-1)
    xq, sx = gpu_lib.quantize_acts(buf[1:].view(4, 64))
    assert np.array_equal(xq.cpu().numpy(), xq_ref) and np.array_equal(sx.cpu().numpy(), sx_ref)


# ------------------------------------------------------------------------------------------------
# the product
# ------------------------------------------------------------------------------------------------
def _run_linear_case(gpu_lib, M, N, K, kernels, layer=0, bf16_acts=False):
    W = synth.weights(N, K, config=0, layer=layer, tensor=0)
    if bf16_acts:
        x, bits = synth.activations(M, K, config=0, layer=layer, bf16=True)
        xd = bf16_tensor(bits).view(M, K)
    else:
        x = synth.activations(M, K, config=0, layer=layer)
        xd = dev(x)
    ref = oracle.bitlinear(x, W)
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    xq, sx = gpu_lib.quantize_acts(xd)
    assert np.array_equal(xq.cpu().numpy(), ref["xq"])
    for kern in kernels:
        acc = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.I32, kernel=kern)
        assert np.array_equal(acc.cpu().numpy(), ref["acc"]), "int32 accumulators differ (kernel %d)" % kern
        y32 = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.F32, kernel=kern)
        check_y(y32.cpu().numpy(), ref["y"], RTOL_F32)
        y16 = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.BF16, kernel=kern)
        check_y(y16.float().cpu().numpy(), ref["y"], RTOL_BF16)
    return ref


def test_worked_example_on_gpu(gpu_lib):
    say("worked example")
    g = json.load(open(os.path.join(GOLDEN, "worked_example.json")))
    W = np.array(g["W"], np.float32)
    x = np.array(g["x"], np.float32)
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    xq, sx = gpu_lib.quantize_acts(dev(x))
    assert gamma.cpu().numpy()[0] == g["gamma"]
    assert gpu_lib.unpack_weights(packed, 2, 4).cpu().numpy().tolist() == g["codes"]
    assert xq.cpu().numpy().tolist() == g["xq"] and sx.cpu().numpy().tolist() == g["sx"]
    acc = gpu_lib.linear(xq, sx, packed, gamma, 2, y_dtype=gpu_lib.I32)
    assert acc.cpu().numpy().tolist() == g["acc"]
    y = gpu_lib.linear(xq, sx, packed, gamma, 2)
    np.testing.assert_allclose(y.cpu().numpy(), np.array(g["y"]), rtol=RTOL_F32)


REF_SHAPES = [(1, 1, 1), (3, 5, 7), (2, 37, 129), (5, 100, 70), (16, 4096, 1536)]


@pytest.mark.parametrize("M,N,K", REF_SHAPES)
def test_linear_reference_kernel(gpu_lib, M, N, K):
    say("linear reference M=%d N=%d K=%d" % (M, N, K))
    _run_linear_case(gpu_lib, M, N, K, [gpu_lib.KERNEL_REFERENCE, gpu_lib.KERNEL_AUTO], layer=M)


# several tiles plus ragged tails in every dimension the GEMV kernel tiles: N (16-row blocks, groups
# of 1/2/4 blocks), K (quads of 64, steps of 256, split over 4 or 8 waves), M (tiles of 16)


@pytest.mark.parametrize("M,N,K", GEMV_SHAPES)
def test_linear_gemv_kernel(gpu_lib, M, N, K):
    say("linear gemv M=%d N=%d K=%d" % (M, N, K))
    _run_linear_case(gpu_lib, M, N, K, [gpu_lib.KERNEL_GEMV, gpu_lib.KERNEL_AUTO], layer=M, bf16_acts=(M % 2 == 0))




@pytest.mark.parametrize("M,N,K", FUSED_SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_linear_fused_matches_oracle(gpu_lib, M, N, K, dtype):
    """x -> y in one launch: the in-kernel activation quantization must reproduce x_q and s_x exactly,
    which shows in the int32 accumulators."""
    say("linear fused %s M=%d N=%d K=%d" % (dtype, M, N, K))
    W = synth.weights(N, K, config=0, layer=M + 20, tensor=0)
    if dtype == "bf16":
        x, bits = synth.activations(M, K, config=0, layer=M + 20, bf16=True)
        xd = bf16_tensor(bits).view(M, K)
    else:
        x = synth.activations(M, K, config=0, layer=M + 20)
        xd = dev(x)
    ref = oracle.bitlinear(x, W)
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    acc = gpu_lib.linear_fused(xd, packed, gamma, N, y_dtype=gpu_lib.I32)
    assert np.array_equal(acc.cpu().numpy(), ref["acc"])
    check_y(gpu_lib.linear_fused(xd, packed, gamma, N, y_dtype=gpu_lib.F32).cpu().numpy(), ref["y"], RTOL_F32)
    check_y(gpu_lib.linear_fused(xd, packed, gamma, N, y_dtype=gpu_lib.BF16).float().cpu().numpy(), ref["y"], RTOL_BF16)


# RMSNorm + quantization + product in one launch: each branch of the decode kernel's selection, token 0 in
# registers and the re-reading path (M > 1, long K), K tails, with and without gain


@pytest.mark.parametrize("M,N,K", NORM_FUSED_SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_rmsnorm_linear_fused_matches_oracle(gpu_lib, M, N, K, dtype):
    """x -> RMSNorm -> int8 -> product in one launch: x_q and s_x must be those of the oracle's RMSNorm
    quantizer (the int32 accumulators show it), and the result that of the two separate GPU calls, bit for bit."""
    say("rmsnorm linear fused %s M=%d N=%d K=%d" % (dtype, M, N, K))
    W = synth.weights(N, K, config=0, layer=M + 30, tensor=0)
    if dtype == "bf16":
        x, bits = synth.activations(M, K, config=2, layer=M + 30, tensor=5, bf16=True)
        xd = bf16_tensor(bits).view(M, K)
    else:
        x = synth.activations(M, K, config=0, layer=M + 30, tensor=5)
        xd = dev(x)
    rng = np.random.default_rng([11, K, M])
    g = (1.0 + 0.25 * rng.standard_normal(K)).astype(np.float32)
    gamma_ref, _ = oracle.absmean_gamma(W)
    codes_ref = oracle.ternarize(W, gamma_ref)
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    for gain, eps in ((g, 1e-5), (None, 1e-6)):
        xq_ref, sx_ref, _ = oracle.rmsnorm_quantize(x, gain, eps)
        acc_ref = oracle.ternary_matmul(xq_ref, codes_ref)
        y_ref = oracle.rescale(acc_ref, gamma_ref, sx_ref)
        gd = None if gain is None else dev(gain)
        acc = gpu_lib.rmsnorm_linear_fused(xd, gd, eps, packed, gamma, N, y_dtype=gpu_lib.I32)
        assert np.array_equal(acc.cpu().numpy(), acc_ref)
        y32 = gpu_lib.rmsnorm_linear_fused(xd, gd, eps, packed, gamma, N, y_dtype=gpu_lib.F32)
        check_y(y32.cpu().numpy(), y_ref, RTOL_F32)
        y16 = gpu_lib.rmsnorm_linear_fused(xd, gd, eps, packed, gamma, N, y_dtype=gpu_lib.BF16)
        check_y(y16.float().cpu().numpy(), y_ref, RTOL_BF16)
        xq, sx = gpu_lib.rmsnorm_quantize(xd, gd, eps)
        assert torch.equal(y32, gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.F32))


def test_rmsnorm_linear_fused_segmented_and_limits(gpu_lib):
    say("rmsnorm linear fused: segment scales, limits")
    M, K, seg_rows = 2, 528, [48, 16, 100]
    N = sum(seg_rows)
    W = synth.weights(N, K, config=0, layer=3, tensor=9)
    W[48:64] *= np.float32(2.5)
    x = synth.activations(M, K, config=0, layer=3, tensor=10)
    g = (1.0 + 0.1 * np.arange(K) / K).astype(np.float32)
    packed, gamma_rb = gpu_lib.quantize_weights_segmented(dev(W), seg_rows)
    xq, sx = gpu_lib.rmsnorm_quantize(dev(x), dev(g), 1e-6)
    want = gpu_lib.linear_segmented(xq, sx, packed, gamma_rb, N, y_dtype=gpu_lib.F32, kernel=gpu_lib.KERNEL_REFERENCE)
    got = gpu_lib.rmsnorm_linear_fused(dev(x), dev(g), 1e-6, packed, gamma_rb, N, y_dtype=gpu_lib.F32, segmented=True)
    assert torch.equal(got, want)
    # an all-zero token: r = 1 / sqrt(eps), z = 0, s_x = 1e-5, y = 0
    z = torch.zeros((1, K), dtype=torch.float32, device="cuda")
    p1, g1 = gpu_lib.quantize_weights(dev(W))
    assert bool((gpu_lib.rmsnorm_linear_fused(z, None, 1e-6, p1, g1, N) == 0).all())
    # limits: more than 16 tokens, a negative eps
    with pytest.raises(gpu_lib.BitnetError) as e:
        gpu_lib.rmsnorm_linear_fused(dev(synth.activations(17, K, config=0, layer=1)), None, 1e-6, p1, g1, N)
    assert e.value.status == 8
    with pytest.raises(gpu_lib.BitnetError) as e:
        gpu_lib.rmsnorm_linear_fused(dev(x), None, -1.0, p1, g1, N)
    assert e.value.status == 2


# SwiGLU + quantization + product in one launch: F (the product's K) from one partial step to the 3B / 7B / 70B
# feed-forward widths, token 0 in registers and the re-reading path, every branch of the kernel selection


@pytest.mark.parametrize("M,N,F", SWIGLU_FUSED_SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_swiglu_linear_fused_matches_oracle(gpu_lib, M, N, F, dtype):
    """[gate | up] -> SwiGLU -> int8 -> product in one launch: h_q and s_h must be those of the oracle's SwiGLU
    quantizer (the int32 accumulators show it), and the result that of the two separate GPU calls, bit for bit."""
    say("swiglu linear fused %s M=%d N=%d F=%d" % (dtype, M, N, F))
    W = synth.weights(N, F, config=0, layer=M + 40, tensor=0)
    if dtype == "bf16":
        gu, bits = synth.activations(M, 2 * F, config=2, layer=M + 40, tensor=6, bf16=True)
        gd = bf16_tensor(bits).view(M, 2 * F)
    else:
        gu = synth.activations(M, 2 * F, config=0, layer=M + 40, tensor=6)
        gd = dev(gu)
    gamma_ref, _ = oracle.absmean_gamma(W)
    codes_ref = oracle.ternarize(W, gamma_ref)
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    hq_ref, sh_ref, _ = oracle.swiglu_quantize(gu)
    acc_ref = oracle.ternary_matmul(hq_ref, codes_ref)
    y_ref = oracle.rescale(acc_ref, gamma_ref, sh_ref)
    acc = gpu_lib.swiglu_linear_fused(gd, packed, gamma, N, y_dtype=gpu_lib.I32)
    assert np.array_equal(acc.cpu().numpy(), acc_ref)
    y32 = gpu_lib.swiglu_linear_fused(gd, packed, gamma, N, y_dtype=gpu_lib.F32)
    check_y(y32.cpu().numpy(), y_ref, RTOL_F32)
    y16 = gpu_lib.swiglu_linear_fused(gd, packed, gamma, N, y_dtype=gpu_lib.BF16)
    check_y(y16.float().cpu().numpy(), y_ref, RTOL_BF16)
    hq, sh = gpu_lib.swiglu_quantize(gd)
    assert torch.equal(y32, gpu_lib.linear(hq, sh, packed, gamma, N, y_dtype=gpu_lib.F32))


def test_swiglu_linear_fused_limits(gpu_lib):
    say("swiglu linear fused: limits")
    F, N = 64, 32
    p, g = gpu_lib.quantize_weights(dev(synth.weights(N, F, config=0, layer=1)))
    z = torch.zeros((2, 2 * F), dtype=torch.float32, device="cuda")       # silu(0) * 0 = 0: s_h = 1e-5, y = 0
    assert bool((gpu_lib.swiglu_linear_fused(z, p, g, N) == 0).all())
    with pytest.raises(gpu_lib.BitnetError) as e:
        gpu_lib.swiglu_linear_fused(dev(synth.activations(17, 2 * F, config=0, layer=1)), p, g, N)
    assert e.value.status == 8


# merged gate | up projection with the gate applied in the epilogue: both workgroup shapes of its selection
# (F / 16 up to 700 and above), K tails, several tokens, with and without RMSNorm, one scale and one per segment
@pytest.mark.parametrize("M,F,K", FFN_GATE_UP_SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ffn_gate_up_fused(gpu_lib, M, F, K, dtype):
    """h = silu(y_gate) * y_up must be the oracle's gate applied to the fp32 outputs of the plain fused launch
    (bit for bit: same y, same fixed-step exponential), and the whole chain must match the oracle's chain."""
    say("ffn gate/up fused %s M=%d F=%d K=%d" % (dtype, M, F, K))
    W = synth.weights(2 * F, K, config=0, layer=M + 50, tensor=0)
    W[F:] *= np.float32(1.5)                       # the halves differ in magnitude: one gamma per half matters
    if dtype == "bf16":
        x, bits = synth.activations(M, K, config=2, layer=M + 50, tensor=7, bf16=True)
        xd = bf16_tensor(bits).view(M, K)
    else:
        x = synth.activations(M, K, config=0, layer=M + 50, tensor=7)
        xd = dev(x)
    rng = np.random.default_rng([13, K, M])
    g = (1.0 + 0.25 * rng.standard_normal(K)).astype(np.float32)
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    packed_s, gamma_rb = gpu_lib.quantize_weights_segmented(dev(W), [F, F])
    # (a) against the plain fused launches + the oracle's gate on their fp32 output
    for norm in (False, True):
        y32 = (gpu_lib.rmsnorm_linear_fused(xd, dev(g), 1e-5, packed, gamma, 2 * F) if norm
               else gpu_lib.linear_fused(xd, packed, gamma, 2 * F)).cpu().numpy()
        h_ref = oracle.swiglu_quantize(y32)[2]
        h32 = gpu_lib.ffn_gate_up_fused(xd, packed, gamma, F, norm=norm, g=dev(g) if norm else None, eps=1e-5)
        assert h32.cpu().numpy().tobytes() == h_ref.tobytes()
        h16 = gpu_lib.ffn_gate_up_fused(xd, packed, gamma, F, norm=norm, g=dev(g) if norm else None, eps=1e-5,
                                        h_dtype=gpu_lib.BF16)
        check_y(h16.float().cpu().numpy(), h_ref, RTOL_BF16)
    y32 = gpu_lib.rmsnorm_linear_fused(xd, None, 1e-6, packed_s, gamma_rb, 2 * F, segmented=True).cpu().numpy()
    h32 = gpu_lib.ffn_gate_up_fused(xd, packed_s, gamma_rb, F, norm=True, g=None, eps=1e-6, gamma_per_block=True)
    assert h32.cpu().numpy().tobytes() == oracle.swiglu_quantize(y32)[2].tobytes()
    # (b) against the oracle end to end: RMSNorm -> int8 -> product -> rescale -> gate
    xq_ref, sx_ref, _ = oracle.rmsnorm_quantize(x, g, 1e-5)
    gamma_ref, _ = oracle.absmean_gamma(W)
    y_ref = oracle.rescale(oracle.ternary_matmul(xq_ref, oracle.ternarize(W, gamma_ref)), gamma_ref, sx_ref)
    h_oracle = oracle.swiglu_quantize(y_ref)[2]
    h32 = gpu_lib.ffn_gate_up_fused(xd, packed, gamma, F, norm=True, g=dev(g), eps=1e-5).cpu().numpy()
    np.testing.assert_allclose(h32, h_oracle, rtol=5e-5, atol=1e-30)


def test_ffn_gate_up_fused_limits(gpu_lib):
    say("ffn gate/up fused: limits")
    K = 64
    p, g = gpu_lib.quantize_weights(dev(synth.weights(64, K, config=0, layer=1)))
    x = dev(synth.activations(1, K, config=0, layer=1))
    with pytest.raises(gpu_lib.BitnetError) as e:            # F must be a multiple of 16
        gpu_lib.ffn_gate_up_fused(x, p, g, 24)
    assert e.value.status == 2
    with pytest.raises(gpu_lib.BitnetError) as e:            # int32 output makes no sense after the gate
        gpu_lib.ffn_gate_up_fused(x, p, g, 32, h_dtype=gpu_lib.I32, h=torch.empty((1, 32), dtype=torch.int32, device="cuda"))
    assert e.value.status == 3
    with pytest.raises(gpu_lib.BitnetError) as e:
        gpu_lib.ffn_gate_up_fused(dev(synth.activations(17, K, config=0, layer=1)), p, g, 32)
    assert e.value.status == 8


def test_linear_fused_rejects_what_it_cannot_run(gpu_lib):
    say("linear fused limits")
    W = dev(synth.weights(32, 8192, config=0, layer=1))
    packed, gamma = gpu_lib.quantize_weights(W)
    x = dev(synth.activations(16, 8192, config=0, layer=1))          # 16 x 8192 int8 does not fit the LDS budget
    with pytest.raises(gpu_lib.BitnetError) as e:
        gpu_lib.linear_fused(x, packed, gamma, 32)
    assert e.value.status == 8
    x17 = dev(synth.activations(17, 64, config=0, layer=1))
    p2, g2 = gpu_lib.quantize_weights(dev(synth.weights(32, 64, config=0, layer=1)))
    with pytest.raises(gpu_lib.BitnetError) as e:
        gpu_lib.linear_fused(x17, p2, g2, 32)
    assert e.value.status == 8


# ragged edges in M, N and K (K steps of 256 with a partial last step), token counts below one tile, and several
# tiles in each direction.  The workgroup tile (64, 96 or 128 tokens x 128 or 256 weight rows) follows a cost model
# of tile count and shape; the last three shapes fill the chip, the others leave most of it idle and get the small
# tiles (each tile shape is also forced on its own in test_linear_gemm_every_tile_shape).


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_linear_gemm_kernel(gpu_lib, M, N, K):
    say("linear gemm M=%d N=%d K=%d" % (M, N, K))
    _run_linear_case(gpu_lib, M, N, K, [gpu_lib.KERNEL_GEMM, gpu_lib.KERNEL_AUTO], layer=M % 13, bf16_acts=(M % 2 == 0))


# every workgroup tile of the prefill kernel (tokens x weight rows), each on shapes with several tiles and ragged
# tails in M, N and K, one of them smaller than a single tile
# (a third entry 2: the eight-wave form with two K groups -- the shapes give its groups 3 + 2, 2 + 1, 1 + 0 and 1 + 1
# K steps, the last one partial; 512 rows: the eight-wave form with two row groups -- the shapes give its second group
# whole, ragged and empty row ranges)
@pytest.mark.parametrize("tile", [(128, 256), (96, 256), (64, 256), (128, 128), (96, 128), (64, 128), (96, 128, 2), (64, 256, 2), (128, 512)])
def test_linear_gemm_every_tile_shape(gpu_lib, tile):
    kern = (gpu_lib.KERNEL_GEMM_TILES_K2[tile[:2]] if len(tile) == 3 else gpu_lib.KERNEL_GEMM_TILES_WIDE[tile] if tile[1] == 512
            else gpu_lib.KERNEL_GEMM_TILES[tile])
    for (M, N, K) in [(300, 520, 1040), (257, 1000, 528), (100, 40, 16), (129, 130, 272), (65, 2100, 80)]:
        say("linear gemm tile %s M=%d N=%d K=%d" % ("x".join(map(str, tile)), M, N, K))
        _run_linear_case(gpu_lib, M, N, K, [kern], layer=(M + tile[0] + tile[1]) % 11, bf16_acts=(M % 2 == 1))


# split-K through a workspace: every split count on ragged shapes (K steps not divisible by the splits, a partial last
# step, fewer steps than splits rejected), per-block scales, and the automatic choice on a shape where it pays
@pytest.mark.parametrize("M,N,K", [(100, 300, 2064), (129, 520, 4112), (65, 40, 528), (300, 1000, 1040)])
def test_linear_splitk_matches_reference(gpu_lib, M, N, K):
    say("split-K M=%d N=%d K=%d" % (M, N, K))
    W = synth.weights(N, K, config=0, layer=M % 7, tensor=15)
    x = synth.activations(M, K, config=0, layer=M % 7, tensor=16)
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    xq, sx = gpu_lib.quantize_acts(dev(x))
    ws = torch.full((8 * M * N * 4 + 64,), 0xCD, dtype=torch.uint8, device="cuda")
    for dt in (gpu_lib.I32, gpu_lib.F32, gpu_lib.BF16):
        ref = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=dt, kernel=gpu_lib.KERNEL_REFERENCE)
        for splits, code in gpu_lib.KERNEL_GEMM_SPLITK.items():
            if splits > (K + 255) // 256:
                with pytest.raises(gpu_lib.BitnetError) as e:
                    gpu_lib.linear_ws(xq, sx, packed, gamma, N, ws[: 8 * M * N * 4], y_dtype=dt, kernel=code)
                assert e.value.status == 6
                continue
            got = gpu_lib.linear_ws(xq, sx, packed, gamma, N, ws[: 8 * M * N * 4], y_dtype=dt, kernel=code)
            assert torch.equal(got, ref)
        assert torch.equal(gpu_lib.linear_ws(xq, sx, packed, gamma, N, ws[: 8 * M * N * 4], y_dtype=dt), ref)
        assert torch.equal(gpu_lib.linear_ws(xq, sx, packed, gamma, N, None, y_dtype=dt), ref)
    assert bool((ws[8 * M * N * 4:] == 0xCD).all())                     # nothing written past the stated size
    with pytest.raises(gpu_lib.BitnetError) as e:                       # too small for the forced split
        gpu_lib.linear_ws(xq, sx, packed, gamma, N, ws[: 2 * M * N * 4 - 16], kernel=gpu_lib.KERNEL_GEMM_SPLITK[2])
    assert e.value.status == 6
    # the oracle on the integer result once
    ref = oracle.bitlinear(x, W)
    acc = gpu_lib.linear_ws(xq, sx, packed, gamma, N, ws[: 8 * M * N * 4], y_dtype=gpu_lib.I32, kernel=gpu_lib.KERNEL_GEMM_SPLITK[2])
    assert np.array_equal(acc.cpu().numpy(), ref["acc"])


# split-K of the batched-decode kernels (5 ... 64 tokens): every split count, both kernel forms (with and without the
# loader wave: N from 8192 / 20480 rows on), ragged K steps, per-block scales; bit-identical to the one-launch result
@pytest.mark.parametrize("M,N,K", [(5, 300, 2064), (16, 1000, 1296), (17, 8200, 1040), (33, 520, 4112), (48, 20500, 784),
                                   (64, 8208, 2320), (64, 40, 528), (40, 32784, 528)])
def test_linear_splitk_batched_decode(gpu_lib, M, N, K):
    say("split-K, batched decode M=%d N=%d K=%d" % (M, N, K))
    W = synth.weights(N, K, config=0, layer=M % 5, tensor=17)
    W[N // 32 * 16:] *= np.float32(0.25)
    x = synth.activations(M, K, config=0, layer=M % 5, tensor=18)
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    packed_rb, gamma_rb = gpu_lib.quantize_weights_segmented(dev(W), [N // 32 * 16, N - N // 32 * 16])
    xq, sx = gpu_lib.quantize_acts(dev(x))
    ws = torch.full((8 * M * N * 4 + 64,), 0xCD, dtype=torch.uint8, device="cuda")
    for dt in (gpu_lib.I32, gpu_lib.F32, gpu_lib.BF16):
        ref = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=dt)
        ref_rb = gpu_lib.linear_segmented(xq, sx, packed_rb, gamma_rb, N, y_dtype=dt)
        for splits, code in gpu_lib.KERNEL_GEMM_SPLITK.items():
            if splits > (K + 255) // 256:
                continue
            assert torch.equal(gpu_lib.linear_ws(xq, sx, packed, gamma, N, ws[: 8 * M * N * 4], y_dtype=dt, kernel=code), ref)
            assert torch.equal(gpu_lib.linear_ws(xq, sx, packed_rb, gamma_rb, N, ws[: 8 * M * N * 4], y_dtype=dt, kernel=code,
                                                 gamma_per_block=True), ref_rb)
    assert bool((ws[8 * M * N * 4:] == 0xCD).all())
    acc = gpu_lib.linear_ws(xq, sx, packed, gamma, N, ws[: 8 * M * N * 4], y_dtype=gpu_lib.I32, kernel=gpu_lib.KERNEL_GEMM_SPLITK[2])
    assert np.array_equal(acc.cpu().numpy(), oracle.bitlinear(x, W)["acc"])


def test_linear_splitk_auto_and_segment_scales(gpu_lib):
    say("split-K: automatic choice, per-block scales, workspace query")
    M, N, K = 520, 2048, 11008                           # 96 tiles of 96 x 128 and 43 K steps: the model splits
    assert gpu_lib.linear_workspace(M, N, K) == 8 * M * N * 4
    assert gpu_lib.linear_workspace(64, N, K) == 0 and gpu_lib.linear_workspace(2048, 27648, 5120) == 0
    W = synth.weights(N, K, config=2, layer=1, tensor=3)
    W[N // 2:] *= np.float32(0.5)
    x, bits = synth.activations(M, K, config=2, layer=1, tensor=103, bf16=True)
    packed, gamma_rb = gpu_lib.quantize_weights_segmented(dev(W), [N // 2, N // 2])
    xq, sx = gpu_lib.quantize_acts(bf16_tensor(bits).view(M, K))
    ws = torch.empty(gpu_lib.linear_workspace(M, N, K), dtype=torch.uint8, device="cuda")
    ref = gpu_lib.linear_segmented(xq, sx, packed, gamma_rb, N, y_dtype=gpu_lib.BF16)
    got = gpu_lib.linear_ws(xq, sx, packed, gamma_rb, N, ws, y_dtype=gpu_lib.BF16, gamma_per_block=True)
    assert torch.equal(got, ref)
    accr = gpu_lib.linear_segmented(xq, sx, packed, gamma_rb, N, y_dtype=gpu_lib.I32, kernel=gpu_lib.KERNEL_REFERENCE)
    assert torch.equal(gpu_lib.linear_ws(xq, sx, packed, gamma_rb, N, ws, y_dtype=gpu_lib.I32, gamma_per_block=True), accr)
    # decode shapes ignore the workspace
    xq1, sx1 = xq[:8].contiguous(), sx[:8].contiguous()
    assert torch.equal(gpu_lib.linear_ws(xq1, sx1, packed, gamma_rb, N, ws, gamma_per_block=True),
                       gpu_lib.linear_segmented(xq1, sx1, packed, gamma_rb, N))


def test_linear_gemm_small_m_and_forced_on_decode_shapes(gpu_lib):
    say("linear gemm forced at small M")
    _run_linear_case(gpu_lib, 1, 100, 80, [gpu_lib.KERNEL_GEMM], layer=2)
    _run_linear_case(gpu_lib, 16, 4096, 1536, [gpu_lib.KERNEL_GEMM], layer=3)


@pytest.mark.parametrize("M,N,K,layer", FULL_SIZE_GEMM)
def test_linear_gemm_full_size_sampled(gpu_lib, M, N, K, layer):
    """13B-class prefill shapes at full size, in the launch configuration the benchmark times; the oracle
    recomputes a seeded sample of 256 tokens x 2048 weight rows (codes, x_q, accumulators bit-exact), and the whole
    integer result is compared with the one-thread-per-output reference kernel."""
    say("linear gemm full size M=%d N=%d K=%d" % (M, N, K))
    W = synth.weights(N, K, config=3, layer=0, tensor=layer)
    x, bits = synth.activations(M, K, config=3, layer=0, tensor=100 + layer, bf16=True)
    gamma_ref, _ = oracle.absmean_gamma(W)
    rng = np.random.default_rng([layer, M])
    rows = np.sort(rng.choice(M, 256, replace=False))
    rows[0], rows[-1] = 0, M - 1
    cols = np.sort(rng.choice(N, 2048, replace=False))
    cols[0], cols[-1] = 0, N - 1
    codes_ref = oracle.ternarize(W[cols], gamma_ref)
    xq_ref, sx_ref = oracle.quantize_acts(x[rows])
    acc_ref = oracle.ternary_matmul(xq_ref, codes_ref)
    y_ref = oracle.rescale(acc_ref, gamma_ref, sx_ref)
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    del W
    xq, sx = gpu_lib.quantize_acts(bf16_tensor(bits).view(M, K))
    assert gamma.cpu().numpy()[0] == gamma_ref
    assert np.array_equal(xq.cpu().numpy()[rows], xq_ref)
    ri = torch.from_numpy(rows).cuda()
    ci = torch.from_numpy(cols).cuda()
    acc = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.I32)
    assert gpu_lib.linear_describe(M, N, K)["kernel"] == "prefill"
    assert np.array_equal(acc[ri][:, ci].cpu().numpy(), acc_ref)
    # any-size property: the whole integer result equals the reference kernel's
    a_ref = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.I32, kernel=gpu_lib.KERNEL_REFERENCE)
    assert torch.equal(a_ref, acc)
    del acc, a_ref
    y16 = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.BF16)
    check_y(y16[ri][:, ci].float().cpu().numpy(), y_ref, RTOL_BF16)
    del y16
    y32 = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.F32)
    check_y(y32[ri][:, ci].cpu().numpy(), y_ref, RTOL_F32)


# the remaining benchmark configurations at full size, every token count the benchmark times


@pytest.mark.parametrize("config,name,K,N,Ms", FULL_SIZE_DECODE)
def test_linear_decode_full_size_sampled(gpu_lib, config, name, K, N, Ms):
    """7B-class batched decode and 70B-class decode shapes at full size through bitnet_linear (and the fused entry
    point at M = 1), as the benchmark launches them; the oracle recomputes a seeded sample of 512 weight rows for
    every token (gamma over the whole matrix, codes, x_q, accumulators bit-exact)."""
    say("linear decode full size config %d %s K=%d N=%d" % (config, name, K, N))
    W = synth.weights(N, K, config=config, layer=0, tensor=len(name))
    gamma_ref, _ = oracle.absmean_gamma(W)
    rng = np.random.default_rng([config, K, N])
    cols = np.sort(rng.choice(N, 512, replace=False))
    cols[0], cols[-1] = 0, N - 1
    codes_ref = oracle.ternarize(W[cols], gamma_ref)
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    W_rows = lambda idx: W[idx]
    assert gamma.cpu().numpy()[0] == gamma_ref
    ci = torch.from_numpy(cols).cuda()
    for M in Ms:
        x, bits = synth.activations(M, K, config=config, layer=M, tensor=100, bf16=True)
        xq_ref, sx_ref = oracle.quantize_acts(x)
        acc_ref = oracle.ternary_matmul(xq_ref, codes_ref)
        y_ref = oracle.rescale(acc_ref, gamma_ref, sx_ref)
        xd = bf16_tensor(bits).view(M, K)
        xq, sx = gpu_lib.quantize_acts(xd)
        assert np.array_equal(xq.cpu().numpy(), xq_ref) and sx.cpu().numpy().tobytes() == sx_ref.tobytes()
        acc = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.I32)
        assert np.array_equal(acc[:, ci].cpu().numpy(), acc_ref)
        y16 = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.BF16)
        check_y(y16[:, ci].float().cpu().numpy(), y_ref, RTOL_BF16)
        if M == 1:
            accf = gpu_lib.linear_fused(xd, packed, gamma, N, y_dtype=gpu_lib.I32)
            assert np.array_equal(accf[:, ci].cpu().numpy(), acc_ref)
        if M == 1 and name == "gate_up":
            # the same matrix as a merged gate | up projection with the gate in the epilogue (RMSNorm in front), as the
            # feed-forward chain of the benchmark launches it: 256 sampled (gate, up) row pairs
            F = N // 2
            pj = np.sort(rng.choice(F, 256, replace=False))
            pj[0], pj[-1] = 0, F - 1
            gain = (1.0 + 0.1 * rng.standard_normal(K)).astype(np.float32)
            xq_n, sx_n, _ = oracle.rmsnorm_quantize(x, gain, 1e-6)
            c2 = oracle.ternarize(W_rows(np.concatenate([pj, pj + F])), gamma_ref)
            y2 = oracle.rescale(oracle.ternary_matmul(xq_n, c2), gamma_ref, sx_n)
            _, _, h_def = _swiglu_definition(y2)
            h16 = gpu_lib.ffn_gate_up_fused(xd, packed, gamma, F, norm=True, g=dev(gain), eps=1e-6, h_dtype=gpu_lib.BF16)
            check_y(h16[:, torch.from_numpy(pj).cuda()].float().cpu().numpy(), h_def, RTOL_BF16)
        # any-size property: the whole integer result equals the reference kernel's
        a_ref = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.I32, kernel=gpu_lib.KERNEL_REFERENCE)
        assert torch.equal(a_ref, acc)


# 13B- and 30B-class projections: between them and the benchmark's 3B / 7B / 70B shapes they reach every launch shape
# the M <= 4 decode dispatch can pick (K = 5120 is the case whose 20 K steps pad badly over four waves)


@pytest.mark.parametrize("name,K,N", FAMILY_DECODE)
def test_linear_decode_family_shapes_sampled(gpu_lib, name, K, N):
    say("linear decode %s K=%d N=%d" % (name, K, N))
    W = synth.weights(N, K, config=3, layer=1, tensor=len(name))
    gamma_ref, _ = oracle.absmean_gamma(W)
    rng = np.random.default_rng([3, K, N])
    cols = np.sort(rng.choice(N, 256, replace=False))
    cols[0], cols[-1] = 0, N - 1
    codes_ref = oracle.ternarize(W[cols], gamma_ref)
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    del W
    assert gamma.cpu().numpy()[0] == gamma_ref
    ci = torch.from_numpy(cols).cuda()
    for M in (1, 3):
        x, bits = synth.activations(M, K, config=3, layer=M, tensor=100, bf16=True)
        xq_ref, sx_ref = oracle.quantize_acts(x)
        acc_ref = oracle.ternary_matmul(xq_ref, codes_ref)
        y_ref = oracle.rescale(acc_ref, gamma_ref, sx_ref)
        xd = bf16_tensor(bits).view(M, K)
        xq, sx = gpu_lib.quantize_acts(xd)
        acc = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.I32)
        assert np.array_equal(acc[:, ci].cpu().numpy(), acc_ref)
        y16 = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.BF16)
        check_y(y16[:, ci].float().cpu().numpy(), y_ref, RTOL_BF16)
        a_ref = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.I32, kernel=gpu_lib.KERNEL_REFERENCE)
        assert torch.equal(a_ref, acc)
        if 128 + M * ((K + 255) // 256) * 256 <= 60 * 1024:            # the fused entry point holds x_q in LDS
            assert torch.equal(gpu_lib.linear_fused(xd, packed, gamma, N, y_dtype=gpu_lib.I32), a_ref)


def test_linear_prefill_70b_full_size_sampled(gpu_lib):
    """70B-class FFN shapes at M = 4096 (the prefill sweep of the last benchmark configuration): the oracle recomputes
    a seeded sample of 128 tokens x 1024 weight rows, and the integer result of 256 more tokens (four runs of 64, from
    both ends and the middle) is compared in full with the batched-decode kernels' result for the same tokens."""
    for (name, K, N) in (("gate_up", 8192, 57344), ("down", 28672, 8192)):
        say("linear prefill full size 70B %s" % name)
        M = 4096
        W = synth.weights(N, K, config=4, layer=1, tensor=len(name))
        gamma_ref, _ = oracle.absmean_gamma(W)
        rng = np.random.default_rng([4, K, N])
        rows = np.sort(rng.choice(M, 128, replace=False))
        rows[0], rows[-1] = 0, M - 1
        cols = np.sort(rng.choice(N, 1024, replace=False))
        cols[0], cols[-1] = 0, N - 1
        codes_ref = oracle.ternarize(W[cols], gamma_ref)
        packed, gamma = gpu_lib.quantize_weights(dev(W))
        del W
        assert gamma.cpu().numpy()[0] == gamma_ref
        x, bits = synth.activations(M, K, config=4, layer=1, tensor=100, bf16=True)
        xq_ref, sx_ref = oracle.quantize_acts(x[rows])
        acc_ref = oracle.ternary_matmul(xq_ref, codes_ref)
        y_ref = oracle.rescale(acc_ref, gamma_ref, sx_ref)
        xq, sx = gpu_lib.quantize_acts(bf16_tensor(bits).view(M, K))
        del x, bits
        ri = torch.from_numpy(rows).cuda()
        ci = torch.from_numpy(cols).cuda()
        assert np.array_equal(xq[ri].cpu().numpy(), xq_ref)
        acc = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.I32)
        assert gpu_lib.linear_describe(M, N, K)["kernel"] == "prefill"
        assert np.array_equal(acc[ri][:, ci].cpu().numpy(), acc_ref)
        for m0 in (0, 1000, 2048, M - 64):
            sub = slice(m0, m0 + 64)
            a_dec = gpu_lib.linear(xq[sub].contiguous(), sx[sub].contiguous(), packed, gamma, N, y_dtype=gpu_lib.I32,
                                   kernel=gpu_lib.KERNEL_GEMV)
            assert torch.equal(a_dec, acc[sub]), (name, m0)
        del acc
        y16 = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.BF16)
        check_y(y16[ri][:, ci].float().cpu().numpy(), y_ref, RTOL_BF16)
        del y16, packed, xq
        torch.cuda.empty_cache()


def test_random_shapes_every_kernel_agrees(gpu_lib):
    """48 seeded shapes drawn across the kernel-selection boundaries (tokens 1..300, rows 1..6000, K a multiple
    of 16 up to 4096): every product kernel that accepts the shape returns the reference kernel's int32
    accumulators bit for bit, and every eighth shape is also recomputed by the oracle."""
    rng = np.random.default_rng(2402)
    for case in range(48):
        M = int(rng.choice([1, 2, 4, 5, 8, 16, 17, 31, 32, 33, 63, 64, 65, 96, 97, 128, 200, 300]))
        N = int(rng.integers(1, 6001))
        K = 16 * int(rng.integers(1, 257))
        say("random shape %d: M=%d N=%d K=%d" % (case, M, N, K))
        W = synth.weights(N, K, config=0, layer=case, tensor=13)
        x = synth.activations(M, K, config=0, layer=case, tensor=14)
        packed, gamma = gpu_lib.quantize_weights(dev(W))
        xq, sx = gpu_lib.quantize_acts(dev(x))
        ref_acc = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.I32, kernel=gpu_lib.KERNEL_REFERENCE)
        kernels = [gpu_lib.KERNEL_AUTO, gpu_lib.KERNEL_GEMM] + ([gpu_lib.KERNEL_GEMV] if M <= 64 else [])
        for kern in kernels:
            acc = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.I32, kernel=kern)
            assert torch.equal(acc, ref_acc), (M, N, K, kern)
        if M <= 16:
            yf = gpu_lib.linear_fused(dev(x), packed, gamma, N, y_dtype=gpu_lib.I32)
            assert torch.equal(yf, ref_acc), (M, N, K, "fused")
        if case % 8 == 0:
            o = oracle.bitlinear(x, W)
            assert np.array_equal(ref_acc.cpu().numpy(), o["acc"])
            y32 = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.F32)
            check_y(y32.cpu().numpy(), o["y"], RTOL_F32)


def test_random_shapes_block_entry_points_match_oracle(gpu_lib):
    """40 seeded shapes (1 ... 16 tokens, 16 ... 4000 rows, K a multiple of 16 within the fused launches' LDS budget, both
    input types) through the entry points that do a block's work in one launch -- RMSNorm in front, SwiGLU in front,
    merged gate / up with the gate behind -- each against the oracle's own chain: accumulators bit for bit, the gate's
    output bit for bit on the oracle's gate of the library's fp32 y and within the bf16 bar end to end."""
    rng = np.random.default_rng(1764)
    for case in range(40):
        M = int(rng.choice([1, 1, 2, 3, 4, 7, 8, 12, 16]))
        F = 16 * int(rng.integers(1, 126))                               # gate / up width; the product has 2 F rows
        N = int(rng.integers(1, 4001))
        K = 16 * int(rng.integers(1, min(257, 60000 // (16 * M))))
        bf16 = case % 2 == 1
        say("random block case %d: M=%d N=%d F=%d K=%d %s" % (case, M, N, F, K, "bf16" if bf16 else "f32"))
        g = (1.0 + 0.25 * rng.standard_normal(K)).astype(np.float32)
        eps = float(rng.choice([0.0, 1e-6, 1e-5]))
        if bf16:
            x, bits = synth.activations(M, K, config=2, layer=case, tensor=51, bf16=True)
            xd = bf16_tensor(bits).view(M, K)
        else:
            x = synth.activations(M, K, config=0, layer=case, tensor=51)
            xd = dev(x)
        # RMSNorm -> int8 -> product
        W = synth.weights(N, K, config=0, layer=case, tensor=52)
        codes, gamma_ref = oracle.quantize_weights(W)
        packed, gamma = gpu_lib.quantize_weights(dev(W))
        xq_ref, sx_ref, _ = oracle.rmsnorm_quantize(x, g, eps)
        acc_ref = oracle.ternary_matmul(xq_ref, codes)
        acc = gpu_lib.rmsnorm_linear_fused(xd, dev(g), eps, packed, gamma, N, y_dtype=gpu_lib.I32)
        assert np.array_equal(acc.cpu().numpy(), acc_ref), ("rmsnorm_linear_fused", M, N, K)
        y16 = gpu_lib.rmsnorm_linear_fused(xd, dev(g), eps, packed, gamma, N, y_dtype=gpu_lib.BF16)
        check_y(y16.float().cpu().numpy(), oracle.rescale(acc_ref, gamma_ref, sx_ref), RTOL_BF16)
        # merged gate / up with RMSNorm in front and the gate behind
        Wgu = synth.weights(2 * F, K, config=0, layer=case, tensor=53)
        codes_gu, gamma_gu = oracle.quantize_weights(Wgu)
        packed_gu, gamma_gu_d = gpu_lib.quantize_weights(dev(Wgu))
        y_gu = oracle.rescale(oracle.ternary_matmul(xq_ref, codes_gu), gamma_gu, sx_ref)
        h_chain = oracle.swiglu_quantize(y_gu.astype(np.float32))[2]
        y32 = gpu_lib.rmsnorm_linear_fused(xd, dev(g), eps, packed_gu, gamma_gu_d, 2 * F).cpu().numpy()
        check_y(y32, y_gu, RTOL_F32)
        h32 = gpu_lib.ffn_gate_up_fused(xd, packed_gu, gamma_gu_d, F, norm=True, g=dev(g), eps=eps)
        assert h32.cpu().numpy().tobytes() == oracle.swiglu_quantize(y32)[2].tobytes(), ("ffn_gate_up_fused", M, F, K)
        nz = np.abs(h_chain) > 1e-6                                      # tiny gated values carry y's 1e-5 into a ratio of near-zeros
        check_y(h32.cpu().numpy()[nz], h_chain.astype(np.float64)[nz], 1e-3)
        # SwiGLU -> int8 -> product (the gated row has F columns: a down projection of N rows)
        if 2 * F * M * (2 if bf16 else 4) <= 10 ** 9 and F <= 60000 // M:
            Wd = synth.weights(N, F, config=0, layer=case, tensor=54)
            codes_d, gamma_d = oracle.quantize_weights(Wd)
            packed_d, gamma_dd = gpu_lib.quantize_weights(dev(Wd))
            if bf16:
                gu, gbits = synth.activations(M, 2 * F, config=2, layer=case, tensor=55, bf16=True)
                gud = bf16_tensor(gbits).view(M, 2 * F)
            else:
                gu = synth.activations(M, 2 * F, config=0, layer=case, tensor=55)
                gud = dev(gu)
            hq_ref, sh_ref, _ = oracle.swiglu_quantize(gu)
            acc_d = oracle.ternary_matmul(hq_ref, codes_d)
            got = gpu_lib.swiglu_linear_fused(gud, packed_d, gamma_dd, N, y_dtype=gpu_lib.I32)
            assert np.array_equal(got.cpu().numpy(), acc_d), ("swiglu_linear_fused", M, N, F)
            y16 = gpu_lib.swiglu_linear_fused(gud, packed_d, gamma_dd, N, y_dtype=gpu_lib.BF16)
            check_y(y16.float().cpu().numpy(), oracle.rescale(acc_d, gamma_d, sh_ref), RTOL_BF16)


# ------------------------------------------------------------------------------------------------
# producers of int8 activations: RMSNorm -> int8, SwiGLU -> int8 (bit-exact codes and scales)
# ------------------------------------------------------------------------------------------------
# register-resident forms (1, 2, 4, 8 loads of 16 bytes per thread at 256 and at 1024 threads, 16 for fp32 at 1024:
# every instantiation of either input type is reached) and the sweeping form (K not a multiple of the load, K >
# 65536), one token and many, with and without gain
PRODUCER_SHAPES = [(1, 3200), (16, 1536), (5, 4), (3, 1), (7, 1003), (2, 16384), (2, 16388), (1, 28672), (33, 8640),
                   (300, 520), (70, 4096), (65, 6656), (64, 13824), (70, 20000), (3, 40000), (2, 70000), (80, 2048),
                   (4, 8192)]


@pytest.mark.parametrize("M,K", PRODUCER_SHAPES)
@pytest.mark.parametrize("bf16", [False, True])
def test_rmsnorm_quantize_matches_oracle(gpu_lib, M, K, bf16):
    say("rmsnorm_quantize M=%d K=%d bf16=%s" % (M, K, bf16))
    x, bits = synth.activations(M, K, config=2, layer=K % 7, tensor=3, bf16=True)
    if not bf16:
        x = synth.activations(M, K, config=0, layer=K % 7, tensor=3)
    rng = np.random.default_rng([7, K])
    g = (1.0 + 0.25 * rng.standard_normal(K)).astype(np.float32)
    xt = bf16_tensor(bits).view(M, K) if bf16 else dev(x)
    for gain, eps in ((None, 1e-6), (g, 1e-5), (g, 0.0)):
        xq_ref, sx_ref, _ = oracle.rmsnorm_quantize(x, gain, eps)
        xq, sx = gpu_lib.rmsnorm_quantize(xt, None if gain is None else dev(gain), eps)
        assert sx.cpu().numpy().tobytes() == sx_ref.tobytes()
        assert np.array_equal(xq.cpu().numpy(), xq_ref)


def test_rmsnorm_quantize_edge_cases(gpu_lib):
    say("rmsnorm_quantize edge cases")
    x = np.zeros((3, 64), np.float32)
    x[1, 5] = 1e-20          # vanishes under eps
    x[2, :] = -3.0
    for eps in (1e-6, 0.25):
        xq_ref, sx_ref, _ = oracle.rmsnorm_quantize(x, None, eps)
        xq, sx = gpu_lib.rmsnorm_quantize(dev(x), None, eps)
        assert sx.cpu().numpy().tobytes() == sx_ref.tobytes()
        assert np.array_equal(xq.cpu().numpy(), xq_ref)
    # an unaligned view (odd element offset) takes the re-reading path and gives the same codes
    M, K = 4, 1000
    xa = synth.activations(M, K + 1, config=0, layer=1, tensor=4)
    flat = dev(xa.reshape(-1))
    view = flat[1:1 + M * K].view(M, K)
    xq_ref, sx_ref, _ = oracle.rmsnorm_quantize(view.cpu().numpy(), None, 1e-6)
    xq, sx = gpu_lib.rmsnorm_quantize(view, None, 1e-6)
    assert np.array_equal(xq.cpu().numpy(), xq_ref) and sx.cpu().numpy().tobytes() == sx_ref.tobytes()


@pytest.mark.parametrize("M,F", [(1, 8640), (16, 1536), (5, 4), (3, 1), (7, 1003), (2, 16384), (2, 16390), (1, 28672),
                                 (40, 11008), (300, 260), (70, 4096), (65, 8640), (64, 13824), (70, 28672), (3, 40000),
                                 (2, 70000)])
@pytest.mark.parametrize("bf16", [False, True])
def test_swiglu_quantize_matches_oracle(gpu_lib, M, F, bf16):
    say("swiglu_quantize M=%d F=%d bf16=%s" % (M, F, bf16))
    gu, bits = synth.activations(M, 2 * F, config=2, layer=F % 5, tensor=5, bf16=True)
    if not bf16:
        gu = synth.activations(M, 2 * F, config=0, layer=F % 5, tensor=5)
    gt = bf16_tensor(bits).view(M, 2 * F) if bf16 else dev(gu)
    hq_ref, sh_ref, _ = oracle.swiglu_quantize(gu)
    hq, sh = gpu_lib.swiglu_quantize(gt)
    assert sh.cpu().numpy().tobytes() == sh_ref.tobytes()
    assert np.array_equal(hq.cpu().numpy(), hq_ref)


def test_swiglu_quantize_edge_cases(gpu_lib):
    say("swiglu_quantize edge cases")
    F = 96
    gu = np.zeros((4, 2 * F), np.float32)
    gu[1, :F] = np.linspace(-120.0, 120.0, F)      # both clamps of the exponential
    gu[1, F:] = 1.0
    gu[2, :F] = 30.0
    gu[2, F:] = np.linspace(-2.0, 2.0, F)
    gu[3, :F] = -1e-30
    gu[3, F:] = 1e30
    hq_ref, sh_ref, _ = oracle.swiglu_quantize(gu)
    hq, sh = gpu_lib.swiglu_quantize(dev(gu))
    assert sh.cpu().numpy().tobytes() == sh_ref.tobytes()
    assert np.array_equal(hq.cpu().numpy(), hq_ref)


def test_producers_feed_the_product(gpu_lib):
    """norm -> gate/up product -> gate -> down product on the library path equals the same chain on the oracle
    (int8 codes, scales and accumulators bit-exact; bf16 hand-over between the two products as a block does)."""
    say("producer chain")
    M, H, F = 6, 512, 1280
    x = synth.activations(M, H, config=0, layer=5, tensor=6)
    Wgu = synth.weights(2 * F, H, config=0, layer=5, tensor=7)
    Wd = synth.weights(H, F, config=0, layer=5, tensor=8)
    # oracle
    xq_r, sx_r, _ = oracle.rmsnorm_quantize(x, None, 1e-6)
    cgu, ggu = oracle.quantize_weights(Wgu)
    acc1_r = oracle.ternary_matmul(xq_r, cgu)
    # library
    xq, sx = gpu_lib.rmsnorm_quantize(dev(x), None, 1e-6)
    pgu, gam_gu = gpu_lib.quantize_weights(dev(Wgu))
    acc1 = gpu_lib.linear(xq, sx, pgu, gam_gu, 2 * F, y_dtype=gpu_lib.I32)
    assert np.array_equal(acc1.cpu().numpy(), acc1_r)
    gu16 = gpu_lib.linear(xq, sx, pgu, gam_gu, 2 * F, y_dtype=gpu_lib.BF16)
    # the oracle continues from the bf16 values the library handed over (its own y is fp64; the hand-over
    # rounding is the library's and was checked against the oracle by the product tests)
    hq_r, sh_r, _ = oracle.swiglu_quantize(gu16.float().cpu().numpy())
    hq, sh = gpu_lib.swiglu_quantize(gu16)
    assert np.array_equal(hq.cpu().numpy(), hq_r) and sh.cpu().numpy().tobytes() == sh_r.tobytes()
    cd, gd = oracle.quantize_weights(Wd)
    pd, gam_d = gpu_lib.quantize_weights(dev(Wd))
    y = gpu_lib.linear(hq, sh, pd, gam_d, H, y_dtype=gpu_lib.F32)
    y_ref = oracle.rescale(oracle.ternary_matmul(hq_r, cd), gd, sh_r)
    check_y(y.cpu().numpy(), y_ref, RTOL_F32)


def _swiglu_definition(gu):
    """silu(gate) * up and its per-token absmax quantization straight from their definitions, in numpy fp64
    (not the oracle's fixed-step exponential: an independent yardstick for it and for the GPU alike)."""
    gu = np.asarray(gu, np.float64)
    F = gu.shape[1] // 2
    a, b = gu[:, :F], gu[:, F:]
    with np.errstate(over="ignore"):
        h = a / (1.0 + np.exp(-a)) * b
    s = np.maximum(np.abs(h).max(axis=1), 1e-5)
    q = np.clip(np.rint(h * (127.0 / s)[:, None]), -127, 127)
    return q, s, h


@pytest.mark.parametrize("M,F", [(1, 8640), (4, 11008), (70, 4096), (2, 28672), (3, 1003)])
@pytest.mark.parametrize("bf16", [False, True])
def test_swiglu_quantize_against_the_fp64_definition(gpu_lib, M, F, bf16):
    """The HIP SwiGLU -> int8 producer against numpy's fp64 evaluation of the definition (the bit-exact test above
    compares it with the oracle, whose exponential follows the same stated steps): scales within 1e-6 relative, every
    code within one step, at least 99 % equal.  Large |gate| values exercise both clamps of the exponential."""
    say("swiglu_quantize vs fp64 definition M=%d F=%d bf16=%s" % (M, F, bf16))
    gu, bits = synth.activations(M, 2 * F, config=2, layer=F % 7, tensor=15, bf16=True)
    if not bf16:
        gu = synth.activations(M, 2 * F, config=0, layer=F % 7, tensor=15)
        gu[0, :8] = [-120.0, -95.0, -88.5, -87.0, 87.5, 88.0, 100.0, 3.0e4]
        gu[0, F:F + 8] = 0.01                                     # small up values: these products must not set the scale
    gt = bf16_tensor(bits).view(M, 2 * F) if bf16 else dev(gu)
    q_def, s_def, _ = _swiglu_definition(gu)
    hq, sh = gpu_lib.swiglu_quantize(gt)
    hq, sh = hq.cpu().numpy().astype(np.int64), sh.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(sh - s_def) <= 1e-6 * s_def), np.abs(sh / s_def - 1).max()
    diff = np.abs(hq - q_def)
    assert diff.max() <= 1 and (diff == 0).mean() >= 0.99, (diff.max(), (diff == 0).mean())


@pytest.mark.parametrize("M,F,K", [(1, 8640, 3200), (2, 1008, 1040)])
def test_ffn_gate_up_fused_against_the_fp64_definition(gpu_lib, M, F, K):
    """h of the gate/up launch with the gate in its epilogue, against numpy fp64: the product's y from the oracle's
    integers (exact) rescaled in fp64, the gate from its definition; fp32 h within 5e-5, bf16 h within 1e-2."""
    say("ffn gate/up vs fp64 definition M=%d F=%d K=%d" % (M, F, K))
    W = synth.weights(2 * F, K, config=0, layer=M + 60, tensor=0)
    x, bits = synth.activations(M, K, config=2, layer=M + 60, tensor=7, bf16=True)
    ref = oracle.bitlinear(x, W)
    _, _, h_def = _swiglu_definition(ref["y"])
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    xd = bf16_tensor(bits).view(M, K)
    h32 = gpu_lib.ffn_gate_up_fused(xd, packed, gamma, F).cpu().numpy().astype(np.float64)
    h16 = gpu_lib.ffn_gate_up_fused(xd, packed, gamma, F, h_dtype=gpu_lib.BF16).float().cpu().numpy().astype(np.float64)
    big = np.abs(h_def) > 1e-30
    assert np.abs(h32[big] / h_def[big] - 1).max() <= 5e-5
    assert np.abs(h16[big] / h_def[big] - 1).max() <= RTOL_BF16
    assert np.all(h32[~big] == 0)


def test_decoder_chain_in_a_hip_graph_matches_the_oracle(gpu_lib):
    """Three layers of the 3B-class decoder's BitLinear chain at M = 1 as the benchmark runs it -- four fused launches
    per layer, captured into one HIP graph, every launch reading what the previous one wrote (the attention itself is
    not on the path: the first `hidden` outputs of the QKV projection stand in for its output).  The graph is replayed
    several times with eager work in between; every replay must equal the eager run bit for bit, and every link is
    recomputed by the oracle from the values its input buffer holds: accumulators bit-exact (read through the I32
    output of the same entry point), bf16 outputs within 1e-2."""
    say("decoder chain graph, 3B shapes")
    H, F, L = 3200, 8640, 3
    eps = 1e-6
    shapes = {"qkv": (H, 3 * H), "o": (H, H), "gate_up": (H, 2 * F), "down": (F, H)}
    Wn, Wd = [], []
    for l in range(L):
        wl, dl = {}, {}
        for t, (name, (K, N)) in enumerate(shapes.items()):
            W = synth.weights(N, K, config=1, layer=l, tensor=t)
            wl[name] = W
            dl[name] = gpu_lib.quantize_weights(dev(W))
        Wn.append(wl)
        Wd.append(dl)
    rng = np.random.default_rng([2402, 1, 77])
    gains = [(1.0 + 0.1 * rng.standard_normal(H)).astype(np.float32) for _ in range(2 * L)]
    gd = [dev(g) for g in gains]
    x0, bits = synth.activations(1, H, config=1, layer=0, tensor=100, bf16=True)
    x0d = bf16_tensor(bits).view(1, H)
    buf = [{"qkv": torch.zeros((1, 3 * H), dtype=torch.bfloat16, device="cuda"),
            "o": torch.zeros((1, H), dtype=torch.bfloat16, device="cuda"),
            "h": torch.zeros((1, F), dtype=torch.bfloat16, device="cuda"),
            "down": torch.zeros((1, H), dtype=torch.bfloat16, device="cuda")} for _ in range(L)]
    att = [torch.zeros((1, H), dtype=torch.bfloat16, device="cuda") for _ in range(L)]

    def chain():
        x = x0d
        for l in range(L):
            d, b = Wd[l], buf[l]
            gpu_lib.rmsnorm_linear_fused(x, gd[2 * l], eps, d["qkv"][0], d["qkv"][1], 3 * H, y_dtype=gpu_lib.BF16, y=b["qkv"])
            att[l].copy_(b["qkv"][:, :H])                         # stand-in for the attention output
            gpu_lib.linear_fused(att[l], d["o"][0], d["o"][1], H, y_dtype=gpu_lib.BF16, y=b["o"])
            gpu_lib.ffn_gate_up_fused(b["o"], d["gate_up"][0], d["gate_up"][1], F, norm=True, g=gd[2 * l + 1], eps=eps,
                                      h_dtype=gpu_lib.BF16, h=b["h"])
            gpu_lib.linear_fused(b["h"], d["down"][0], d["down"][1], H, y_dtype=gpu_lib.BF16, y=b["down"])
            x = b["down"]

    def snapshot():
        torch.cuda.synchronize()
        return [{k: v.clone() for k, v in b.items()} for b in buf]

    chain()
    eager = snapshot()
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        chain()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        chain()
    for rep in range(3):
        for b in buf:                                             # eager work between the replays: wipe the buffers
            for v in b.values():
                v.fill_(float(rep + 1))
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for l in range(L):
            for k in eager[l]:
                assert torch.equal(got[l][k], eager[l][k]), (rep, l, k)

    def f32(t):
        return t.float().cpu().numpy()

    # every link against the oracle, from the values in its input buffer
    x_in = x0
    for l in range(L):
        W, d, b = Wn[l], Wd[l], eager[l]
        x_in_d = x0d if l == 0 else eager[l - 1]["down"]
        # QKV: RMSNorm -> int8 -> product
        xq, sx, _ = oracle.rmsnorm_quantize(x_in, gains[2 * l], eps)
        c, g = oracle.quantize_weights(W["qkv"])
        acc = oracle.ternary_matmul(xq, c)
        acc_gpu = gpu_lib.rmsnorm_linear_fused(x_in_d, gd[2 * l], eps, d["qkv"][0], d["qkv"][1], 3 * H, y_dtype=gpu_lib.I32)
        assert np.array_equal(acc_gpu.cpu().numpy(), acc), (l, "qkv")
        check_y(f32(b["qkv"]), oracle.rescale(acc, g, sx), RTOL_BF16)
        # O: absmax -> int8 -> product, on the stand-in attention output
        a_in = f32(b["qkv"])[:, :H]
        xq, sx = oracle.quantize_acts(a_in)
        c, g = oracle.quantize_weights(W["o"])
        acc = oracle.ternary_matmul(xq, c)
        acc_gpu = gpu_lib.linear_fused(b["qkv"][:, :H].contiguous(), d["o"][0], d["o"][1], H, y_dtype=gpu_lib.I32)
        assert np.array_equal(acc_gpu.cpu().numpy(), acc), (l, "o")
        check_y(f32(b["o"]), oracle.rescale(acc, g, sx), RTOL_BF16)
        # gate/up: RMSNorm -> int8 -> product -> gate
        xq, sx, _ = oracle.rmsnorm_quantize(f32(b["o"]), gains[2 * l + 1], eps)
        c, g = oracle.quantize_weights(W["gate_up"])
        acc = oracle.ternary_matmul(xq, c)
        acc_gpu = gpu_lib.rmsnorm_linear_fused(b["o"], gd[2 * l + 1], eps, d["gate_up"][0], d["gate_up"][1], 2 * F,
                                               y_dtype=gpu_lib.I32)
        assert np.array_equal(acc_gpu.cpu().numpy(), acc), (l, "gate_up")
        _, _, h_def = _swiglu_definition(oracle.rescale(acc, g, sx))
        check_y(f32(b["h"]), h_def, RTOL_BF16)
        # down
        xq, sx = oracle.quantize_acts(f32(b["h"]))
        c, g = oracle.quantize_weights(W["down"])
        acc = oracle.ternary_matmul(xq, c)
        acc_gpu = gpu_lib.linear_fused(b["h"], d["down"][0], d["down"][1], H, y_dtype=gpu_lib.I32)
        assert np.array_equal(acc_gpu.cpu().numpy(), acc), (l, "down")
        check_y(f32(b["down"]), oracle.rescale(acc, g, sx), RTOL_BF16)
        x_in = f32(b["down"])


# ------------------------------------------------------------------------------------------------
# a matrix quantized in row shards with the gamma of the whole (Eq. (3) is one mean per matrix)
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("N,K,bounds", [(4096, 1536, None), (1000, 528, [0, 16, 400, 1000]), (250, 4100, [0, 96, 250]),
                                        (33, 70, [0, 32, 33])])
@pytest.mark.parametrize("fmt", ["2bit", "trit5"])
def test_sharded_weight_quantization_reproduces_the_whole_tensor(gpu_lib, N, K, bounds, fmt):
    """G = 2, 4, 8 equal row shards (and ragged ones): each shard reports its (hi, lo) share of sum |W|, every shard is
    then quantized with all the shares; gamma and the codes must be those of one whole-tensor call and of the oracle,
    bit for bit, whatever the split and whatever the order of the shares."""
    say("sharded quantization %s N=%d K=%d" % (fmt, N, K))
    f = gpu_lib.PACK_2BIT if fmt == "2bit" else gpu_lib.PACK_TRIT5
    W = synth.weights(N, K, config=0, layer=N % 5, tensor=21)
    W[: N // 3] *= np.float32(3.0)                                # shards of different magnitude
    codes_ref, gamma_ref = oracle.quantize_weights(W)
    Wd = dev(W)
    _, gamma_whole = gpu_lib.quantize_weights(Wd, fmt=f)
    assert gamma_whole.cpu().numpy()[0] == gamma_ref
    splits = [bounds] if bounds else [[N * i // G for i in range(G + 1)] for G in (2, 4, 8)]
    for bnd in splits:
        shards = [Wd[bnd[i]:bnd[i + 1]].contiguous() for i in range(len(bnd) - 1)]
        sums = torch.stack([gpu_lib.abs_sum(s) for s in shards])
        hi_lo = sums.cpu().numpy()
        for i, s in enumerate(shards):                            # each share is the exact sum of its rows
            import math
            exact = math.fsum(np.abs(W[bnd[i]:bnd[i + 1]]).astype(np.float64).ravel().tolist())
            assert hi_lo[i, 0] == exact and abs(hi_lo[i, 1]) <= abs(exact) * 2.0 ** -52
        for order in (sums, sums.flip(0).contiguous()):
            for i, s in enumerate(shards):
                rows = bnd[i + 1] - bnd[i]
                packed, gamma = gpu_lib.quantize_weights_sharded(s, order, N, fmt=f)
                assert gamma.cpu().numpy()[0] == gamma_ref
                codes = gpu_lib.unpack_weights(packed, rows, K, fmt=f).cpu().numpy()
                assert np.array_equal(codes, codes_ref[bnd[i]:bnd[i + 1]])


# ------------------------------------------------------------------------------------------------
# one gamma per row segment (merged projections keep the scale of each original matrix, Eq. (3))
# ------------------------------------------------------------------------------------------------
def _segmented_reference(W, x, seg_rows):
    xq, sx = oracle.quantize_acts(x)
    codes, gammas, y_parts = [], [], []
    r0 = 0
    for rows in seg_rows:
        c, g = oracle.quantize_weights(W[r0:r0 + rows])
        codes.append(c)
        gammas.append(g)
        r0 += rows
    codes = np.vstack(codes)
    acc = oracle.ternary_matmul(xq, codes)
    y = np.empty(acc.shape, np.float64)
    gamma_rb = np.empty((W.shape[0] + 15) // 16, np.float32)
    r0 = 0
    for rows, g in zip(seg_rows, gammas):
        y[:, r0:r0 + rows] = oracle.rescale(np.ascontiguousarray(acc[:, r0:r0 + rows]), g, sx)
        gamma_rb[r0 // 16:(r0 + rows + 15) // 16] = g
        r0 += rows
    return dict(xq=xq, sx=sx, codes=codes, acc=acc, y=y, gamma_rb=gamma_rb)


SEGMENT_CASES = [  # (M, K, segment rows): every product kernel, ragged last segment, unequal segments
    (1, 528, [160, 48, 45]), (3, 272, [16, 16, 16, 16, 7]), (9, 1040, [4096, 1024, 1024]), (40, 528, [320, 64, 64]),
    (64, 2048, [8192, 8200]), (100, 272, [256, 256, 250]), (300, 528, [1280, 2560]), (1, 80, [33]),
]


@pytest.mark.parametrize("M,K,seg_rows", SEGMENT_CASES)
def test_segmented_gamma_matches_oracle(gpu_lib, M, K, seg_rows):
    say("segmented M=%d K=%d segs=%s" % (M, K, seg_rows))
    N = sum(seg_rows)
    W = synth.weights(N, K, config=0, layer=len(seg_rows), tensor=9)
    r0 = 0
    for i, rows in enumerate(seg_rows):          # segments of different magnitude, so that one gamma would be wrong
        W[r0:r0 + rows] *= np.float32(1.0 + 0.75 * i)
        r0 += rows
    x = synth.activations(M, K, config=0, layer=len(seg_rows), tensor=10)
    ref = _segmented_reference(W, x, seg_rows)
    packed, gamma_rb = gpu_lib.quantize_weights_segmented(dev(W), seg_rows)
    assert gamma_rb.cpu().numpy().tobytes() == ref["gamma_rb"].tobytes()
    assert np.array_equal(gpu_lib.unpack_weights(packed, N, K).cpu().numpy(), ref["codes"])
    xq, sx = gpu_lib.quantize_acts(dev(x))
    kernels = [gpu_lib.KERNEL_AUTO, gpu_lib.KERNEL_REFERENCE, gpu_lib.KERNEL_GEMM,
               gpu_lib.KERNEL_GEMM_TILES[(96, 128)], gpu_lib.KERNEL_GEMM_TILES[(64, 128)], gpu_lib.KERNEL_GEMM_TILES[(128, 256)],
               gpu_lib.KERNEL_GEMM_TILES_K2[(96, 128)], gpu_lib.KERNEL_GEMM_TILES_K2[(64, 256)], gpu_lib.KERNEL_GEMM_TILES_WIDE[(128, 512)]]
    if M <= 64:
        kernels.append(gpu_lib.KERNEL_GEMV)
    for kern in kernels:
        acc = gpu_lib.linear_segmented(xq, sx, packed, gamma_rb, N, y_dtype=gpu_lib.I32, kernel=kern)
        assert np.array_equal(acc.cpu().numpy(), ref["acc"])
        y32 = gpu_lib.linear_segmented(xq, sx, packed, gamma_rb, N, y_dtype=gpu_lib.F32, kernel=kern)
        check_y(y32.cpu().numpy(), ref["y"], RTOL_F32)
        y16 = gpu_lib.linear_segmented(xq, sx, packed, gamma_rb, N, y_dtype=gpu_lib.BF16, kernel=kern)
        check_y(y16.float().cpu().numpy(), ref["y"], RTOL_BF16)
    if M <= 16:
        yf = gpu_lib.linear_fused_segmented(dev(x), packed, gamma_rb, N, y_dtype=gpu_lib.F32)
        check_y(yf.cpu().numpy(), ref["y"], RTOL_F32)


def test_segmented_with_one_segment_equals_plain(gpu_lib):
    say("segmented, one segment")
    N, K, M = 1000, 528, 5
    W = synth.weights(N, K, config=0, layer=3, tensor=11)
    x = synth.activations(M, K, config=0, layer=3, tensor=12)
    p1, g1 = gpu_lib.quantize_weights(dev(W))
    p2, grb = gpu_lib.quantize_weights_segmented(dev(W), [N])
    assert torch.equal(p1, p2)
    assert torch.equal(grb, g1.expand(grb.numel()))
    xq, sx = gpu_lib.quantize_acts(dev(x))
    assert torch.equal(gpu_lib.linear(xq, sx, p1, g1, N), gpu_lib.linear_segmented(xq, sx, p2, grb, N))


# ------------------------------------------------------------------------------------------------
# the 5-trits-per-byte format
# ------------------------------------------------------------------------------------------------
TRIT_WEIGHT_SHAPES = [(4096, 1536), (16, 320), (1, 1), (37, 129), (100, 70), (17, 1000), (250, 4100)]


@pytest.mark.parametrize("N,K", TRIT_WEIGHT_SHAPES)
def test_trit5_quantize_weights_matches_oracle(gpu_lib, N, K):
    say("trit5 quantize_weights N=%d K=%d" % (N, K))
    W = synth.weights(N, K, config=0, layer=N % 5, tensor=2)
    codes_ref, gamma_ref = oracle.quantize_weights(W)
    packed, gamma = gpu_lib.quantize_weights(dev(W), fmt=gpu_lib.PACK_TRIT5)
    assert gamma.cpu().numpy()[0].tobytes() == np.float32(gamma_ref).tobytes()
    assert packed.numel() == gpu_lib.packed_bytes(N, K, gpu_lib.PACK_TRIT5)
    assert np.array_equal(gpu_lib.unpack_weights(packed, N, K, fmt=gpu_lib.PACK_TRIT5).cpu().numpy(), codes_ref)
    dec, pad_zero = decode_trit5(packed.cpu().numpy(), N, K)
    assert pad_zero and np.array_equal(dec, codes_ref)
    # same codes as the 2-bit format, from bf16 weights too
    Wf, bits = synth.to_bf16(W)
    p5, _ = gpu_lib.quantize_weights(bf16_tensor(bits).view(N, K), fmt=gpu_lib.PACK_TRIT5)
    p2, _ = gpu_lib.quantize_weights(bf16_tensor(bits).view(N, K))
    assert torch.equal(gpu_lib.unpack_weights(p5, N, K, fmt=gpu_lib.PACK_TRIT5), gpu_lib.unpack_weights(p2, N, K))


TRIT_LINEAR_SHAPES = [(1, 4096, 1536), (16, 4096, 1536), (1, 17, 16), (3, 100, 80), (7, 250, 1040), (1, 3200, 3200),
                      (2, 32800, 528), (2, 64, 8640), (16, 300, 4112), (20, 70, 336), (70, 40, 640),
                      (33, 1000, 656), (100, 2000, 320),      # more than 16 tokens: walked 16 at a time
                      # the two-row-block forms: 65 steps (the last partial) on 513 row blocks; 13 steps on 1025
                      (2, 8200, 20496), (3, 16400, 4112)]


@pytest.mark.parametrize("M,N,K", TRIT_LINEAR_SHAPES)
def test_trit5_linear_matches_oracle(gpu_lib, M, N, K):
    say("trit5 linear M=%d N=%d K=%d" % (M, N, K))
    W = synth.weights(N, K, config=0, layer=M + 40, tensor=0)
    x = synth.activations(M, K, config=0, layer=M + 40)
    ref = oracle.bitlinear(x, W)
    packed, gamma = gpu_lib.quantize_weights(dev(W), fmt=gpu_lib.PACK_TRIT5)
    xq, sx = gpu_lib.quantize_acts(dev(x))
    kernels = [gpu_lib.KERNEL_AUTO, gpu_lib.KERNEL_REFERENCE] + ([gpu_lib.KERNEL_GEMV] if M <= 16 else [])
    for kern in kernels:
        acc = gpu_lib.linear(xq, sx, packed, gamma, N, fmt=gpu_lib.PACK_TRIT5, y_dtype=gpu_lib.I32, kernel=kern)
        assert np.array_equal(acc.cpu().numpy(), ref["acc"]), "kernel %d" % kern
        y32 = gpu_lib.linear(xq, sx, packed, gamma, N, fmt=gpu_lib.PACK_TRIT5, y_dtype=gpu_lib.F32, kernel=kern)
        check_y(y32.cpu().numpy(), ref["y"], RTOL_F32)
        y16 = gpu_lib.linear(xq, sx, packed, gamma, N, fmt=gpu_lib.PACK_TRIT5, y_dtype=gpu_lib.BF16, kernel=kern)
        check_y(y16.float().cpu().numpy(), ref["y"], RTOL_BF16)
    if M > 16:
        with pytest.raises(gpu_lib.BitnetError) as e:
            gpu_lib.linear(xq, sx, packed, gamma, N, fmt=gpu_lib.PACK_TRIT5, kernel=gpu_lib.KERNEL_GEMV)
        assert e.value.status == 8


@pytest.mark.parametrize("N,K", [(4096, 1536), (16, 320), (1, 1), (37, 129), (100, 70), (17, 1000), (250, 4100), (33, 641), (3200, 3200)])
def test_repack_between_the_formats_is_byte_exact(gpu_lib, N, K):
    """The device repacking in both directions: the result must be the very bytes bitnet_quantize_weights writes in
    the target format (codes from the oracle's quantizer, padding zero), for K not a multiple of 64, 80 or 320 too."""
    say("repack N=%d K=%d" % (N, K))
    W = synth.weights(N, K, config=0, layer=N % 7, tensor=41)
    codes_ref, _ = oracle.quantize_weights(W)
    p2, _ = gpu_lib.quantize_weights(dev(W), fmt=gpu_lib.PACK_2BIT)
    p5, _ = gpu_lib.quantize_weights(dev(W), fmt=gpu_lib.PACK_TRIT5)
    to2 = torch.full_like(p2, 0x5A)
    to5 = torch.full_like(p5, 0x5A)
    gpu_lib.repack_weights(p5, N, K, gpu_lib.PACK_TRIT5, gpu_lib.PACK_2BIT, out=to2)
    gpu_lib.repack_weights(p2, N, K, gpu_lib.PACK_2BIT, gpu_lib.PACK_TRIT5, out=to5)
    assert torch.equal(to2, p2) and torch.equal(to5, p5)
    dec2, pad2 = decode_2bit(to2.cpu().numpy(), N, K)
    dec5, pad5 = decode_trit5(to5.cpu().numpy(), N, K)
    assert pad2 and pad5 and np.array_equal(dec2, codes_ref) and np.array_equal(dec5, codes_ref)
    lib = gpu_lib.load()
    assert lib.bitnet_repack_weights(p2.data_ptr(), 0, N, K, to5.data_ptr(), 0, None) == 4      # same format both sides
    assert lib.bitnet_repack_weights(None, 0, N, K, to5.data_ptr(), 1, None) == 1
    assert lib.bitnet_repack_weights(p2.data_ptr() + 1, 0, N, K, to5.data_ptr(), 1, None) == 5


@pytest.mark.parametrize("M,N,K", [(17, 300, 528), (65, 300, 528), (100, 520, 1040), (300, 1000, 3200), (130, 8000, 272),
                                   (513, 270, 4112), (256, 4096, 1296), (2048, 5120, 640)])
def test_trit5_prefill_through_the_workspace_matches_oracle(gpu_lib, M, N, K):
    """5-trit weights at more than 16 tokens through bitnet_linear_ws: repacked to 2 bits in the workspace, then the
    batched-decode or MFMA prefill kernel -- accumulators bit-exact, outputs within the bars; with a workspace that
    cannot hold the copy the 16-tokens-at-a-time route gives the same integers."""
    say("trit5 prefill M=%d N=%d K=%d" % (M, N, K))
    W = synth.weights(N, K, config=0, layer=M % 9, tensor=42)
    x = synth.activations(M, K, config=0, layer=M % 9, tensor=43)
    ref = oracle.bitlinear(x, W)
    p5, gamma = gpu_lib.quantize_weights(dev(W), fmt=gpu_lib.PACK_TRIT5)
    xq, sx = gpu_lib.quantize_acts(dev(x))
    need = gpu_lib.linear_workspace(M, N, K, fmt=gpu_lib.PACK_TRIT5)
    assert need >= gpu_lib.packed_bytes(N, K, gpu_lib.PACK_2BIT)
    ws = torch.full((need + 64,), 0x77, dtype=torch.uint8, device="cuda")
    acc = gpu_lib.linear_ws(xq, sx, p5, gamma, N, ws[:need], fmt=gpu_lib.PACK_TRIT5, y_dtype=gpu_lib.I32)
    assert np.array_equal(acc.cpu().numpy(), ref["acc"])
    assert bool((ws[need:] == 0x77).all())                                  # nothing written past the stated size
    check_y(gpu_lib.linear_ws(xq, sx, p5, gamma, N, ws[:need], fmt=gpu_lib.PACK_TRIT5, y_dtype=gpu_lib.F32).cpu().numpy(), ref["y"], RTOL_F32)
    check_y(gpu_lib.linear_ws(xq, sx, p5, gamma, N, ws[:need], fmt=gpu_lib.PACK_TRIT5, y_dtype=gpu_lib.BF16).float().cpu().numpy(),
            ref["y"], RTOL_BF16)
    small = ws[:1024]
    acc2 = gpu_lib.linear_ws(xq, sx, p5, gamma, N, small, fmt=gpu_lib.PACK_TRIT5, y_dtype=gpu_lib.I32)
    assert torch.equal(acc2, acc)
    assert gpu_lib.linear_workspace(16, N, K, fmt=gpu_lib.PACK_TRIT5) == 0  # the decode kernel reads 5-trit weights directly


def test_trit5_is_rejected_where_unsupported(gpu_lib):
    say("trit5 limits")
    W = dev(synth.weights(32, 320, config=0, layer=1))
    packed, gamma = gpu_lib.quantize_weights(W, fmt=gpu_lib.PACK_TRIT5)
    x = dev(synth.activations(1, 320, config=0, layer=1))
    with pytest.raises(gpu_lib.BitnetError) as e:
        gpu_lib.linear_fused(x, packed, gamma, 32, fmt=gpu_lib.PACK_TRIT5)
    assert e.value.status == 4
    xq, sx = gpu_lib.quantize_acts(x)
    with pytest.raises(gpu_lib.BitnetError) as e:
        gpu_lib.linear(xq, sx, packed, gamma, 32, fmt=gpu_lib.PACK_TRIT5, kernel=gpu_lib.KERNEL_GEMM)
    assert e.value.status == 8


@pytest.mark.parametrize("M,K", [(2, 28672), (2, 262144), (20, 262144), (70, 262144)])
def test_linear_extreme_accumulators(gpu_lib, M, K):
    """Every product at +-127 with all-(+1) / all-(-1) rows: the largest accumulators a shape can give, up to the
    largest K the library accepts (262144: 64 * 127 * K is the last value below 2^31 that the kernels' scaled
    accumulators must hold), on the M <= 4, skinny and MFMA paths."""
    say("linear extreme accumulators M=%d K=%d" % (M, K))
    N = 32
    W = np.ones((N, K), np.float32)
    W[1::2] = -1.0
    x = np.full((M, K), 3.0, np.float32)
    x[1::2] = -3.0
    ref = oracle.bitlinear(x, W)
    assert abs(int(ref["acc"][0, 0])) == 127 * K
    packed, gamma = gpu_lib.quantize_weights(dev(W))
    xq, sx = gpu_lib.quantize_acts(dev(x))
    for kern in (gpu_lib.KERNEL_REFERENCE, gpu_lib.KERNEL_GEMM) + ((gpu_lib.KERNEL_GEMV,) if M <= 64 else ()):
        acc = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.I32, kernel=kern)
        assert np.array_equal(acc.cpu().numpy(), ref["acc"])
    with pytest.raises(gpu_lib.BitnetError) as e:            # one column more than the accumulators can take
        gpu_lib.packed_bytes(N, K + 16) if K == 262144 else gpu_lib.packed_bytes(0, K)
    assert e.value.status == 2


def test_linear_is_deterministic(gpu_lib):
    say("linear determinism")
    M, N, K = 8, 1000, 3200
    packed, gamma = gpu_lib.quantize_weights(dev(synth.weights(N, K, config=0, layer=3)))
    xq, sx = gpu_lib.quantize_acts(dev(synth.activations(M, K, config=0, layer=3)))
    a = gpu_lib.linear(xq, sx, packed, gamma, N)
    b = gpu_lib.linear(xq, sx, packed, gamma, N)
    assert torch.equal(a, b)


def test_outputs_do_not_spill_past_their_buffers(gpu_lib):
    say("canaries")
    M, N, K = 3, 50, 144
    W = dev(synth.weights(N, K, config=0, layer=4))
    x = dev(synth.activations(M, K, config=0, layer=4))
    nbytes = gpu_lib.packed_bytes(N, K)
    big = torch.full((nbytes + 64,), 0xAB, dtype=torch.uint8, device="cuda")
    packed, gamma = gpu_lib.quantize_weights(W, packed=big[:nbytes])
    assert bool((big[nbytes:] == 0xAB).all())
    xq_big = torch.full((M * K + 64,), 0x55, dtype=torch.int8, device="cuda")
    xq, sx = gpu_lib.quantize_acts(x, xq=xq_big[: M * K].view(M, K))
    assert bool((xq_big[M * K:] == 0x55).all())
    y_big = torch.full((M * N + 16,), 7.0, dtype=torch.float32, device="cuda")
    for kern in ((gpu_lib.KERNEL_REFERENCE, gpu_lib.KERNEL_GEMV, gpu_lib.KERNEL_GEMM) + tuple(gpu_lib.KERNEL_GEMM_TILES.values()) +
                 tuple(gpu_lib.KERNEL_GEMM_TILES_K2.values()) + tuple(gpu_lib.KERNEL_GEMM_TILES_WIDE.values())):
        gpu_lib.linear(xq, sx, packed, gamma, N, y=y_big[: M * N].view(M, N), kernel=kern)
        assert bool((y_big[M * N:] == 7.0).all())


# ------------------------------------------------------------------------------------------------
# maximum sizes: operands beyond 2^31 elements (an output-embedding-sized matrix, a prefill's worth of logits)
# ------------------------------------------------------------------------------------------------
def test_matrix_and_output_beyond_2_to_31_elements(gpu_lib):
    """135168 x 16384 weights (2.2e9 > 2^31 elements, 8.9 GB in fp32) and 16384 x 135168 outputs: every index that is a
    product of two dimensions must be 64 bits wide.  The matrix is a 4224-element pattern repeated 2^19 times (the pattern
    is not aligned with rows or row blocks), so its gamma and codes are those the oracle gives for the pattern -- the
    exact sum scales by a power of two and the fp64 division sees the same quotient -- and the expected tensors are laid
    out by torch, not by this library.  Accumulators are compared with torch's fp32 matrix product of the expected codes
    and the oracle-checked x_q, which is exact here (|acc| <= 127 * 16384 < 2^24)."""
    N, K, period = 135168, 16384, 4224
    if torch.cuda.mem_get_info()[0] < 60e9:
        pytest.skip("needs 60 GB of free device memory")
    say("beyond 2^31 elements: N=%d K=%d" % (N, K))
    assert N * K > 2 ** 31 and (N * K) % period == 0 and K % period != 0
    reps = N * K // period
    assert reps == 2 ** 19
    P = synth.weights(33, 128, config=0, layer=3, tensor=41).reshape(1, period)
    codes_p, gamma_p = oracle.quantize_weights(P)
    W = dev(P.reshape(-1)).repeat(reps).view(N, K)
    packed, gamma = gpu_lib.quantize_weights(W)
    del W
    assert gamma.cpu().numpy()[0] == gamma_p
    expected = dev(codes_p.reshape(-1)).repeat(reps).view(N, K)
    codes = gpu_lib.unpack_weights(packed, N, K)
    assert torch.equal(codes, expected)
    del codes
    ef = expected.to(torch.float32)
    del expected

    # decode: 1 and 4 tokens (and the launch that quantizes x itself), accumulators over all 135168 rows
    x, bits = synth.activations(4, K, config=2, layer=1, tensor=42, bf16=True)
    xq_ref, sx_ref = oracle.quantize_acts(x)
    xd = bf16_tensor(bits).view(4, K)
    xq, sx = gpu_lib.quantize_acts(xd)
    assert np.array_equal(xq.cpu().numpy(), xq_ref) and sx.cpu().numpy().tobytes() == sx_ref.tobytes()
    acc_ref = (ef @ xq.to(torch.float32).T).T.contiguous().to(torch.int32)
    assert int(acc_ref.abs().max()) < 2 ** 24
    say("beyond 2^31 elements: decode")
    for M in (1, 4):
        acc = gpu_lib.linear(xq[:M], sx[:M], packed, gamma, N, y_dtype=gpu_lib.I32)
        assert torch.equal(acc, acc_ref[:M])
    assert torch.equal(gpu_lib.linear_fused(xd[:1], packed, gamma, N, y_dtype=gpu_lib.I32), acc_ref[:1])
    y = gpu_lib.linear(xq, sx, packed, gamma, N, y_dtype=gpu_lib.F32).cpu().numpy()
    check_y(y, oracle.rescale(acc_ref.cpu().numpy(), gamma_p, sx_ref), RTOL_F32)

    # prefill: 16384 tokens, 2.2e9 outputs; sampled tokens on both sides of element 2^31 of y, the first and the last
    M = 16384
    say("beyond 2^31 elements: prefill, M=%d" % M)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(4242)
    X = torch.randn((M, K), device="cuda", generator=gen, dtype=torch.float32).to(torch.bfloat16)
    xq2, sx2 = gpu_lib.quantize_acts(X)
    edge = 2 ** 31 // N
    rows = [0, 1, 127, 128, edge - 1, edge, edge + 1, M - 129, M - 2, M - 1]
    xs = X[rows].to(torch.float32).cpu().numpy()
    xq_s, sx_s = oracle.quantize_acts(xs)
    assert np.array_equal(xq2[rows].cpu().numpy(), xq_s) and sx2[rows].cpu().numpy().tobytes() == sx_s.tobytes()
    acc_s = (ef @ xq2[rows].to(torch.float32).T).T.contiguous().to(torch.int32)
    del ef
    acc2 = gpu_lib.linear(xq2, sx2, packed, gamma, N, y_dtype=gpu_lib.I32)
    assert tuple(acc2.shape) == (M, N) and acc2.numel() > 2 ** 31
    assert torch.equal(acc2[rows], acc_s)
    del acc2
    y2 = gpu_lib.linear(xq2, sx2, packed, gamma, N, y_dtype=gpu_lib.BF16)
    check_y(y2[rows].to(torch.float32).cpu().numpy(), oracle.rescale(acc_s.cpu().numpy(), gamma_p, sx_s), RTOL_BF16)


def test_activations_beyond_2_to_31_elements(gpu_lib):
    """75198 tokens of 28672 elements (2.16e9 > 2^31): the three producers of int8 activations on sampled tokens on both
    sides of element 2^31, the first and the last, against the oracle."""
    K = 28672
    M = 2 ** 31 // K + 300
    if torch.cuda.mem_get_info()[0] < 20e9:
        pytest.skip("needs 20 GB of free device memory")
    say("activations beyond 2^31 elements: M=%d K=%d" % (M, K))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(777)
    X = torch.empty((M, K), device="cuda", dtype=torch.bfloat16)
    for m0 in range(0, M, 8192):                                     # drawn in slabs: no fp32 copy of the whole tensor
        m1 = min(M, m0 + 8192)
        X[m0:m1] = torch.randn((m1 - m0, K), device="cuda", generator=gen, dtype=torch.float32).to(torch.bfloat16)
    assert X.numel() > 2 ** 31
    edge = 2 ** 31 // K
    rows = [0, 1, edge - 1, edge, edge + 1, M - 2, M - 1]
    xs = X[rows].to(torch.float32).cpu().numpy()
    g = (1.0 + 0.25 * np.random.default_rng(5).standard_normal(K)).astype(np.float32)

    xq, sx = gpu_lib.quantize_acts(X)
    xq_ref, sx_ref = oracle.quantize_acts(xs)
    assert np.array_equal(xq[rows].cpu().numpy(), xq_ref) and sx[rows].cpu().numpy().tobytes() == sx_ref.tobytes()
    del xq
    zq, sz = gpu_lib.rmsnorm_quantize(X, dev(g), 1e-5)
    zq_ref, sz_ref, _ = oracle.rmsnorm_quantize(xs, g, 1e-5)
    assert np.array_equal(zq[rows].cpu().numpy(), zq_ref) and sz[rows].cpu().numpy().tobytes() == sz_ref.tobytes()
    del zq
    hq, sh = gpu_lib.swiglu_quantize(X)                              # rows as [gate | up] of F = K / 2
    hq_ref, sh_ref, _ = oracle.swiglu_quantize(xs)
    assert np.array_equal(hq[rows].cpu().numpy(), hq_ref) and sh[rows].cpu().numpy().tobytes() == sh_ref.tobytes()


# ------------------------------------------------------------------------------------------------
# the yardstick kernels that bench.py and the measurement tools time next to the product: they run and return
# ------------------------------------------------------------------------------------------------
@pytest.mark.gpu
def test_yardstick_kernels_run(gpu_lib):
    """The read-only, MFMA-only, K-loop-ladder and L2-read kernels of libbitnet_floors.so on small inputs: every launch
    is accepted and the device is healthy afterwards (their results are rates, not values -- nothing to compare)."""
    from paper_2402_17764_amd import floors
    lib = floors.load()
    s = torch.cuda.current_stream().cuda_stream
    a = torch.randint(-127, 128, (1 << 22,), dtype=torch.int8, device="cuda")
    b = (torch.randint(-1, 2, (1 << 22,), dtype=torch.int8, device="cuda") * 64).to(torch.int8)
    big = torch.zeros(64 << 20, dtype=torch.uint8, device="cuda")
    out = torch.zeros(8, dtype=torch.int32, device="cuda")
    say("yardsticks: read_only")
    for (blocks, unroll) in floors.READ_SHAPES:
        assert lib.read_only_launch(big.data_ptr(), big.numel(), out.data_ptr(), blocks, unroll, s) == 0
    say("yardsticks: mfma_only")
    assert lib.mfma_only_launch(a.data_ptr(), b.data_ptr(), a.numel(), 512, 4, out.data_ptr(), s) == 0
    for rung in range(10):
        say("yardsticks: ladder rung %d" % rung)
        assert lib.prefill_ladder_launch(rung, a.data_ptr(), b.data_ptr(), a.numel(), 512, 3, big.data_ptr(), big.numel(),
                                         out.data_ptr(), s) == 0
    say("yardsticks: l2_read")
    for to_lds in (0, 1):
        assert lib.l2_read_launch(big.data_ptr(), 2 << 20, 2, 512, to_lds, out.data_ptr(), s) == 0
    torch.cuda.synchronize()
    assert int(out[2]) > 0                      # the ladder's last rung stamped its clocks

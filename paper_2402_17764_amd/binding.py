"""ctypes binding of the BitLinear HIP library: the names and arguments of include/bitnet.h.

Marshalling only: every function takes torch tensors that already live on the GPU (torch is used
for device memory and streams, nothing else), checks dtype / shape / contiguity, passes raw device
pointers and the current HIP stream through the C ABI, and raises BitnetError on a non-zero status.
There is no fallback: if the shared library has not been built, load() raises.  BITNET_HIP_LIBRARY names another build
of the same library to load instead (the host-sanitized one of paper_2402_17764_amd.build.build_library(sanitize=True)).
"""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("BITNET_HIP_LIBRARY") or os.path.join(HERE, "libbitnet_hip.so")

# enums of bitnet.h
OK = 0
F32, BF16, I32 = 0, 1, 2
PACK_2BIT, PACK_TRIT5 = 0, 1
KERNEL_AUTO, KERNEL_REFERENCE, KERNEL_GEMV, KERNEL_GEMM = 0, 1, 2, 3
ENTRY_LINEAR, ENTRY_LINEAR_FUSED, ENTRY_RMSNORM_LINEAR_FUSED, ENTRY_SWIGLU_LINEAR_FUSED = 0, 1, 2, 3
ENTRY_FFN_GATE_UP, ENTRY_FFN_GATE_UP_NORM = 4, 5
# the prefill kernel with a fixed workgroup tile, tokens x weight rows (tuning and tests)
KERNEL_GEMM_SPLITK = {2: 0x202, 4: 0x204, 8: 0x208}       # bitnet_linear_ws only
KERNEL_GEMM_TILES = {(128, 256): 0x142, (96, 256): 0x132, (64, 256): 0x122, (128, 128): 0x141, (96, 128): 0x131, (64, 128): 0x121}
KERNEL_GEMM_TILES_K2 = {(96, 128): 0x1B1, (64, 256): 0x1A2}      # eight waves in two K groups
KERNEL_GEMM_TILES_WIDE = {(128, 512): 0x14A}      # eight waves in two row groups

SYMBOLS = [
    "bitnet_version", "bitnet_status_string", "bitnet_packed_bytes", "bitnet_quantize_weights_workspace",
    "bitnet_quantize_weights", "bitnet_quantize_acts", "bitnet_linear", "bitnet_linear_variant",
    "bitnet_linear_fused", "bitnet_unpack_weights", "bitnet_rmsnorm_quantize", "bitnet_swiglu_quantize",
    "bitnet_quantize_weights_segmented", "bitnet_linear_segmented", "bitnet_linear_fused_segmented",
    "bitnet_rmsnorm_linear_fused", "bitnet_rmsnorm_linear_fused_segmented", "bitnet_swiglu_linear_fused",
    "bitnet_ffn_gate_up_fused", "bitnet_linear_workspace", "bitnet_linear_ws", "bitnet_linear_describe",
    "bitnet_entry_describe", "bitnet_abs_sum", "bitnet_quantize_weights_sharded", "bitnet_quantize_weights_static",
    "bitnet_repack_weights", "bitnet_linear_workspace_format",
]

_lib = None


class BitnetError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        msg = _lib.bitnet_status_string(status).decode() if _lib is not None else str(status)
        super().__init__("%s: %s (status %d)" % (where, msg, status))


def load():
    """Load libbitnet_hip.so (built by paper_2402_17764_amd.build).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("HIP library not built: %s is missing; run `python -m paper_2402_17764_amd.build`" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    i64, vp, ci, sz = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.bitnet_version.restype = ci
    lib.bitnet_version.argtypes = []
    lib.bitnet_status_string.restype = ctypes.c_char_p
    lib.bitnet_status_string.argtypes = [ci]
    lib.bitnet_packed_bytes.argtypes = [i64, i64, ci, ctypes.POINTER(sz)]
    lib.bitnet_quantize_weights_workspace.argtypes = [i64, i64, ctypes.POINTER(sz)]
    lib.bitnet_quantize_weights.argtypes = [vp, ci, i64, i64, ci, vp, vp, vp, sz, vp]
    lib.bitnet_quantize_weights_static.argtypes = [vp, ci, i64, i64, ci, vp, vp, vp]
    lib.bitnet_repack_weights.argtypes = [vp, ci, i64, i64, vp, ci, vp]
    lib.bitnet_linear_workspace_format.argtypes = [i64, i64, i64, ci, ctypes.POINTER(sz)]
    lib.bitnet_abs_sum.argtypes = [vp, ci, i64, i64, vp, vp, sz, vp]
    lib.bitnet_quantize_weights_sharded.argtypes = [vp, ci, i64, i64, ci, vp, ci, i64, vp, vp, vp]
    lib.bitnet_quantize_acts.argtypes = [vp, ci, i64, i64, vp, vp, vp]
    lib.bitnet_linear.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, vp, ci, vp]
    lib.bitnet_linear_variant.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, vp, ci, ci, vp]
    lib.bitnet_linear_fused.argtypes = [vp, ci, vp, vp, i64, i64, i64, ci, vp, ci, vp]
    lib.bitnet_unpack_weights.argtypes = [vp, i64, i64, ci, vp, vp]
    lib.bitnet_rmsnorm_quantize.argtypes = [vp, ci, vp, ctypes.c_float, i64, i64, vp, vp, vp]
    lib.bitnet_swiglu_quantize.argtypes = [vp, ci, i64, i64, vp, vp, vp]
    lib.bitnet_quantize_weights_segmented.argtypes = [vp, ci, i64, i64, ci, ctypes.POINTER(i64), ci, vp, vp, vp, sz, vp]
    lib.bitnet_linear_segmented.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, vp, ci, ci, vp]
    lib.bitnet_linear_fused_segmented.argtypes = [vp, ci, vp, vp, i64, i64, i64, ci, vp, ci, vp]
    lib.bitnet_rmsnorm_linear_fused.argtypes = [vp, ci, vp, ctypes.c_float, vp, vp, i64, i64, i64, ci, vp, ci, vp]
    lib.bitnet_rmsnorm_linear_fused_segmented.argtypes = [vp, ci, vp, ctypes.c_float, vp, vp, i64, i64, i64, ci, vp, ci, vp]
    lib.bitnet_swiglu_linear_fused.argtypes = [vp, ci, vp, vp, i64, i64, i64, ci, vp, ci, vp]
    lib.bitnet_linear_workspace.argtypes = [i64, i64, i64, ctypes.POINTER(sz)]
    lib.bitnet_linear_describe.argtypes = [i64, i64, i64, ctypes.c_int, sz, ctypes.c_char_p, sz]
    lib.bitnet_entry_describe.argtypes = [ci, ci, i64, i64, i64, ci, sz, ctypes.c_char_p, sz]
    lib.bitnet_linear_ws.argtypes = [vp, vp, vp, vp, ci, i64, i64, i64, ci, vp, ci, ci, vp, sz, vp]
    lib.bitnet_ffn_gate_up_fused.argtypes = [vp, ci, ci, vp, ctypes.c_float, vp, vp, ci, i64, i64, i64, ci, vp, ci, vp]
    for name in SYMBOLS[2:]:
        getattr(lib, name).restype = ci
    _lib = lib
    return lib


def _check(status, where):
    if status != OK:
        raise BitnetError(status, where)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, name, dtypes=None, ndim=None):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a CUDA/HIP tensor" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtypes is not None and t.dtype not in dtypes:
        raise TypeError("%s has dtype %s" % (name, t.dtype))
    if ndim is not None and t.dim() != ndim:
        raise ValueError("%s must be %d-D" % (name, ndim))
    return ctypes.c_void_p(t.data_ptr())


_FLOAT = {torch.float32: F32, torch.bfloat16: BF16}
_OUT = {F32: torch.float32, BF16: torch.bfloat16, I32: torch.int32}


def version():
    return int(load().bitnet_version())


def packed_bytes(N, K, fmt=PACK_2BIT):
    out = ctypes.c_size_t(0)
    _check(load().bitnet_packed_bytes(N, K, fmt, ctypes.byref(out)), "bitnet_packed_bytes")
    return int(out.value)


def quantize_weights_workspace(N, K):
    out = ctypes.c_size_t(0)
    _check(load().bitnet_quantize_weights_workspace(N, K, ctypes.byref(out)), "bitnet_quantize_weights_workspace")
    return int(out.value)


def quantize_weights(W, fmt=PACK_2BIT, packed=None, gamma=None, workspace=None):
    """W [N,K] fp32/bf16 on the GPU -> (packed uint8 tensor, gamma float32[1]); Eq. (1)-(3)."""
    lib = load()
    wp = _dev(W, "W", _FLOAT, 2)
    N, K = W.shape
    if packed is None:
        packed = torch.empty(packed_bytes(N, K, fmt), dtype=torch.uint8, device=W.device)
    if gamma is None:
        gamma = torch.empty(1, dtype=torch.float32, device=W.device)
    if workspace is None:
        workspace = torch.empty(quantize_weights_workspace(N, K), dtype=torch.uint8, device=W.device)
    _check(lib.bitnet_quantize_weights(wp, _FLOAT[W.dtype], N, K, fmt, _dev(packed, "packed"), _dev(gamma, "gamma"),
                                       _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                                       _stream()), "bitnet_quantize_weights")
    return packed, gamma


def quantize_weights_static(W, packed, gamma, fmt=PACK_2BIT):
    """quantize_weights through the entry point that allocates nothing: the caller passes every buffer, the scratch is
    the library's static device array."""
    lib = load()
    wp = _dev(W, "W", _FLOAT, 2)
    N, K = W.shape
    _check(lib.bitnet_quantize_weights_static(wp, _FLOAT[W.dtype], N, K, fmt, _dev(packed, "packed"),
                                              _dev(gamma, "gamma", (torch.float32,)), _stream()),
           "bitnet_quantize_weights_static")
    return packed, gamma


def abs_sum(W, out=None, workspace=None):
    """One row shard's share of Eq. (3): W [N,K] -> float64[2] (hi, lo) with hi + lo = sum |W|."""
    lib = load()
    wp = _dev(W, "W", _FLOAT, 2)
    N, K = W.shape
    if out is None:
        out = torch.empty(2, dtype=torch.float64, device=W.device)
    if workspace is None:
        workspace = torch.empty(quantize_weights_workspace(N, K), dtype=torch.uint8, device=W.device)
    _check(lib.bitnet_abs_sum(wp, _FLOAT[W.dtype], N, K, _dev(out, "sum", (torch.float64,)), _dev(workspace, "workspace"),
                              workspace.numel() * workspace.element_size(), _stream()), "bitnet_abs_sum")
    return out


def quantize_weights_sharded(W, sums, total_rows, fmt=PACK_2BIT, packed=None, gamma=None):
    """The rows W [N,K] of a matrix of total_rows rows, quantized with the gamma of the whole matrix: sums is a
    float64 [G,2] tensor of every shard's abs_sum pair -> (packed, gamma float32[1])."""
    lib = load()
    wp = _dev(W, "W", _FLOAT, 2)
    N, K = W.shape
    sp = _dev(sums, "sums", (torch.float64,))
    if sums.numel() % 2:
        raise ValueError("sums holds (hi, lo) pairs")
    if packed is None:
        packed = torch.empty(packed_bytes(N, K, fmt), dtype=torch.uint8, device=W.device)
    if gamma is None:
        gamma = torch.empty(1, dtype=torch.float32, device=W.device)
    _check(lib.bitnet_quantize_weights_sharded(wp, _FLOAT[W.dtype], N, K, fmt, sp, sums.numel() // 2, int(total_rows),
                                               _dev(packed, "packed"), _dev(gamma, "gamma", (torch.float32,)), _stream()),
           "bitnet_quantize_weights_sharded")
    return packed, gamma


def quantize_acts(x, xq=None, sx=None):
    """x [M,K] fp32/bf16 -> (x_q int8 [M,K], s_x float32 [M]); Section 2."""
    lib = load()
    xp = _dev(x, "x", _FLOAT, 2)
    M, K = x.shape
    if xq is None:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
    if sx is None:
        sx = torch.empty(M, dtype=torch.float32, device=x.device)
    _check(lib.bitnet_quantize_acts(xp, _FLOAT[x.dtype], M, K, _dev(xq, "xq", (torch.int8,)),
                                    _dev(sx, "sx", (torch.float32,)), _stream()), "bitnet_quantize_acts")
    return xq, sx


def rmsnorm_quantize(x, g=None, eps=1e-6, xq=None, sx=None):
    """RMSNorm (optional gain g [K], float32) fused with the activation quantization:
    x [M,K] fp32/bf16 -> (x_q int8 [M,K], s_x float32 [M])."""
    lib = load()
    xp = _dev(x, "x", _FLOAT, 2)
    M, K = x.shape
    if xq is None:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
    if sx is None:
        sx = torch.empty(M, dtype=torch.float32, device=x.device)
    gp = None if g is None else _dev(g, "g", (torch.float32,))
    if g is not None and tuple(g.shape) != (K,):
        raise ValueError("g must have one entry per column")
    _check(lib.bitnet_rmsnorm_quantize(xp, _FLOAT[x.dtype], gp, float(eps), M, K, _dev(xq, "xq", (torch.int8,)),
                                       _dev(sx, "sx", (torch.float32,)), _stream()), "bitnet_rmsnorm_quantize")
    return xq, sx


def swiglu_quantize(gu, hq=None, sh=None):
    """SwiGLU gating fused with the activation quantization: gu [M,2F] fp32/bf16 (gate | up) ->
    (h_q int8 [M,F], s_h float32 [M]) with h = silu(gate) * up."""
    lib = load()
    gp = _dev(gu, "gu", _FLOAT, 2)
    M, F2 = gu.shape
    if F2 % 2:
        raise ValueError("gu must have an even number of columns")
    F = F2 // 2
    if hq is None:
        hq = torch.empty((M, F), dtype=torch.int8, device=gu.device)
    if sh is None:
        sh = torch.empty(M, dtype=torch.float32, device=gu.device)
    _check(lib.bitnet_swiglu_quantize(gp, _FLOAT[gu.dtype], M, F, _dev(hq, "hq", (torch.int8,)),
                                      _dev(sh, "sh", (torch.float32,)), _stream()), "bitnet_swiglu_quantize")
    return hq, sh


def linear(xq, sx, packed, gamma, N, fmt=PACK_2BIT, y_dtype=F32, y=None, kernel=KERNEL_AUTO):
    """y [M,N] = (x_q . Wt^T) * gamma * s_x / 127 (or the raw int32 accumulator for y_dtype=I32)."""
    lib = load()
    M, K = xq.shape
    if y is None:
        y = torch.empty((M, N), dtype=_OUT[y_dtype], device=xq.device)
    args = (_dev(xq, "xq", (torch.int8,), 2), _dev(sx, "sx", (torch.float32,)), _dev(packed, "packed"),
            _dev(gamma, "gamma", (torch.float32,)), M, N, K, fmt, _dev(y, "y", (_OUT[y_dtype],)), y_dtype)
    if kernel == KERNEL_AUTO:
        _check(lib.bitnet_linear(*args, _stream()), "bitnet_linear")
    else:
        _check(lib.bitnet_linear_variant(*args, kernel, _stream()), "bitnet_linear_variant")
    return y


def linear_workspace(M, N, K, fmt=PACK_2BIT):
    """Bytes of scratch with which linear_ws can use every variant it may choose for this shape and weight format:
    split-K partials, and for 5-trit weights at more than 16 tokens the 2-bit copy of the matrix (0: none)."""
    lib = load()
    out = ctypes.c_size_t(0)
    _check(lib.bitnet_linear_workspace_format(M, N, K, fmt, ctypes.byref(out)), "bitnet_linear_workspace_format")
    return int(out.value)


def repack_weights(packed, N, K, f_in, f_out, out=None):
    """The packed matrix in the other format (device to device)."""
    lib = load()
    if out is None:
        out = torch.empty(packed_bytes(N, K, f_out), dtype=torch.uint8, device=packed.device)
    _check(lib.bitnet_repack_weights(_dev(packed, "packed"), f_in, N, K, _dev(out, "out"), f_out, _stream()),
           "bitnet_repack_weights")
    return out


def _parse_plan(text):
    f = dict(kv.split("=", 1) for kv in text.split())
    gx, gy = f["grid"].split("x")
    return {"kernel": f["kernel"], "params": [int(v) for v in f["params"].split(",") if v], "grid": (int(gx), int(gy)),
            "block": int(f["block"]), "lds": int(f["lds"]), "splits": int(f["splits"]), "repack": f.get("repack")}


def linear_describe(M, N, K, fmt=PACK_2BIT, workspace_bytes=0):
    """The kernel family and launch shape linear (or linear_ws with a workspace of that size) takes for a shape; host
    only, no device needed -> dict(kernel=str, params=[int], grid=(x, y), block=int, lds=int, splits=int, repack=str or
    None: "trit5_to_2bit" where linear_ws first repacks 5-trit weights into the workspace)."""
    lib = load()
    buf = ctypes.create_string_buffer(256)
    _check(lib.bitnet_linear_describe(M, N, K, fmt, workspace_bytes, buf, len(buf)), "bitnet_linear_describe")
    return _parse_plan(buf.value.decode())


def entry_describe(entry, M, N, K, x_dtype=BF16, fmt=PACK_2BIT, workspace_bytes=0):
    """The same for any entry point (ENTRY_*): the decode-kernel instantiation a fused call with these sizes launches.
    N and K as the entry point takes them (swiglu_linear_fused: K = F; ffn gate/up: N = F)."""
    lib = load()
    buf = ctypes.create_string_buffer(256)
    _check(lib.bitnet_entry_describe(entry, x_dtype, M, N, K, fmt, workspace_bytes, buf, len(buf)), "bitnet_entry_describe")
    return _parse_plan(buf.value.decode())


def linear_ws(xq, sx, packed, gamma, N, workspace, fmt=PACK_2BIT, y_dtype=F32, y=None, kernel=KERNEL_AUTO,
              gamma_per_block=False):
    """bitnet_linear with a scratch buffer (uint8 tensor or None) that lets the prefill kernel split K."""
    lib = load()
    M, K = xq.shape
    if y is None:
        y = torch.empty((M, N), dtype=_OUT[y_dtype], device=xq.device)
    wp = None if workspace is None else _dev(workspace, "workspace")
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.bitnet_linear_ws(_dev(xq, "xq", (torch.int8,), 2), _dev(sx, "sx", (torch.float32,)), _dev(packed, "packed"),
                                _dev(gamma, "gamma", (torch.float32,)), 1 if gamma_per_block else 0, M, N, K, fmt,
                                _dev(y, "y", (_OUT[y_dtype],)), y_dtype, kernel, wp, wb, _stream()), "bitnet_linear_ws")
    return y


def linear_fused(x, packed, gamma, N, fmt=PACK_2BIT, y_dtype=F32, y=None):
    """Decode path in one launch: activation quantization fused into the weight-streaming kernel."""
    lib = load()
    xp = _dev(x, "x", _FLOAT, 2)
    M, K = x.shape
    if y is None:
        y = torch.empty((M, N), dtype=_OUT[y_dtype], device=x.device)
    _check(lib.bitnet_linear_fused(xp, _FLOAT[x.dtype], _dev(packed, "packed"), _dev(gamma, "gamma", (torch.float32,)),
                                   M, N, K, fmt, _dev(y, "y", (_OUT[y_dtype],)), y_dtype, _stream()),
           "bitnet_linear_fused")
    return y


def quantize_weights_segmented(W, seg_rows, fmt=PACK_2BIT, packed=None, gamma_rb=None, workspace=None):
    """W [N,K] split into consecutive row segments (seg_rows, e.g. the Q, K, V parts of a merged projection),
    each quantized with its own gamma -> (packed uint8 tensor, gamma_rb float32[ceil(N/16)])."""
    lib = load()
    wp = _dev(W, "W", _FLOAT, 2)
    N, K = W.shape
    seg = (ctypes.c_int64 * len(seg_rows))(*[int(r) for r in seg_rows])
    if packed is None:
        packed = torch.empty(packed_bytes(N, K, fmt), dtype=torch.uint8, device=W.device)
    if gamma_rb is None:
        gamma_rb = torch.empty((N + 15) // 16, dtype=torch.float32, device=W.device)
    if workspace is None:
        workspace = torch.empty(quantize_weights_workspace(N, K), dtype=torch.uint8, device=W.device)
    _check(lib.bitnet_quantize_weights_segmented(wp, _FLOAT[W.dtype], N, K, len(seg_rows), seg, fmt,
                                                 _dev(packed, "packed"), _dev(gamma_rb, "gamma_rb", (torch.float32,)),
                                                 _dev(workspace, "workspace"),
                                                 workspace.numel() * workspace.element_size(), _stream()),
           "bitnet_quantize_weights_segmented")
    return packed, gamma_rb


def linear_segmented(xq, sx, packed, gamma_rb, N, fmt=PACK_2BIT, y_dtype=F32, y=None, kernel=KERNEL_AUTO):
    """bitnet_linear with one gamma per 16-row block (gamma_rb from quantize_weights_segmented)."""
    lib = load()
    M, K = xq.shape
    if y is None:
        y = torch.empty((M, N), dtype=_OUT[y_dtype], device=xq.device)
    if gamma_rb.numel() < (N + 15) // 16:
        raise ValueError("gamma_rb needs one entry per 16-row block")
    _check(lib.bitnet_linear_segmented(_dev(xq, "xq", (torch.int8,), 2), _dev(sx, "sx", (torch.float32,)),
                                       _dev(packed, "packed"), _dev(gamma_rb, "gamma_rb", (torch.float32,)), M, N, K, fmt,
                                       _dev(y, "y", (_OUT[y_dtype],)), y_dtype, kernel, _stream()),
           "bitnet_linear_segmented")
    return y


def linear_fused_segmented(x, packed, gamma_rb, N, fmt=PACK_2BIT, y_dtype=F32, y=None):
    """bitnet_linear_fused with one gamma per 16-row block."""
    lib = load()
    xp = _dev(x, "x", _FLOAT, 2)
    M, K = x.shape
    if y is None:
        y = torch.empty((M, N), dtype=_OUT[y_dtype], device=x.device)
    if gamma_rb.numel() < (N + 15) // 16:
        raise ValueError("gamma_rb needs one entry per 16-row block")
    _check(lib.bitnet_linear_fused_segmented(xp, _FLOAT[x.dtype], _dev(packed, "packed"),
                                             _dev(gamma_rb, "gamma_rb", (torch.float32,)), M, N, K, fmt,
                                             _dev(y, "y", (_OUT[y_dtype],)), y_dtype, _stream()),
           "bitnet_linear_fused_segmented")
    return y


def rmsnorm_linear_fused(x, g, eps, packed, gamma, N, fmt=PACK_2BIT, y_dtype=F32, y=None, segmented=False):
    """y = BitLinear(RMSNorm(x) * g) in one launch (decode path; g [K] float32 or None).  With segmented=True
    `gamma` holds one scale per 16-row block (from quantize_weights_segmented)."""
    lib = load()
    xp = _dev(x, "x", _FLOAT, 2)
    M, K = x.shape
    if y is None:
        y = torch.empty((M, N), dtype=_OUT[y_dtype], device=x.device)
    gp = None if g is None else _dev(g, "g", (torch.float32,))
    if g is not None and tuple(g.shape) != (K,):
        raise ValueError("g must have one entry per column")
    if segmented and gamma.numel() < (N + 15) // 16:
        raise ValueError("gamma needs one entry per 16-row block")
    fn = lib.bitnet_rmsnorm_linear_fused_segmented if segmented else lib.bitnet_rmsnorm_linear_fused
    _check(fn(xp, _FLOAT[x.dtype], gp, float(eps), _dev(packed, "packed"), _dev(gamma, "gamma", (torch.float32,)),
              M, N, K, fmt, _dev(y, "y", (_OUT[y_dtype],)), y_dtype, _stream()),
           "bitnet_rmsnorm_linear_fused_segmented" if segmented else "bitnet_rmsnorm_linear_fused")
    return y


def swiglu_linear_fused(gu, packed, gamma, N, fmt=PACK_2BIT, y_dtype=F32, y=None):
    """y = BitLinear(silu(gate) * up) in one launch (decode path): gu [M,2F] fp32/bf16 (gate | up), packed an [N,F] matrix."""
    lib = load()
    gp = _dev(gu, "gu", _FLOAT, 2)
    M, F2 = gu.shape
    if F2 % 2:
        raise ValueError("gu must hold a gate and an up half")
    if y is None:
        y = torch.empty((M, N), dtype=_OUT[y_dtype], device=gu.device)
    _check(lib.bitnet_swiglu_linear_fused(gp, _FLOAT[gu.dtype], _dev(packed, "packed"), _dev(gamma, "gamma", (torch.float32,)),
                                          M, N, F2 // 2, fmt, _dev(y, "y", (_OUT[y_dtype],)), y_dtype, _stream()),
           "bitnet_swiglu_linear_fused")
    return y


def ffn_gate_up_fused(x, packed, gamma, F, norm=False, g=None, eps=1e-6, gamma_per_block=False, fmt=PACK_2BIT,
                      h_dtype=F32, h=None):
    """h [M,F] = silu(y_gate) * y_up with [y_gate | y_up] = BitLinear(pre(x)) over a merged gate|up matrix [2F,K] in one
    decode launch; pre = RMSNorm (gain g or None, eps) when norm, else the plain absmax quantization."""
    lib = load()
    xp = _dev(x, "x", _FLOAT, 2)
    M, K = x.shape
    if h is None:
        h = torch.empty((M, F), dtype=_OUT[h_dtype], device=x.device)
    gp = None if g is None else _dev(g, "g", (torch.float32,))
    _check(lib.bitnet_ffn_gate_up_fused(xp, _FLOAT[x.dtype], 1 if norm else 0, gp, float(eps), _dev(packed, "packed"),
                                        _dev(gamma, "gamma", (torch.float32,)), 1 if gamma_per_block else 0, M, F, K, fmt,
                                        _dev(h, "h", (_OUT[h_dtype],)), h_dtype, _stream()), "bitnet_ffn_gate_up_fused")
    return h


def unpack_weights(packed, N, K, fmt=PACK_2BIT, codes=None):
    """packed -> int8 codes [N,K] in {-1,0,+1} (test helper)."""
    lib = load()
    if codes is None:
        codes = torch.empty((N, K), dtype=torch.int8, device=packed.device)
    _check(lib.bitnet_unpack_weights(_dev(packed, "packed"), N, K, fmt, _dev(codes, "codes", (torch.int8,)), _stream()),
           "bitnet_unpack_weights")
    return codes

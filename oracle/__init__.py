"""CPU oracle for the BitLinear W1.58A8 product (BitNet b1.58, arXiv 2402.17764, Section 2).

TEST INFRASTRUCTURE ONLY.  Tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; the GPU library and its Python binding never do.  The arithmetic lives in
bitnet_oracle.c (plain scalar C); this module only marshals numpy arrays into it.

Functions follow the paper's order:
    absmean_gamma      Eq. (3)
    ternarize          Eq. (1)-(2)
    quantize_weights   Eq. (1)-(3) together
    quantize_acts      Section 2, per-token absmax int8
    ternary_matmul     the integer product
    rescale            undoing gamma and s_x / 127
    bitlinear          all of it, x and W in, y out

Setting BITNET_ORACLE_LIBRARY to the path of another build of bitnet_oracle.c (the sanitized one of
oracle.build.build_oracle_sanitized) makes this module load that instead.
"""
import ctypes
import os

import numpy as np

from .build import build_oracle

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(os.environ.get("BITNET_ORACLE_LIBRARY") or build_oracle())
        i64, vp = ctypes.c_int64, ctypes.c_void_p
        lib.oracle_absmean_gamma.argtypes = [vp, i64, i64, vp, vp]
        lib.oracle_ternarize.argtypes = [vp, i64, i64, ctypes.c_float, vp]
        lib.oracle_quantize_acts.argtypes = [vp, i64, i64, vp, vp]
        lib.oracle_ternary_matmul.argtypes = [vp, vp, i64, i64, i64, vp]
        lib.oracle_rescale.argtypes = [vp, ctypes.c_float, vp, i64, i64, vp]
        lib.oracle_rmsnorm_quantize.argtypes = [vp, vp, ctypes.c_float, i64, i64, vp, vp, vp]
        lib.oracle_swiglu_quantize.argtypes = [vp, i64, i64, vp, vp, vp]
        lib.oracle_exp32.argtypes = [ctypes.c_float]
        lib.oracle_exp32.restype = ctypes.c_float
        for f in (lib.oracle_absmean_gamma, lib.oracle_ternarize, lib.oracle_quantize_acts,
                  lib.oracle_ternary_matmul, lib.oracle_rescale, lib.oracle_num_threads,
                  lib.oracle_rmsnorm_quantize, lib.oracle_swiglu_quantize):
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


_ERR = {1: "NULL pointer", 2: "non-positive size", 3: "non-finite input"}


def _check(rc, what):
    if rc != 0:
        raise ValueError("oracle %s: %s" % (what, _ERR.get(rc, "error %d" % rc)))


def _f32_2d(a, name):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if a.ndim != 2:
        raise ValueError("%s must be 2-D" % name)
    return a


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def absmean_gamma(W):
    """Eq. (3).  Returns (gamma as np.float32, fp64 sum of |W|)."""
    W = _f32_2d(W, "W")
    g = np.zeros(1, np.float32)
    s = np.zeros(1, np.float64)
    _check(_load().oracle_absmean_gamma(_ptr(W), W.shape[0], W.shape[1], _ptr(g), _ptr(s)), "absmean_gamma")
    return g[0], float(s[0])


def ternarize(W, gamma):
    """Eq. (1)-(2).  Returns int8 codes in {-1, 0, +1}, shape of W."""
    W = _f32_2d(W, "W")
    codes = np.empty(W.shape, np.int8)
    _check(_load().oracle_ternarize(_ptr(W), W.shape[0], W.shape[1], np.float32(gamma), _ptr(codes)), "ternarize")
    return codes


def quantize_weights(W):
    """Eq. (1)-(3).  Returns (codes int8 [N,K], gamma np.float32)."""
    gamma, _ = absmean_gamma(W)
    return ternarize(W, gamma), gamma


def quantize_acts(x):
    """Per-token absmax quantization.  Returns (x_q int8 [M,K], s_x float32 [M])."""
    x = _f32_2d(x, "x")
    xq = np.empty(x.shape, np.int8)
    sx = np.empty(x.shape[0], np.float32)
    _check(_load().oracle_quantize_acts(_ptr(x), x.shape[0], x.shape[1], _ptr(xq), _ptr(sx)), "quantize_acts")
    return xq, sx


def rmsnorm_quantize(x, g=None, eps=1e-6):
    """RMSNorm (optional gain g [K]) followed by per-token absmax quantization.
    Returns (x_q int8 [M,K], s_x float32 [M], z float32 [M,K] = the normalised rows)."""
    x = _f32_2d(x, "x")
    M, K = x.shape
    gp = None
    if g is not None:
        g = np.ascontiguousarray(g, dtype=np.float32)
        if g.shape != (K,):
            raise ValueError("g must have one entry per column")
        gp = _ptr(g)
    xq = np.empty((M, K), np.int8)
    sx = np.empty(M, np.float32)
    z = np.empty((M, K), np.float32)
    _check(_load().oracle_rmsnorm_quantize(_ptr(x), gp, np.float32(eps), M, K, _ptr(xq), _ptr(sx), _ptr(z)),
           "rmsnorm_quantize")
    return xq, sx, z


def exp32(t):
    """The fixed-step fp32 exponential used by swiglu_quantize."""
    return np.float32(_load().oracle_exp32(np.float32(t)))


def swiglu_quantize(gu):
    """h = silu(gu[:, :F]) * gu[:, F:] followed by per-token absmax quantization.
    Returns (h_q int8 [M,F], s_h float32 [M], h float32 [M,F])."""
    gu = _f32_2d(gu, "gu")
    M, F2 = gu.shape
    if F2 % 2:
        raise ValueError("gu must have an even number of columns")
    F = F2 // 2
    hq = np.empty((M, F), np.int8)
    sh = np.empty(M, np.float32)
    h = np.empty((M, F), np.float32)
    _check(_load().oracle_swiglu_quantize(_ptr(gu), M, F, _ptr(hq), _ptr(sh), _ptr(h)), "swiglu_quantize")
    return hq, sh, h


def ternary_matmul(xq, codes):
    """acc[m,n] = sum_k x_q[m,k] * code[n,k] as int32."""
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    if xq.ndim != 2 or codes.ndim != 2 or xq.shape[1] != codes.shape[1]:
        raise ValueError("shape mismatch: x_q %s, codes %s" % (xq.shape, codes.shape))
    M, K = xq.shape
    N = codes.shape[0]
    acc = np.empty((M, N), np.int32)
    _check(_load().oracle_ternary_matmul(_ptr(xq), _ptr(codes), M, N, K, _ptr(acc)), "ternary_matmul")
    return acc


def rescale(acc, gamma, sx):
    """y = acc * gamma * s_x / 127 in fp64."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    sx = np.ascontiguousarray(sx, dtype=np.float32)
    M, N = acc.shape
    if sx.shape != (M,):
        raise ValueError("s_x must have one entry per token")
    y = np.empty((M, N), np.float64)
    _check(_load().oracle_rescale(_ptr(acc), np.float32(gamma), _ptr(sx), M, N, _ptr(y)), "rescale")
    return y


def bitlinear(x, W):
    """The whole path.  Returns dict(codes, gamma, xq, sx, acc, y)."""
    codes, gamma = quantize_weights(W)
    xq, sx = quantize_acts(x)
    acc = ternary_matmul(xq, codes)
    return dict(codes=codes, gamma=gamma, xq=xq, sx=sx, acc=acc, y=rescale(acc, gamma, sx))

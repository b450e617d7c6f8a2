"""Decoders of the packed weight layouts, written from the format description in include/bitnet.h
(test code: numpy only, shares nothing with the kernels or the oracle)."""
import numpy as np


def quad_index_2bit(n, kq, N, K):
    """Index of the 16-byte quad that holds row n, columns 64*kq .. 64*kq+63."""
    RB = (N + 15) // 16
    Kq = (K + 63) // 64
    rb, r = divmod(n, 16)
    s, g = divmod(kq, 4)
    nq = min(4, Kq - 4 * s)
    return 64 * RB * s + 16 * nq * rb + 16 * g + r


def decode_2bit(packed_bytes, N, K):
    """bytes of a BITNET_PACK_2BIT buffer -> (codes [N,K] int8, padding_is_zero bool)."""
    Np = 16 * ((N + 15) // 16)
    Kq = (K + 63) // 64
    if isinstance(packed_bytes, (bytes, bytearray)):
        raw = bytes(packed_bytes)
    else:
        raw = np.ascontiguousarray(packed_bytes, dtype=np.uint8).tobytes()
    words = np.frombuffer(raw, dtype="<u4")
    assert words.size == Np * Kq * 4, "buffer size does not match the documented layout"
    quads = words.reshape(-1, 4)
    # gather quads into [n][kq][word]
    n_idx = np.arange(Np)[:, None]
    kq_idx = np.arange(Kq)[None, :]
    rb, r = n_idx // 16, n_idx % 16
    s, g = kq_idx // 4, kq_idx % 4
    nq = np.minimum(4, Kq - 4 * s)
    qi = 64 * (Np // 16) * s + 16 * nq * rb + 16 * g + r
    assert np.array_equal(np.sort(qi.ravel()), np.arange(Np * Kq)), "layout is not a bijection"
    by_row = quads[qi]                                        # [Np][Kq][4]
    full = np.zeros((Np, Kq, 64), np.int8)
    for j in range(4):
        for i in range(4):
            for b in range(4):
                field = (by_row[:, :, j] >> np.uint32(8 * b + 2 * i)) & np.uint32(3)
                assert not np.any(field == 2), "code 10 must never occur"
                full[:, :, 16 * j + 4 * i + b] = np.where(field == 3, -1, field.astype(np.int8))
    full = full.reshape(Np, Kq * 64)
    codes = full[:N, :K].copy()
    pad_zero = (not full[N:, :].any()) and (not full[:, K:].any())
    return codes, pad_zero


def decode_trit5(packed_bytes, N, K):
    """bytes of a BITNET_PACK_TRIT5 buffer -> (codes [N,K] int8, padding_is_zero bool)."""
    RB = (N + 15) // 16
    steps = (K + 319) // 320
    if isinstance(packed_bytes, (bytes, bytearray)):
        raw = np.frombuffer(bytes(packed_bytes), dtype=np.uint8)
    else:
        raw = np.ascontiguousarray(packed_bytes, dtype=np.uint8).ravel()
    assert raw.size == RB * 16 * steps * 320 // 5, "buffer size does not match the documented layout"
    assert raw.max() <= 242, "a byte holds five base-3 digits"
    quads = raw.reshape(steps, RB, 4, 16, 16)              # [s][rb][g][r][p]
    full = np.zeros((RB * 16, steps * 320), np.int8)
    view = full.reshape(RB, 16, steps, 4, 80)              # [rb][r][s][g][column in quad]
    v = quads.astype(np.int32)
    for d in range(5):
        digit = (v // (3 ** d)) % 3 - 1                    # [s][rb][g][r][p]
        digit = digit.transpose(1, 3, 0, 2, 4)             # [rb][r][s][g][p]
        if d < 4:
            view[:, :, :, :, d:64:4] = digit               # columns 4p + d
        else:
            view[:, :, :, :, 64:80] = digit                # columns 64 + p
    codes = full[:N, :K].copy()
    pad_zero = (not full[N:, :].any()) and (not full[:, K:].any())
    return codes, pad_zero

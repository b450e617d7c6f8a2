"""Decoders of the packed weight layouts, written from the format description in include/bitnet.h
(test code: numpy only, shares nothing with the kernels or the oracle)."""
import numpy as np


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
    # quad index ((rb*Kq + kb)*16 + r), 4 words per quad
    words = words.reshape(Np // 16, Kq, 16, 4)                 # [rb][kb][r][j]
    full = np.zeros((Np, Kq * 64), np.int8)
    for j in range(4):
        for i in range(4):
            for b in range(4):
                col = 16 * j + 4 * i + b
                field = (words[:, :, :, j] >> np.uint32(8 * b + 2 * i)) & np.uint32(3)   # [rb][kb][r]
                val = np.where(field == 3, -1, field.astype(np.int8)).astype(np.int8)
                assert not np.any(field == 2), "code 10 must never occur"
                # rows rb*16 + r, columns kb*64 + col
                full.reshape(Np // 16, 16, Kq, 64)[:, :, :, col] = val.transpose(0, 2, 1)
    codes = full[:N, :K].copy()
    pad_zero = (not full[N:, :].any()) and (not full[:, K:].any())
    return codes, pad_zero

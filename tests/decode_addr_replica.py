"""Host replica of the address arithmetic of the M <= 16 decode kernel (csrc/linear_gemv.hip, linear_gemv16_2bit): for
one launch -- template parameters, shape, launch geometry as the host code computes them -- it enumerates every
workgroup, lane and K item and returns, per buffer, the lowest and highest byte touched, so that a CPU test can hold them
against the buffer sizes.  It re-states the kernel's index expressions in numpy; it shares no code with the kernel."""
import numpy as np

HEADER = 32 * 16                     # bytes in front of the x region: reduction scratch, s_x, the RMSNorm doubles


def ceil_div(a, b):
    return -(-a // b)


class Span:
    def __init__(self):
        self.lo, self.hi = None, None

    def add(self, first, nbytes):
        first = np.asarray(first, np.int64)
        if first.size == 0:
            return
        lo, hi = int(first.min()), int(first.max()) + nbytes
        self.lo = lo if self.lo is None else min(self.lo, lo)
        self.hi = hi if self.hi is None else max(self.hi, hi)

    def within(self, size):
        return self.lo is None or (self.lo >= 0 and self.hi <= size)


def decode_launch_spans(kR, kS, kW, kD, xmode, pair, M, N, K, out_bytes=2, gstride=0):
    """N: output features (pair: F, the packed matrix has 2 F rows).  Returns (spans, sizes, lds_bytes, grid)."""
    fused = xmode >= 2
    bf16 = xmode in (2, 4, 6)
    norm, swiglu = xmode in (4, 5), xmode in (6, 7)
    Kq = ceil_div(K, 64)
    pair_off = N // 16 if pair else 0
    RB = 2 * pair_off if pair else ceil_div(N, 16)
    steps = ceil_div(Kq, 4)
    items = ceil_div(ceil_div(ceil_div(K, 256), kS), kD) * kD
    tail_quads = 16 * (Kq - 4 * (steps - 1))
    Kpad = steps * 256
    lds_fold = kW * kS * kR * 64 * 16 if kS > 1 else 0
    lds_x = M * ceil_div(K, 256) * 256
    lds = HEADER + (lds_x if (xmode != 0 and lds_x > lds_fold) else lds_fold)
    grid = ceil_div(pair_off, kW) if pair else ceil_div(RB, kW * kR)
    threads = kS * kW * 64
    esz = 2 if bf16 else 4
    kE = 8 if bf16 else 4

    sp = {k: Span() for k in ("packed", "x", "gamma", "sx", "y", "gain", "lds")}
    blk = np.arange(grid, dtype=np.int64)[:, None]
    tid = np.arange(threads, dtype=np.int64)[None, :]
    lane, wave = tid & 63, tid >> 6
    r, g = lane & 15, lane >> 4
    ws, ww = wave % kS, wave // kS
    rbw = (blk * kW + ww) if pair else (blk * kW + ww) * kR
    rbc = [(np.minimum(rbw, pair_off - 1) + a * pair_off) if pair else np.minimum(rbw + a, RB - 1) for a in range(kR)]
    mrow = np.minimum(r, M - 1)
    wstride = RB * 64
    for item in range(items):
        sl = np.minimum(ws + item * kS, steps - 1)
        cq = np.where(sl == steps - 1, tail_quads, 64)
        ln = np.minimum(lane, cq - 1)
        for a in range(kR):
            sp["packed"].add(16 * (sl * wstride + rbc[a] * cq + ln), 16)
        for j in range(4):
            if xmode == 0:
                col = np.minimum(sl * 256 + 64 * g + 16 * j, K - 16)
                sp["x"].add(mrow * K + col + 0 * blk, 16)
            else:
                sp["lds"].add(HEADER + 16 * (mrow * (Kpad >> 4) + 4 * g + sl * 16 + j) + 0 * blk, 16)
    if xmode == 1:                                              # x_q staged in LDS
        v = np.arange(M * (Kpad >> 4), dtype=np.int64)
        m, kv = v // (Kpad >> 4), v % (Kpad >> 4)
        ok = kv * 16 + 16 <= K
        sp["x"].add((m * K + kv * 16)[ok], 16)
        sp["lds"].add(HEADER + 16 * v, 16)
    if fused:
        nvec = K // kE
        row_bytes = (2 if swiglu else 1) * K * esz
        t = np.arange(threads, dtype=np.int64)
        if nvec <= 4 * threads:                                 # token 0 prefetched into registers
            for v in range(4):
                idx = np.minimum(v * threads + t, nvec - 1)
                sp["x"].add(16 * idx, 16)
                if swiglu:
                    sp["x"].add(16 * (nvec + idx), 16)
                if norm and v < (0 if threads >= 1024 else 2):
                    for h in range(2 if bf16 else 1):
                        sp["gain"].add(16 * (idx * (2 if bf16 else 1) + h), 16)
        vv = np.arange(nvec, dtype=np.int64)
        for m in range(M):
            sp["x"].add(m * row_bytes + 16 * vv, 16)
            if swiglu:
                sp["x"].add(m * row_bytes + 16 * (nvec + vv), 16)
            if norm:
                for h in range(kE // 4):
                    sp["gain"].add(4 * (vv * kE + 4 * h), 16)
            vp = np.arange(Kpad // kE, dtype=np.int64)          # real vectors and the zero padding
            words = (2 * vp[:, None] + np.arange(2)[None, :]) if bf16 else vp[:, None]
            sp["lds"].add(HEADER + 4 * (m * (Kpad >> 2) + words), 4)
        sp["lds"].add(4 * np.arange(16 + 16, dtype=np.int64), 4)                       # red[], s_x
        sp["lds"].add(128 + 8 * np.arange(2 * (threads // 64), dtype=np.int64).clip(0, 31), 8)   # the RMSNorm doubles
    if kS > 1:
        for a in range(kR):
            sp["lds"].add(HEADER + 16 * (((ww * kS + ws) * kR + a) * 64 + lane) + 0 * blk, 16)
    for a in range(kR):
        sp["gamma"].add(4 * gstride * rbc[a], 4)
    if not fused:
        sp["sx"].add(4 * mrow + 0 * blk, 4)
    for a in range(1 if pair else kR):
        n0 = (rbw if pair else rbw + a) * 16 + 4 * g
        for e in range(4):
            ok = (r < M) & (ws == 0) & (n0 + e < N)
            sp["y"].add(out_bytes * (r * N + n0 + e)[ok], out_bytes)
    rows = 2 * N if pair else N
    sizes = {"packed": 16 * ceil_div(rows, 16) * 64 * ceil_div(K, 64) // 4,
             "x": M * (2 if swiglu else 1) * K * (esz if fused else 1), "gamma": 4 * (ceil_div(rows, 16) if gstride else 1),
             "sx": 4 * M, "y": out_bytes * M * N, "gain": 4 * K, "lds": lds}
    return sp, sizes, lds, grid

"""Where the time of a decode launch goes: per-workgroup wall-clock stamps inside the M <= 16 decode kernel.

    python -m paper_2402_17764_amd.decode_timeline [70b|3b]

Builds an instrumented copy of csrc/linear_gemv.hip (the kernel source with a stamp written by thread 0 of every
workgroup at fixed points: start, absmax reduced, activations staged, K loop done, fold done, output stored) into a
library of its own under _build/, replays a HIP graph of launches over distinct weight buffers through the library's own
launch selection, and prints the distribution of each stamp over the workgroups of the last launch, in nanoseconds after
that launch's first workgroup started, next to the time per launch.  The instrumented kernel is a few percent slower
than the product kernel (the stamps are stores, and the last one waits for the output store to be acknowledged).
For tuning and for the figures quoted in the design notes; nothing in the product path uses it.
"""
import ctypes
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
BUILD = os.path.join(HERE, "_build", "timeline")
NAMES = ["start", None, "absmax reduced", "activations staged", None, "K loop done (wave 0)", "fold done", "output stored"]


def instrumented_source():
    src = open(os.path.join(HERE, "csrc", "linear_gemv.hip")).read()

    def put(anchor, text, after=True):
        nonlocal src
        assert src.count(anchor) == 1, "anchor not found once: " + anchor[:60]
        i = src.index(anchor) + (len(anchor) if after else 0)
        src = src[:i] + text + src[i:]

    put("namespace bitnet {\n", "__device__ unsigned long long g_ts[8 * 8192];\n"
        "#define TS(k_) do { __builtin_amdgcn_sched_barrier(0); if (threadIdx.x == 0 && blockIdx.x < 8192) "
        "{ g_ts[blockIdx.x * 8 + (k_)] = wall_clock64(); } __builtin_amdgcn_sched_barrier(0); } while (0)\n")
    put("    extern __shared__ uint4 smem[];\n    constexpr int kThreads = kS * kW * kWave;", "\n    TS(0);")
    put("        const float sc = block_absmax_to_scale<kThreads>(amax, red);", "\n        if (m == 0) TS(2);")
    put("    int i = 0;\n    for (; i + kD < items; i += kD) {", "    TS(3);\n", after=False)
    put("    for (int d = 0; d < kD; ++d) mac(st[d], i + d);\n\n    if (kFused && yt != OutType::I32)",
        "", after=False)
    src = src.replace("    for (int d = 0; d < kD; ++d) mac(st[d], i + d);\n\n    if (kFused && yt != OutType::I32)",
                      "    for (int d = 0; d < kD; ++d) mac(st[d], i + d);\n    asm volatile(\"\" :: \"v\"(acc[0].x));\n    TS(5);\n\n"
                      "    if (kFused && yt != OutType::I32)")
    put("            acc[a] = s;\n        }\n    }\n", "    TS(6);\n")
    tail = ("            if (n0 < N) store_row4(y, yt, (int64_t)r * N + n0, n0, N, acc[a], scale);\n        }\n    }\n}")
    assert src.count(tail) == 1
    src = src.replace(tail, tail[:-1] + "    __builtin_amdgcn_s_waitcnt(0);\n    TS(7);\n}")
    src += '''
extern "C" int timeline_linear(const void* xq, const float* sx, const void* packed, const float* gamma, long long M, long long N,
                               long long K, void* y, void* stream) {
    return (int)bitnet::launch_linear_gemv16_2bit((const int8_t*)xq, sx, packed, gamma, 0, M, N, K, y, bitnet::OutType::BF16, (hipStream_t)stream, nullptr);
}
extern "C" int timeline_linear_fused(const void* x, const void* packed, const float* gamma, long long M, long long N, long long K,
                                     void* y, void* stream) {
    return (int)bitnet::launch_linear_fused_2bit(x, true, packed, gamma, 0, M, N, K, y, bitnet::OutType::BF16, (hipStream_t)stream, nullptr);
}
extern "C" int timeline_read(void* dst, long long bytes) { return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(bitnet::g_ts), bytes); }
extern "C" int timeline_clear() {
    void* p;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(bitnet::g_ts));
    if (e != hipSuccess) return (int)e;
    return (int)hipMemset(p, 0, sizeof(unsigned long long) * 8 * 8192);
}
'''
    return src


def build():
    from paper_2402_17764_amd.build import HIPCC, FLAGS
    os.makedirs(BUILD, exist_ok=True)
    path = os.path.join(BUILD, "linear_gemv_timeline.hip")
    open(path, "w").write(instrumented_source())
    lib = os.path.join(BUILD, "libdecode_timeline.so")
    r = subprocess.run([HIPCC, *FLAGS, "-shared", path, "-o", lib], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(r.stderr)
    return lib


def run(which="70b"):
    import numpy as np
    import torch
    from paper_2402_17764_amd import binding as B
    lib = ctypes.CDLL(os.path.join(BUILD, "libdecode_timeline.so") if os.path.exists(os.path.join(BUILD, "libdecode_timeline.so")) else build())
    vp, i64 = ctypes.c_void_p, ctypes.c_longlong
    lib.timeline_linear.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, vp]
    lib.timeline_linear_fused.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp]
    lib.timeline_read.argtypes = [vp, i64]
    shapes = {"70b": [("70B gate_up", 57344, 8192), ("70B down", 8192, 28672)],
              "3b": [("3B qkv", 9600, 3200), ("3B o", 3200, 3200), ("3B gate_up", 17280, 3200), ("3B down", 3200, 8640)]}[which]
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    for (name, N, K) in shapes:
        layers = max(8, min(40, int(1.2e9 // (N * K // 4))))
        packs = []
        for _ in range(layers):
            W = torch.randn((N, K), device="cuda", generator=g) * 0.02
            packs.append(B.quantize_weights(W))
            del W
        x = torch.randn((1, K), device="cuda", generator=g).to(torch.bfloat16)
        xq, sx = B.quantize_acts(x)
        y = torch.empty((1, N), dtype=torch.bfloat16, device="cuda")
        for fused in (True, False):
            def launches(s):
                for (p, gm) in packs:
                    rc = (lib.timeline_linear_fused(x.data_ptr(), p.data_ptr(), gm.data_ptr(), 1, N, K, y.data_ptr(), s) if fused
                          else lib.timeline_linear(xq.data_ptr(), sx.data_ptr(), p.data_ptr(), gm.data_ptr(), 1, N, K, y.data_ptr(), s))
                    assert rc == 0, rc
            st = torch.cuda.Stream()
            st.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(st):
                launches(st.cuda_stream)
            torch.cuda.synchronize()
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=st):
                launches(st.cuda_stream)
            for _ in range(3):
                gr.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                gr.replay()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / (5 * layers)
            assert lib.timeline_clear() == 0
            gr.replay()
            torch.cuda.synchronize()
            buf = np.zeros(8 * 8192, dtype=np.uint64)
            assert lib.timeline_read(buf.ctypes.data, buf.nbytes) == 0
            t = buf.reshape(8192, 8).astype(np.int64)
            t = t[: int((t[:, 0] != 0).sum())]
            r = (t - t[:, 0].min()) * 10.0                              # the wall clock ticks at 100 MHz
            form = B.entry_describe(B.ENTRY_LINEAR_FUSED if fused else B.ENTRY_LINEAR, 1, N, K)
            print("%s %d -> %d, M = 1, %s, form %s: %.2f us per launch (instrumented), %d workgroups; ns after the launch's first workgroup started"
                  % (name, K, N, "bf16 x quantized in the launch" if fused else "int8 x", form["params"], us, len(t)))
            for k, nm in enumerate(NAMES):
                if nm and (t[:, k] != 0).all():
                    v = r[:, k]
                    print("   %-22s min %6.0f  p10 %6.0f  median %6.0f  p90 %6.0f  max %6.0f"
                          % (nm, v.min(), np.percentile(v, 10), np.median(v), np.percentile(v, 90), v.max()))
            sys.stdout.flush()
        del packs
        torch.cuda.empty_cache()


if __name__ == "__main__":
    build()
    run(sys.argv[1] if len(sys.argv) > 1 else "70b")

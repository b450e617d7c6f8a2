#!/usr/bin/env python3
"""Benchmark of the BitLinear W1.58A8 hot path (BitNet b1.58, arXiv 2402.17764, Section 2) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 3b_decode|7b_decode|70b_decode]

A "step" is one pass of the per-token hot path over one batch of synthetic activations: for every
layer of the workload and every projection shape, per-token int8 activation quantization, the
ternary product and the rescale (M = 1 token for the decode workloads) -- one bitnet_linear_fused
launch per product, or bitnet_quantize_acts + bitnet_linear with --unfused.  The step is captured
once into a HIP graph and replayed, the way a decode loop would run it.  Weight quantization +
packing (Eq. 1-3) happens once per layer before the timed region, as it does for inference, and is
timed separately (`weight_quant`).  The prefill GEMM (M = 2048, 13B-class shapes) is timed as its
own leg (`gemm_m2048`), batched decode (M = 1 ... 64, 7B-class shapes) as `batched_decode_7b`.  Every input is seeded and synthetic (see paper_2402_17764_amd/synth.py for the
recipe); big tensors are drawn on the device with the same distributions.

Prints ONE JSON line.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
INT8_MFMA_PEAK_TOPS = 5000.0   # MI355X dense int8 MFMA, published (5.0 POP/s)

WORKLOADS = {
    # name: (config index in synth.CONFIGS, M, layers)
    "3b_decode": (1, 1, 26),
    "7b_decode": (2, 1, 32),
    "70b_decode": (4, 1, 80),
}


def gemv_bytes(M, N, K, out_bytes=2):
    """Algorithmic bytes of one product call: packed 2-bit weights + int8 x + scales + y."""
    return N * K // 4 + M * K + 4 * M + M * N * out_bytes


def measured_traffic(N, K):
    """HBM bytes per launch of the M = 1 product on an N x K layer, from the committed rocprofv3 --pmc summary
    (profiles/hbm_traffic.json: FETCH_SIZE + WRITE_SIZE, each scaled by what the counter reads for a plain
    256 MiB copy).  None if the summary has no entry for this launch shape."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        table = json.load(f)
    for key, v in table.get("kernels", {}).items():
        if key.startswith("linear_gemv16_2bit") and v.get("N") == N and v.get("K") == K:
            return int(v["fetch_bytes"] + v["write_bytes"])
    return None


def make_acts(torch, M, K, gen, seed_channels):
    import numpy as np
    from paper_2402_17764_amd import synth
    x = torch.randn((M, K), device="cuda", generator=gen, dtype=torch.float32)
    ch = torch.from_numpy(synth.outlier_channels(K, config=seed_channels)).cuda()
    x[:, ch] *= synth.OUTLIER_SCALE
    return x.to(torch.bfloat16)


def time_graph(torch, fn, warmup, steps, stream):
    """Capture fn() (launches on the current stream) into a HIP graph; time `steps` replays."""
    with torch.cuda.stream(stream):
        fn()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        fn()
    # warm-up: at least `warmup` replays and at least 30 ms of them (clocks and caches settle over the first
    # tens of milliseconds of a new kind of load)
    t_w = time.perf_counter()
    done = 0
    while done < max(1, warmup) or time.perf_counter() - t_w < 0.030:
        graph.replay()
        done += 1
        if done % 8 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall_ms / steps, graph


def cpu_baseline(cfg_idx, M, seconds_target=12.0):
    """The oracle's per-token path (activation quantization, integer product, rescale) timed on the
    host cores for two layer sets of the workload; same algorithmic-bytes unit as the GPU value."""
    import numpy as np
    import oracle
    from paper_2402_17764_amd import synth
    cfg = synth.CONFIGS[cfg_idx]
    layers = []
    nbytes = 0
    for l in range(2):
        for t, (name, K, N) in enumerate(cfg["shapes"]):
            if N * K > 150e6:          # keep host memory and set-up time bounded
                N = N // 8
            W = synth.weights(N, K, config=cfg_idx, layer=l, tensor=t)
            codes, gamma = oracle.quantize_weights(W)
            x, _ = synth.activations(M, K, config=cfg_idx, layer=l, tensor=100 + t, bf16=True)
            layers.append((x, codes, gamma, N, K))
            nbytes += gemv_bytes(M, N, K)
            del W
    def one_pass():
        for (x, codes, gamma, N, K) in layers:
            xq, sx = oracle.quantize_acts(x)
            acc = oracle.ternary_matmul(xq, codes)
            oracle.rescale(acc, gamma, sx)
    one_pass()
    t0 = time.perf_counter()
    one_pass()
    per = time.perf_counter() - t0
    reps = max(1, min(200, int(seconds_target / max(per, 1e-6))))
    t0 = time.perf_counter()
    for _ in range(reps):
        one_pass()
    dt = (time.perf_counter() - t0) / reps
    return {
        "value": round(nbytes / dt / 1e9, 3), "unit": "GB/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": "2 layer sets of %s at M=%d (%d product calls, %.0f MB of packed-weight-equivalent bytes), "
                  "activation quantization + integer product + rescale, mean of %d passes"
                  % (cfg["name"], M, len(layers), nbytes / 1e6, reps),
    }


def large_gemv_leg(torch, B, synth, gen, stream, args):
    """The 70B-class FFN shapes (the sizes at which a weight stream can approach the HBM roofline): M = 1 with each
    shape replayed over 2.4 GB of distinct layers (a quarter of the model's 80: far beyond the 256 MB memory-side
    cache, and enough launches per graph replay that the gap between replays does not show), the M = 4096 prefill
    product, and the one-off weight quantization + packing time per layer."""
    res = {}
    for (name, K, N) in synth.CONFIGS[4]["shapes"]:
        per = N * K // 4
        layers = max(3, int(math.ceil(2.4e9 / per)))
        packs = []
        wq_ms = []
        for l in range(layers):
            W = torch.randn((N, K), device="cuda", generator=gen, dtype=torch.float32) * synth.SIGMA_W
            if l >= 1:
                torch.cuda.synchronize()
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                packs.append(B.quantize_weights(W))
                e1.record()
                torch.cuda.synchronize()
                wq_ms.append(e0.elapsed_time(e1))
            else:
                packs.append(B.quantize_weights(W))
            del W
        x = make_acts(torch, 1, K, gen, 4)
        y = torch.empty((1, N), dtype=torch.bfloat16, device="cuda")

        def run():
            for (p, g) in packs:
                B.linear_fused(x, p, g, N, y_dtype=B.BF16, y=y)

        ms, _, _ = time_graph(torch, run, args.warmup, args.steps, stream)
        us = ms * 1e3 / layers
        gbs = gemv_bytes(1, N, K) / (us * 1e-6) / 1e9
        res[name] = {"K": K, "N": N, "layers": layers, "us_per_launch": round(us, 2), "GB/s": round(gbs, 1),
                     "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                     "weight_quant_ms_per_layer": round(min(wq_ms), 3),
                     "weight_quant_GB/s": round(8.25 * N * K / (min(wq_ms) * 1e-3) / 1e9, 1)}
        # prefill on the same shape
        M = 4096
        xp = make_acts(torch, M, K, gen, 4)
        xq, sx = B.quantize_acts(xp)
        del xp
        yp = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        p0, g0 = packs[0]
        t_w = time.perf_counter()
        while time.perf_counter() - t_w < 0.030:
            B.linear(xq, sx, p0, g0, N, y_dtype=B.BF16, y=yp)
            torch.cuda.synchronize()
        iters = 5
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            B.linear(xq, sx, p0, g0, N, y_dtype=B.BF16, y=yp)
        e1.record()
        torch.cuda.synchronize()
        us_p = e0.elapsed_time(e1) * 1e3 / iters
        tops = 2.0 * M * N * K / (us_p * 1e-6) / 1e12
        res[name]["prefill_m4096"] = {"us_linear": round(us_p, 1), "TOPS": round(tops, 1),
                                      "frac_int8_mfma_peak": round(tops / INT8_MFMA_PEAK_TOPS, 4)}
        del packs, xq, sx, yp
        torch.cuda.empty_cache()
    res["ffn_chain_m1"] = large_ffn_chain(torch, B, synth, gen, stream, args)
    return res


def large_ffn_chain(torch, B, synth, gen, stream, args, layers=80):
    """One token through the feed-forward halves of all 80 layers of the 70B-class model, every layer's packed
    weights resident (14.1 GB), as one HIP graph of two launches per layer: the merged gate/up projection with
    RMSNorm + quantization in front and the SwiGLU gate in its epilogue, then the down projection with absmax
    quantization in front.  The attention half (QKV, attention, O) is not in the workload's shape list and is
    left out; residual additions likewise."""
    shapes = {name: (K, N) for (name, K, N) in synth.CONFIGS[4]["shapes"]}
    H, N_gu = shapes["gate_up"]
    F = shapes["down"][0]
    assert N_gu == 2 * F and shapes["down"][1] == H
    packs = []
    for l in range(layers):
        d = {}
        for name, (K, N) in shapes.items():
            W = torch.randn((N, K), device="cuda", generator=gen, dtype=torch.float32) * synth.SIGMA_W
            d[name] = B.quantize_weights(W)
            del W
        packs.append(d)
    x0 = make_acts(torch, 1, H, gen, 4)
    gain = torch.ones(H, dtype=torch.float32, device="cuda")
    h_f = torch.empty((1, F), dtype=torch.bfloat16, device="cuda")
    y_d = [torch.empty((1, H), dtype=torch.bfloat16, device="cuda") for _ in range(2)]

    def run():
        x = x0
        for l, d in enumerate(packs):
            B.ffn_gate_up_fused(x, d["gate_up"][0], d["gate_up"][1], F, norm=True, g=gain, eps=1e-6, h_dtype=B.BF16, h=h_f)
            B.linear_fused(h_f, d["down"][0], d["down"][1], H, y_dtype=B.BF16, y=y_d[l & 1])
            x = y_d[l & 1]

    ms, _, _ = time_graph(torch, run, args.warmup, args.steps, stream)
    nbytes = layers * sum(gemv_bytes(1, N, K) for (K, N) in shapes.values())
    out = {"layers": layers, "launches": 2 * layers, "resident_GB": round(layers * (N_gu * H + H * F) / 4 / 1e9, 2),
           "ms_per_token": round(ms, 4), "us_per_layer": round(ms * 1e3 / layers, 2),
           "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1), "frac_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
           "note": "ffn_gate_up_fused (RMSNorm in, SwiGLU out) + linear_fused(down) per layer, each layer feeding "
                   "the next; the attention half is not in this workload's shape list"}
    del packs
    torch.cuda.empty_cache()
    return out


def format_leg(torch, B, synth, gen, stream, args):
    """The 5-trits-per-byte format measured against the 2-bit one on the M = 1 product (bitnet_linear on
    pre-quantized activations), same weights, on the dominant 3B shape and the 70B gate/up shape."""
    res = {}
    for (tag, K, N) in (("3b_gate_up", 3200, 17280), ("70b_gate_up", 8192, 57344)):
        entry = {"K": K, "N": N}
        x = make_acts(torch, 1, K, gen, 1)
        xq, sx = B.quantize_acts(x)
        y = torch.empty((1, N), dtype=torch.bfloat16, device="cuda")
        for (fname, fmt) in (("2bit", B.PACK_2BIT), ("trit5", B.PACK_TRIT5)):
            per = B.packed_bytes(N, K, fmt)
            layers = max(3, int(math.ceil(600e6 / per)))
            g2 = torch.Generator(device="cuda")
            g2.manual_seed(1234)
            packs = []
            for l in range(layers):
                W = torch.randn((N, K), device="cuda", generator=g2, dtype=torch.float32) * synth.SIGMA_W
                packs.append(B.quantize_weights(W, fmt=fmt))
                del W

            def run():
                for (p, g) in packs:
                    B.linear(xq, sx, p, g, N, fmt=fmt, y_dtype=B.BF16, y=y)

            ms, _, _ = time_graph(torch, run, args.warmup, args.steps, stream)
            us = ms * 1e3 / layers
            entry[fname] = {"packed_bytes": per, "us_per_launch": round(us, 2), "GB/s": round(per / (us * 1e-6) / 1e9, 1)}
            del packs
            torch.cuda.empty_cache()
        entry["time_ratio_trit5_over_2bit"] = round(entry["trit5"]["us_per_launch"] / entry["2bit"]["us_per_launch"], 3)
        res[tag] = entry
    return res


def batched_decode_leg(torch, B, synth, gen, stream, args):
    """The transition between decode and prefill: M = 1 ... 64 tokens (and 128, the first prefill-kernel size) on the
    7B-class shapes, bitnet_linear on pre-quantized activations, each shape replayed over enough distinct layers to exceed the memory-side
    cache.  Both rooflines are reported because M = 64 sits near the ridge between them."""
    res = {}
    for (name, K, N) in synth.CONFIGS[2]["shapes"]:
        per = N * K // 4
        layers = max(3, int(math.ceil(550e6 / per)))
        packs = []
        for l in range(layers):
            W = torch.randn((N, K), device="cuda", generator=gen, dtype=torch.float32) * synth.SIGMA_W
            packs.append(B.quantize_weights(W))
            del W
        entry = {"K": K, "N": N, "layers": layers}
        for M in (1, 8, 16, 32, 64):
            x = make_acts(torch, M, K, gen, 2)
            xq, sx = B.quantize_acts(x)
            y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")

            def run():
                for (p, g) in packs:
                    B.linear(xq, sx, p, g, N, y_dtype=B.BF16, y=y)

            ms, _, graph = time_graph(torch, run, max(2, args.warmup // 5), max(5, args.steps // 5), stream)
            us = ms * 1e3 / layers
            entry["M=%d" % M] = {"us_per_launch": round(us, 2),
                                 "GB/s": round(gemv_bytes(M, N, K) / (us * 1e-6) / 1e9, 1),
                                 "TOPS": round(2.0 * M * N * K / us * 1e-6, 1)}
            del graph
        # the serving regime just above 64 tokens: small layers still run the token-tiled decode kernels, the others
        # the prefill kernel, timed without and with a split-K workspace (bitnet_linear_ws)
        for M in (128, 256):
            x = make_acts(torch, M, K, gen, 2)
            xq, sx = B.quantize_acts(x)
            y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
            ws = torch.empty(max(16, B.linear_workspace(M, N, K)), dtype=torch.uint8, device="cuda")

            def run_plain():
                for (p, g) in packs:
                    B.linear(xq, sx, p, g, N, y_dtype=B.BF16, y=y)

            def run_ws():
                for (p, g) in packs:
                    B.linear_ws(xq, sx, p, g, N, ws, y_dtype=B.BF16, y=y)

            ms_p, _, g1 = time_graph(torch, run_plain, max(2, args.warmup // 5), max(5, args.steps // 5), stream)
            ms_w, _, g2 = time_graph(torch, run_ws, max(2, args.warmup // 5), max(5, args.steps // 5), stream)
            entry["M=%d" % M] = {"us_per_launch": round(ms_p * 1e3 / layers, 2), "us_with_workspace": round(ms_w * 1e3 / layers, 2),
                                 "TOPS": round(2.0 * M * N * K / (min(ms_p, ms_w) * 1e3 / layers) * 1e-6, 1),
                                 "kernel": B.linear_describe(M, N, K)["kernel"]}
            del g1, g2
        res[name] = entry
        del packs
        torch.cuda.empty_cache()
    return res


def decoder_block_leg(torch, B, synth, gen, stream, args, cfg_idx=1, layers=26):
    """Per-token latency of the BitLinear chain of a decoder stack at M = 1, two ways, each one HIP graph:
    "fused": RMSNorm+quantization fused into the QKV and gate/up launches, the SwiGLU gate into the epilogue of the
    gate/up launch, absmax quantization into the O and down launches -- four launches per layer;
    "handover": int8 activations handed from producer to product -- RMSNorm->int8, QKV, quantize, O, RMSNorm->int8,
    gate/up, SwiGLU->int8, down -- eight launches per layer.
    Attention itself and the residual additions are not part of the path and are left out (the attention output
    buffer is quantized as it would arrive)."""
    cfg = synth.CONFIGS[cfg_idx]
    shapes = {name: (K, N) for (name, K, N) in cfg["shapes"]}
    H = shapes["qkv"][0]
    F = shapes["down"][0]
    packs = []
    for l in range(layers):
        d = {}
        for name, (K, N) in shapes.items():
            W = torch.randn((N, K), device="cuda", generator=gen, dtype=torch.float32) * synth.SIGMA_W
            d[name] = B.quantize_weights(W)
            del W
        packs.append(d)
    M = 1
    h = make_acts(torch, M, H, gen, cfg_idx)
    att = make_acts(torch, M, H, gen, cfg_idx)
    gain = torch.ones(H, dtype=torch.float32, device="cuda")
    xq_h = torch.empty((M, H), dtype=torch.int8, device="cuda")
    xq_f = torch.empty((M, F), dtype=torch.int8, device="cuda")
    s1 = torch.empty(M, dtype=torch.float32, device="cuda")
    y_qkv = torch.empty((M, shapes["qkv"][1]), dtype=torch.bfloat16, device="cuda")
    y_o = torch.empty((M, H), dtype=torch.bfloat16, device="cuda")
    y_gu = torch.empty((M, 2 * F), dtype=torch.bfloat16, device="cuda")
    y_d = torch.empty((M, H), dtype=torch.bfloat16, device="cuda")
    h_f = torch.empty((M, F), dtype=torch.bfloat16, device="cuda")

    def run_handover():
        x = h
        for d in packs:
            B.rmsnorm_quantize(x, gain, 1e-6, xq=xq_h, sx=s1)
            B.linear(xq_h, s1, d["qkv"][0], d["qkv"][1], shapes["qkv"][1], y_dtype=B.BF16, y=y_qkv)
            B.quantize_acts(att, xq=xq_h, sx=s1)
            B.linear(xq_h, s1, d["o"][0], d["o"][1], H, y_dtype=B.BF16, y=y_o)
            B.rmsnorm_quantize(y_o, gain, 1e-6, xq=xq_h, sx=s1)
            B.linear(xq_h, s1, d["gate_up"][0], d["gate_up"][1], 2 * F, y_dtype=B.BF16, y=y_gu)
            B.swiglu_quantize(y_gu, hq=xq_f, sh=s1)
            B.linear(xq_f, s1, d["down"][0], d["down"][1], H, y_dtype=B.BF16, y=y_d)
            x = y_d

    def run_fused():
        x = h
        for d in packs:
            B.rmsnorm_linear_fused(x, gain, 1e-6, d["qkv"][0], d["qkv"][1], shapes["qkv"][1], y_dtype=B.BF16, y=y_qkv)
            B.linear_fused(att, d["o"][0], d["o"][1], H, y_dtype=B.BF16, y=y_o)
            B.ffn_gate_up_fused(y_o, d["gate_up"][0], d["gate_up"][1], F, norm=True, g=gain, eps=1e-6, h_dtype=B.BF16, h=h_f)
            B.linear_fused(h_f, d["down"][0], d["down"][1], H, y_dtype=B.BF16, y=y_d)
            x = y_d

    ms_f, _, _ = time_graph(torch, run_fused, args.warmup, args.steps, stream)
    ms_h, _, _ = time_graph(torch, run_handover, args.warmup, args.steps, stream)
    nbytes = layers * sum(gemv_bytes(M, N, K) for (K, N) in shapes.values())
    return {"model": cfg["name"], "layers": layers, "launches": 4 * layers, "ms_per_token": round(ms_f, 4),
            "GB/s": round(nbytes / (ms_f * 1e-3) / 1e9, 1),
            "note": "rmsnorm_linear_fused(qkv), linear_fused(o), ffn_gate_up_fused (RMSNorm in, SwiGLU out), "
                    "linear_fused(down) per layer; attention and residual adds excluded",
            "int8_handover": {"launches": 8 * layers, "ms_per_token": round(ms_h, 4),
                              "note": "rmsnorm_quantize, linear(qkv), quantize_acts, linear(o), rmsnorm_quantize, "
                                      "linear(gate_up), swiglu_quantize, linear(down) per layer"}}


def gemm_leg(torch, B, synth, gen, args, M=2048):
    """Prefill: M = 2048 tokens on the 13B-class shapes, bitnet_quantize_acts + bitnet_linear (MFMA kernel)."""
    res = {"M": M, "shapes": {}}
    tot_ops, tot_us = 0.0, 0.0
    for (name, K, N) in synth.CONFIGS[3]["shapes"]:
        W = torch.randn((N, K), device="cuda", generator=gen, dtype=torch.float32) * synth.SIGMA_W
        p, g = B.quantize_weights(W)
        del W
        x = make_acts(torch, M, K, gen, 3)
        xq, sx = B.quantize_acts(x)
        y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        iters = max(5, args.steps // 2)
        t_w = time.perf_counter()                    # clocks settle over the first tens of milliseconds of MFMA load
        done = 0
        while done < max(3, args.warmup) or time.perf_counter() - t_w < 0.030:
            B.linear(xq, sx, p, g, N, y_dtype=B.BF16, y=y)
            done += 1
            if done % 8 == 0:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            B.linear(xq, sx, p, g, N, y_dtype=B.BF16, y=y)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / iters
        e0.record()
        for _ in range(iters):
            B.quantize_acts(x, xq=xq, sx=sx)
        e1.record()
        torch.cuda.synchronize()
        us_q = e0.elapsed_time(e1) * 1e3 / iters
        ops = 2.0 * M * N * K
        res["shapes"][name] = {"K": K, "N": N, "us_linear": round(us, 1), "us_quantize_acts": round(us_q, 1),
                               "TOPS": round(ops / us * 1e-6, 1), "frac_int8_mfma_peak": round(ops / us * 1e-6 / INT8_MFMA_PEAK_TOPS, 4)}
        tot_ops += ops
        tot_us += us
        del p, x, xq, y
        torch.cuda.empty_cache()
    res["TOPS"] = round(tot_ops / tot_us * 1e-6, 1)
    res["roofline"] = {"bound": "mfma", "kernel": "linear_gemm_2bit", "achieved": round(tot_ops / tot_us * 1e-6, 1),
                       "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s", "frac": round(tot_ops / tot_us * 1e-6 / INT8_MFMA_PEAK_TOPS, 4)}
    return res


def run_leg_in_child(leg, args):
    """One extra leg in a child process (this process keeps its GPU context and waits)."""
    import subprocess
    cmd = [sys.executable, os.path.abspath(__file__), "--only", leg, "--steps", str(args.steps), "--warmup", str(args.warmup)]
    try:
        r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    except subprocess.TimeoutExpired:
        return {"error": "timed out"}
    for line in reversed(r.stdout.strip().splitlines()):
        if line.startswith("{"):
            try:
                return json.loads(line)[leg]
            except (ValueError, KeyError):
                break
    return {"error": "exit code %d: %s" % (r.returncode, r.stderr.strip()[-300:])}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="3b_decode", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--unfused", action="store_true",
                    help="two launches per product (bitnet_quantize_acts + bitnet_linear) instead of bitnet_linear_fused")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (torch copy_) three times, so that a rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE run of this command contains a kernel of known traffic to scale by")
    ap.add_argument("--no-extras", action="store_true", help="skip the weight_quant and large-shape legs")
    ap.add_argument("--inprocess", action="store_true",
                    help="run the extra legs inside this process (one process for a profiler to follow); by default "
                         "each runs in a child process, so that a failure there cannot take the headline line with it")
    ap.add_argument("--only", default=None,
                    choices=["gemm_m2048", "gemv_70b_m1", "batched_decode_7b", "trit5_vs_2bit_m1", "decoder_chain_3b_m1"],
                    help="run one of the extra legs alone and print only its result (profiling a single kernel family)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the hot path is a single-GPU kernel; it would shard along "
              "the output features with no collective on the path); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2402_17764_amd import binding as B
    from paper_2402_17764_amd import synth
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    B.load()

    if args.pmc_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cfg_idx, M, L = WORKLOADS[args.workload]
    cfg = synth.CONFIGS[cfg_idx]
    shapes = cfg["shapes"]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(240217764)

    if args.only:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        legs = {"gemm_m2048": lambda: gemm_leg(torch, B, synth, gen, args),
                "gemv_70b_m1": lambda: large_gemv_leg(torch, B, synth, gen, side, args),
                "batched_decode_7b": lambda: batched_decode_leg(torch, B, synth, gen, side, args),
                "trit5_vs_2bit_m1": lambda: format_leg(torch, B, synth, gen, side, args),
                "decoder_chain_3b_m1": lambda: decoder_block_leg(torch, B, synth, gen, side, args)}
        print(json.dumps({"only": args.only, "steps": args.steps, "warmup": args.warmup, args.only: legs[args.only]()}))
        return

    # ---- weights: draw, quantize + pack through the library (timed per call with events) ----------
    packed, wq_ms, wq_bytes = {}, 0.0, 0
    ws_bytes = max(B.quantize_weights_workspace(N, K) for (_, K, N) in shapes)
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    for l in range(L):
        for (name, K, N) in shapes:
            W = torch.randn((N, K), device="cuda", generator=gen, dtype=torch.float32) * synth.SIGMA_W
            if l == 0:
                B.quantize_weights(W, workspace=workspace)          # warm the code path
                torch.cuda.synchronize()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            packed[(l, name)] = B.quantize_weights(W, workspace=workspace)
            e1.record()
            torch.cuda.synchronize()
            wq_ms += e0.elapsed_time(e1)
            wq_bytes += int(N * K * 8.25)
            del W
    acts = {K: make_acts(torch, M, K, gen, cfg_idx) for K in sorted({K for (_, K, _) in shapes})}
    xq = {K: torch.empty((M, K), dtype=torch.int8, device="cuda") for K in acts}
    sx = {K: torch.empty(M, dtype=torch.float32, device="cuda") for K in acts}
    ys = {name: torch.empty((M, N), dtype=torch.bfloat16, device="cuda") for (name, K, N) in shapes}

    def step():
        for l in range(L):
            for (name, K, N) in shapes:
                p, g = packed[(l, name)]
                if args.unfused:
                    B.quantize_acts(acts[K], xq=xq[K], sx=sx[K])
                    B.linear(xq[K], sx[K], p, g, N, y_dtype=B.BF16, y=ys[name])
                else:
                    B.linear_fused(acts[K], p, g, N, y_dtype=B.BF16, y=ys[name])

    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    ms_per_step, wall_ms, _ = time_graph(torch, step, args.warmup, args.steps, stream)
    step_bytes = L * sum(gemv_bytes(M, N, K) for (_, K, N) in shapes)
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- roofline of the dominant kernel: the product on the shape that moves the most bytes --------
    dom = max(shapes, key=lambda s: s[1] * s[2])
    dname, dK, dN = dom
    B.quantize_acts(acts[dK], xq=xq[dK], sx=sx[dK])

    def dom_only():
        for l in range(L):
            p, g = packed[(l, dname)]
            if args.unfused:
                B.linear(xq[dK], sx[dK], p, g, dN, y_dtype=B.BF16, y=ys[dname])
            else:
                B.linear_fused(acts[dK], p, g, dN, y_dtype=B.BF16, y=ys[dname])

    dom_ms, _, _ = time_graph(torch, dom_only, args.warmup, args.steps, stream)
    dom_us = dom_ms * 1e3 / L
    dom_bytes = gemv_bytes(M, dN, dK)
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9
    roofline = {
        "bound": "hbm", "kernel": "linear_gemv16_2bit", "shape": "%s K=%d N=%d M=%d" % (dname, dK, dN, M),
        "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
        "bytes_per_launch": dom_bytes, "us_per_launch": round(dom_us, 3), "traffic": measured_traffic(dN, dK),
    }

    out = {
        "metric": "BitLinear GEMV GB/s (%HBM peak) @M=1", "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8xint2->int32",
        "data": "synthetic",
        "config": {"workload": "%s: %s, M=%d, %d layer sets x %s, bf16 in/out, 2-bit packed weights"
                               % (args.workload, cfg["name"], M, L, [(n, k, nn) for (n, k, nn) in shapes]),
                   "launch": "HIP graph replay of %d x %s" % (L * len(shapes), "(bitnet_quantize_acts + bitnet_linear)"
                                                                if args.unfused else "bitnet_linear_fused"),
                   "bytes_per_step": step_bytes},
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "roofline": roofline,
    }

    if not args.no_extras:
        out["weight_quant"] = {"ms_per_pass": round(wq_ms, 3), "tensors": L * len(shapes),
                               "GB/s": round(wq_bytes / (wq_ms * 1e-3) / 1e9, 1),
                               "note": "quantize + pack of every layer, 8.25 algorithmic bytes per weight"}
        del packed, acts
        torch.cuda.empty_cache()
        legs = ["gemv_70b_m1", "gemm_m2048", "batched_decode_7b", "trit5_vs_2bit_m1", "decoder_chain_3b_m1"]
        if args.pmc_calibration:
            # under counter collection the 208-launch decoder chain is left out: one such run ended in a hardware
            # exception inside the profiler's queue that no un-profiled or kernel-trace run of the leg shows
            legs.remove("decoder_chain_3b_m1")
        inproc = {"gemv_70b_m1": lambda: large_gemv_leg(torch, B, synth, gen, stream, args),
                  "gemm_m2048": lambda: gemm_leg(torch, B, synth, gen, args),
                  "batched_decode_7b": lambda: batched_decode_leg(torch, B, synth, gen, stream, args),
                  "trit5_vs_2bit_m1": lambda: format_leg(torch, B, synth, gen, stream, args),
                  "decoder_chain_3b_m1": lambda: decoder_block_leg(torch, B, synth, gen, stream, args)}
        for leg in legs:
            if args.inprocess:
                out[leg] = inproc[leg]()
            else:
                out[leg] = run_leg_in_child(leg, args)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg_idx, M)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

"""What a launch that only reads the packed weights would take: the floor under the M = 1 decode launches.

    python -m paper_2402_17764_amd.read_floor

Uses a plain streaming-read kernel (csrc/floors.hip: 128-bit loads with the streaming cache policy, nothing else; a
library of its own next to the BitLinear one), and for each decode layer of the benchmark's configurations replays a HIP graph of back-to-back
launches over distinct buffers of the layer's packed size -- the same way bench.py times the product -- for nine launch
shapes (256 / 512 / 1024 workgroups of 512 threads x 2 / 4 / 8 loads in flight per thread), printing the fastest next to
the product launches (bitnet_linear_fused on bf16 x, bitnet_linear on int8 x) timed in the same run.  The HBM peak is a
rate; a launch of a few megabytes also pays for starting and ending, and this is how much of that no kernel avoids.
For the figures quoted in the design notes; nothing in the product path uses it.
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

def time_graph(torch, run, layers, replays=5):
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        run(st.cuda_stream)
    torch.cuda.synchronize()
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gr, stream=st):
        run(torch.cuda.current_stream().cuda_stream)
    for _ in range(3):
        gr.replay()
    torch.cuda.synchronize()
    best = 1e9
    for _ in range(3):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(replays):
            gr.replay()
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) * 1e3 / (replays * layers))
    return best


def main():
    import torch
    from paper_2402_17764_amd import binding as B
    from paper_2402_17764_amd import floors, synth
    lib = floors.load()
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1)
    print("M = 1, microseconds per launch inside a HIP graph of back-to-back launches over distinct buffers (total > 600 MB):")
    print("%-34s %10s %14s %22s %12s %12s %s" % ("layer", "packed MB", "plain read us", "(TB/s; blocks x loads)", "fused us", "int8 us", "read / fused"))
    for ci in (1, 2, 4):
        cfg = synth.CONFIGS[ci]
        for (name, K, N) in cfg["shapes"]:
            nbytes = N * K // 4
            layers = max(3, min(64, int(2.4e9 // nbytes)))
            packs = []
            for _ in range(layers):
                W = torch.randn((N, K), device="cuda", generator=gen, dtype=torch.float32) * synth.SIGMA_W
                packs.append(B.quantize_weights(W))
                del W
            res = []
            for (blocks, unroll) in floors.READ_SHAPES:
                def run(s):
                    for (p, _) in packs:
                        lib.read_only_launch(p.data_ptr(), nbytes, sink.data_ptr(), blocks, unroll, s)
                res.append((time_graph(torch, run, layers), blocks, unroll))
            res.sort()
            x = torch.randn((1, K), device="cuda", generator=gen, dtype=torch.float32).to(torch.bfloat16)
            xq, sx = B.quantize_acts(x)
            y = torch.empty((1, N), dtype=torch.bfloat16, device="cuda")

            def run_fused(s):                     # the binding launches on torch's current stream, which is s here
                for (p, g) in packs:
                    B.linear_fused(x, p, g, N, y_dtype=B.BF16, y=y)

            def run_int8(s):
                for (p, g) in packs:
                    B.linear(xq, sx, p, g, N, y_dtype=B.BF16, y=y)

            uf = time_graph(torch, run_fused, layers)
            ui = time_graph(torch, run_int8, layers)
            print("%-34s %10.1f %14.2f %22s %12.2f %12.2f %11.0f %%" % (
                "%s %s %d->%d" % (cfg["name"].split()[0], name, K, N), nbytes / 1e6, res[0][0],
                "(%.2f; %d x %d)" % (nbytes / res[0][0] / 1e6, res[0][1], res[0][2]), uf, ui, 100.0 * res[0][0] / uf), flush=True)
            del packs
            torch.cuda.empty_cache()


if __name__ == "__main__":
    main()

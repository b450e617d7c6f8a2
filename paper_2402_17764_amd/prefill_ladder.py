"""What each ingredient of the prefill kernel's K loop costs the matrix pipe.

    python -m paper_2402_17764_amd.prefill_ladder

Times csrc/prefill_ladder.hip: a loop of v_mfma_i32_32x32x32_i8 on eight accumulator fragments per wave (two workgroups of
four waves per CU, as the 128 x 256 tile of the prefill kernel), to which the loop's other ingredients are added one at
a time -- the barrier per K step, the decode arithmetic, the LDS operand reads, the weight loads from global memory, the
LDS-DMA copies of the activations -- on operand data like the benchmark's (absmax-quantized activations with outlier
channels, ternary codes x 64).  For every rung: operations per second, the shader clock measured inside the kernel, and
the share of that clock's cycles the matrix pipe was issuing (rate / (5.0 POP/s x clock / 2.4 GHz)).
For the figures quoted in the design notes; nothing in the product path uses it.
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

RUNGS = [(0, "MFMAs only"), (1, "+ barrier per 64 MFMAs"), (2, "+ decode arithmetic (2 instructions per MFMA)"),
         (3, "+ LDS operand reads (4 x 16 B per lane per 8 MFMAs)"),
         (4, "+ weight loads, 4 x 16 B per lane and step, streaming through the L2"),
         (5, "+ LDS-DMA copies, 8 KiB per wave and step, streaming: the product's K loop"),
         (6, "as the last but one, the loads at the same addresses every step"),
         (7, "as the last but one, loads and copies at the same addresses every step"),
         (8, "MFMAs + barrier + the streaming weight loads alone"), (9, "MFMAs + barrier + the streaming LDS-DMA copies alone")]


def main():
    import torch
    from paper_2402_17764_amd import floors, synth
    lib = floors.load()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1)
    n = 1 << 24
    x = torch.randn(n, device="cuda", generator=gen)
    x = torch.where(torch.rand(n, device="cuda", generator=gen) < synth.OUTLIER_FRACTION, x * synth.OUTLIER_SCALE, x)
    xq = torch.clamp(torch.round(x * (127.0 / 70.0)), -127, 127).to(torch.int8)          # an absmax of about 70 with the outliers
    w = torch.randn(n, device="cuda", generator=gen)
    codes = (torch.clamp(torch.round(w / 0.798), -1, 1) * 64).to(torch.int8)            # absmean of a unit Gaussian
    stream_src = torch.randint(0, 2 ** 31 - 1, (64 << 20,), dtype=torch.int32, device="cuda")   # 256 MiB
    out = torch.zeros(4, dtype=torch.int32, device="cuda")
    blocks, steps = 512, 2000
    ops = blocks * 4.0 * steps * 64 * 65536
    s = torch.cuda.current_stream().cuda_stream
    print("%-78s %9s %9s %10s" % ("rung (512 workgroups x 4 waves, 2000 steps of 64 MFMAs per wave)", "TOP/s", "clock GHz", "pipe busy"))
    for rung, name in RUNGS:
        best, clock = None, 0.0
        for _ in range(3):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            rc = lib.prefill_ladder_launch(rung, xq.data_ptr(), codes.data_ptr(), n, blocks, steps, stream_src.data_ptr(),
                                           stream_src.numel() * 4, out.data_ptr(), s)
            e1.record()
            torch.cuda.synchronize()
            assert rc == 0, rc
            ms = e0.elapsed_time(e1)
            if best is None or ms < best:
                o = out.cpu().numpy()
                best, clock = ms, o[1] / max(1, o[2]) * 0.1
        tops = ops / (best * 1e-3) / 1e12
        print("%-78s %9.0f %9.2f %9.0f %%" % (name, tops, clock, 100.0 * tops / (5000.0 * clock / 2.4)), flush=True)
    # the rate at which the L2s feed the CUs when nothing else happens: 512 workgroups of 256 threads read a 2 MiB buffer
    # (resident in every XCD's L2) over and over, each from a place of its own
    print()
    buf = torch.randint(0, 2 ** 31 - 1, (2 << 18,), dtype=torch.int32, device="cuda")        # 2 MiB
    reps = 400
    for to_lds, name in ((0, "plain 16-byte loads into registers"), (1, "LDS-DMA copies (16 bytes per lane) into LDS")):
        best = None
        for _ in range(3):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            rc = lib.l2_read_launch(buf.data_ptr(), buf.numel() * 4, reps, blocks, to_lds, out.data_ptr(), s)
            e1.record()
            torch.cuda.synchronize()
            assert rc == 0, rc
            ms = e0.elapsed_time(e1)
            best = ms if best is None or ms < best else best
        tbs = blocks * reps * buf.numel() * 4.0 / (best * 1e-3) / 1e12
        print("L2 -> CU, %-46s %6.1f TB/s over 256 CUs = %5.1f bytes per clock and CU at 2.1 GHz" % (name + ":", tbs, tbs * 1e12 / 256 / 2.1e9), flush=True)
    print("the prefill kernel's 128 x 256 tile takes 48 KB through this path per 8.39 M multiply-adds: 175 multiply-adds per byte")


if __name__ == "__main__":
    main()

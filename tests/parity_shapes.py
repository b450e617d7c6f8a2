"""Shape lists of the GPU parity tests (tests/test_gpu_parity.py), kept apart from them so that a CPU test can
enumerate which kernel instantiations they reach (tests/test_dispatch_cpu.py) without a GPU.  Each tuple is (M, N, K)
unless its comment says otherwise; every case is compared with the CPU oracle element by element."""

GEMV_SHAPES = [(1, 4096, 1536), (16, 4096, 1536), (1, 16, 64), (1, 17, 16), (3, 100, 80), (7, 250, 1040),
               (16, 33, 4112), (17, 70, 528), (32, 1000, 3200), (33, 130, 272), (64, 96, 1024), (50, 49, 2064),
               # one shape per branch of the kernel-selection heuristic (row blocks x K steps)
               (2, 32800, 528), (3, 16400, 4112), (1, 16400, 272), (5, 6416, 16400), (4, 6416, 1040),
               (2, 100, 6160), (16, 1000, 8192), (1, 600, 16400), (1, 100, 11008), (8, 300, 2048), (6, 16400, 512),
               (12, 16400, 8192),
               # the skinny kernel: 16 < M <= 64, ragged token tiles, every branch of its selection (row blocks
               # below 512, below 1280, above; up to 32 tokens and above), K tails, K steps from 1 to 17 and
               # fewer steps than K groups
               (20, 16400, 272), (48, 300, 4112), (64, 100, 1040), (40, 1000, 528), (33, 260, 2048), (56, 16400, 512),
               (24, 20488, 272), (50, 20500, 528), (35, 48, 64), (18, 20, 16), (64, 8200, 4096),
               # ... and its single-token-tile form for 4 < M <= 16, one shape per row-block class
               (9, 9000, 528), (10, 32800, 272), (5, 40, 16), (13, 16400, 1040),
               # ... and the form with a loader wave (many row blocks, more than 16 tokens): each of its five selections,
               # K from one partial step to 33 steps
               (30, 32784, 272), (60, 32800, 144), (17, 20490, 80), (64, 20480, 8208), (40, 8200, 1040),
               # ... two and eight row blocks per workgroup (257 ... 512 and 1537 ... 2047 row blocks) at every token tile
               (9, 5000, 528), (12, 5008, 8208), (20, 6000, 272), (50, 8000, 1040), (9, 26000, 272), (30, 28000, 144), (64, 30000, 528),
               # M <= 4: depth 5 where depth 4 would pad (34 K steps over four waves), two row blocks per wave from 512
               # row blocks on with more than one token
               (2, 100, 8640), (3, 9000, 3200),
               # one token on the 3B QKV and gate/up layers at their exact sizes: four K-split waves on x_q staged in LDS
               (1, 9600, 3200), (1, 17280, 3200),
               # 65 ... 256 tokens on small layers: token tiles of 32 and of 64 over grid z, ragged last tiles, every
               # form such launches can pick
               (65, 40, 528), (96, 300, 2064), (100, 4000, 1040), (128, 6000, 272), (130, 8000, 528), (192, 3200, 784),
               (200, 5120, 528), (250, 8000, 272), (256, 4096, 1296), (128, 12000, 144),
               # ... and up to 512 tokens where K >= 5120
               (300, 3200, 5136), (512, 4096, 5120), (400, 2000, 5392)]

FUSED_SHAPES = [(1, 4096, 1536), (16, 4096, 1536), (1, 17, 16), (3, 100, 80), (7, 250, 1040), (2, 32800, 528),
                (3, 16400, 4112), (1, 16400, 272), (4, 6416, 1040), (2, 100, 6160), (1, 3200, 8640), (1, 17280, 3200),
                (1, 600, 16400), (1, 100, 11008), (2, 64, 28672),
                # the attention projections of the 3B and 7B decode workloads at their exact sizes (13 and 16 K steps on
                # 200 ... 768 row blocks: four K-split waves on one row block), and two and four tokens on them
                (1, 9600, 3200), (1, 3200, 3200), (1, 12288, 4096), (1, 4096, 4096), (2, 9600, 3200), (4, 3200, 3200),
                # 2048 row blocks and more with 32 K steps and more: depth 3 with two extra steps requested up front
                # (ragged rows, a partial 33rd step)
                (2, 32816, 8208),
                # eight tokens and more: the forms with more row blocks per workgroup (1024 row blocks and more; 385 ... 1023;
                # fewer), ragged and at the 3B / 7B / 13B sizes, K beyond the wave-per-token quantizer's 4096 included
                (8, 16400, 528), (16, 17280, 3200), (9, 6160, 272), (16, 9600, 3200), (8, 12288, 4096), (16, 3200, 3200),
                (12, 5120, 5120),
                # three and four tokens of rows too long for one wave per token: quantized one after the other
                (4, 300, 8640), (3, 4096, 11008)]

NORM_FUSED_SHAPES = [(1, 4096, 1536), (1, 100, 3200), (3, 250, 1040), (1, 33, 4112), (16, 70, 528), (1, 16400, 272),
                     (2, 16400, 4112), (1, 600, 16400), (1, 6416, 8640), (4, 300, 8192), (1, 32800, 528), (5, 40, 16)]

SWIGLU_FUSED_SHAPES = [(1, 3200, 8640), (1, 100, 1536), (3, 250, 1040), (1, 33, 4112), (16, 70, 528), (1, 16400, 272),
                       (2, 6416, 4112), (1, 64, 28672), (1, 4096, 11008), (4, 300, 8192), (1, 32800, 528), (5, 40, 16)]

GEMM_SHAPES = [(65, 300, 528), (128, 256, 256), (100, 40, 16), (300, 520, 1040), (257, 1000, 3200), (513, 270, 4112),
               (1024, 512, 1536), (96, 256, 64), (97, 257, 272), (300, 35850, 80), (520, 15400, 144), (512, 27700, 80)]

FULL_SIZE_DECODE = [(2, "gate_up", 4096, 22016, (1, 8, 32, 64)), (2, "down", 11008, 4096, (1, 8, 32, 64)),
                    (2, "qkv", 4096, 12288, (16, 64)), (4, "gate_up", 8192, 57344, (1, 64)), (4, "down", 28672, 8192, (1, 32))]

FAMILY_DECODE = [("13b_qkv", 5120, 15360), ("13b_o", 5120, 5120), ("13b_gate_up", 5120, 27648), ("13b_down", 13824, 5120),
                 ("30b_qkv", 6656, 19968), ("30b_o", 6656, 6656), ("30b_gate_up", 6656, 35840), ("30b_down", 17920, 6656)]

# merged gate | up projection with the gate in the epilogue, (M, F, K): both workgroup shapes of its selection (F / 16 up
# to 700 and above), K tails, several tokens
FFN_GATE_UP_SHAPES = [(1, 8640, 3200), (1, 11008, 4096), (3, 1008, 1040), (1, 16, 16), (2, 11216, 272), (16, 48, 528),
                      (1, 4000, 4112), (1, 16400, 272), (2, 16640, 528),   # the last two: more than 1024 pairs (eight per workgroup)
                      (1, 16400, 8208)]                                     # ... and 32 K steps and more (extra steps up front)

# prefill at full size, (M, N, K, tensor index of the seed): the four 13B-class projections at 2048 and at 512 tokens
FULL_SIZE_GEMM = [(2048, 15360, 5120, 0), (2048, 5120, 5120, 1), (2048, 27648, 5120, 2), (2048, 5120, 13824, 3),
                  (512, 15360, 5120, 0), (512, 5120, 5120, 1), (512, 27648, 5120, 2), (512, 5120, 13824, 3)]

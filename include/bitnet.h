/*
 * bitnet.h -- C ABI of the MI355X (gfx950) BitLinear W1.58A8 library.
 *
 * The library computes the BitLinear product of BitNet b1.58 (arXiv 2402.17764, Section 2):
 *
 *     gamma  = mean_ij |W_ij|                                   Eq. (3)
 *     Wt     = RoundClip(W / (gamma + eps), -1, 1)              Eq. (1)-(2), eps = 1e-5
 *     s_x[m] = max(max_k |x[m,k]|, 1e-5)                         per-token absmax (Section 2)
 *     x_q    = clip(round(x * 127 / s_x[m]), -127, 127)          8-bit, symmetric, no zero point
 *     acc    = x_q . Wt^T        (int32, exact)                  the "integer addition only" product
 *     y      = acc * gamma * s_x[m] / 127                        undoing both scales
 *
 * round() is IEEE round-half-to-even everywhere.  gamma is the fp32 rounding of an fp64 quotient
 * whose numerator is accumulated with compensated (double-double) summation, so it does not depend
 * on the reduction order.
 *
 * Conventions for every entry point
 *   - Matrices are row-major: W [N][K], x and x_q [M][K], y [M][N]  (y = x . W^T, the orientation of
 *     a linear layer's weight).
 *   - Every data pointer is DEVICE memory owned by the caller, unless marked (host).  The library
 *     allocates nothing and keeps no state between calls (beyond raising, once per device, the
 *     dynamic-LDS limit of the kernels that need it).  Inputs are never written; outputs are fully
 *     overwritten; workspaces are scratch.  gamma and s_x stay on the device, so no call synchronizes with the host.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls are asynchronous
 *     on that stream and may be captured into a HIP graph.
 *   - Arguments are validated on the host before anything is launched; on any error nothing has been
 *     launched and no output has been touched.  A launch failure reported by the runtime maps to
 *     BITNET_ERR_HIP.  Non-finite input values are a precondition violation: the result is
 *     unspecified but no memory outside the outputs is touched.
 *   - Results are deterministic run to run (no floating-point atomics anywhere).
 *   - Limits: 1 <= M, N, K;  N*K < 2^40;  K <= 262144 (so 64*127*K fits the int32 accumulator the
 *     kernels use internally);  M*K and M*N < 2^40.
 */
#ifndef BITNET_H
#define BITNET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Every enum below ends in an *_INT_RANGE_ member that is never a valid argument: it makes every non-negative int a
 * representable value of the type, so that a caller's out-of-range code reaches the library's own check (and comes
 * back as BITNET_ERR_DTYPE / _FORMAT / _KERNEL) instead of being undefined in a C++ translation unit. */
typedef enum bitnet_status {
    BITNET_OK = 0,
    BITNET_ERR_NULL = 1,        /* a required pointer is NULL */
    BITNET_ERR_SHAPE = 2,       /* a size is <= 0 or beyond the limits above */
    BITNET_ERR_DTYPE = 3,       /* dtype not accepted by this argument */
    BITNET_ERR_FORMAT = 4,      /* unknown packing format, or not supported by this call */
    BITNET_ERR_ALIGN = 5,       /* a pointer is not aligned as documented */
    BITNET_ERR_WORKSPACE = 6,   /* workspace smaller than the call needs (see the call's workspace query) */
    BITNET_ERR_HIP = 7,         /* the HIP runtime refused the launch */
    BITNET_ERR_KERNEL = 8,      /* requested kernel variant cannot run this shape */
    BITNET_STATUS_INT_RANGE_ = 0x7fffffff
} bitnet_status;

typedef enum bitnet_dtype {
    BITNET_F32 = 0,
    BITNET_BF16 = 1,
    BITNET_I32 = 2,             /* only as y_dtype: raw int32 accumulators, for exactness checks */
    BITNET_DTYPE_INT_RANGE_ = 0x7fffffff
} bitnet_dtype;

/*
 * Storage formats for the ternary matrix Wt (Section 3 of the paper stores 2 bits per weight and
 * notes that 1.58 bits leaves room below that).
 *
 * BITNET_PACK_2BIT -- 4 codes per byte, tiled for 64-lane wavefronts, K-step major.
 *   N is padded to Np = 16*ceil(N/16) rows (RB = Np/16 row blocks) and K to Kp = 64*ceil(K/64)
 *   columns (Kq = Kp/64) with zero codes.  The buffer is an array of 16-byte "quads"; one quad holds
 *   the 64 codes of one row for 64 consecutive columns.  Columns are grouped into steps of 256
 *   (4 quads); the last step may hold fewer: nq(s) = min(4, Kq - 4*s).  The quad of row
 *   n = 16*rb + r, columns 64*(4*s + g) .. +63  (g < nq(s)) has index
 *       64*RB*s + 16*nq(s)*rb + 16*g + r,
 *   i.e. for each step all row blocks follow one another, and one (step, row block) chunk is the
 *   1 KiB that the 64 lanes of a wavefront fetch with one 128-bit load each (lane = 16*g + r).
 *   A quad is four little-endian 32-bit words; word j holds columns 16*j .. 16*j+15 of the quad;
 *   inside a word the code of column 16*j + 4*i + b  (i, b in 0..3) sits in bits
 *   [8*b + 2*i, 8*b + 2*i + 1].  A code is 2-bit two's complement: 00 = 0, 01 = +1, 11 = -1
 *   (10 never occurs).  Size: Np * Kp / 4 bytes.
 *
 * BITNET_PACK_TRIT5 -- 5 codes per byte (1.6 bits per weight), base 3, K-step major like the 2-bit format.
 *   N is padded to Np = 16*ceil(N/16) rows (RB row blocks), K to Kp = 320*ceil(K/320) columns with zero
 *   codes.  A quad (16 bytes) holds the 80 codes of one row for 80 consecutive columns; a step is 320
 *   columns (4 quads).  The quad of row n = 16*rb + r, columns 320*s + 80*g .. +79 has index
 *       64*(RB*s + rb) + 16*g + r.
 *   Byte p (0..15) of a quad holds five base-3 digits, value = sum_d (code_d + 1) * 3^d  (0..242):
 *   digits 0..3 are the codes of columns 4*p + 0..3 of the quad, digit 4 the code of column 64 + p.
 *   (So one table look-up per byte yields four consecutive codes, i.e. one 32-bit MFMA operand
 *   register, and the sixteen fifth digits of a quad form the operand of a fifth MFMA.)
 *   Size: Np * Kp / 5 bytes.  Supported by bitnet_quantize_weights, bitnet_unpack_weights and
 *   bitnet_linear (weight-streaming kernel for 16 tokens at a time: more tokens re-stream the weights per
 *   group of 16, so this is a storage format rather than a prefill one; the reference kernel serves shapes
 *   the streaming kernel cannot); bitnet_linear_fused, the per-segment scales and the MFMA prefill kernel
 *   take the 2-bit format only.
 */
typedef enum bitnet_format {
    BITNET_PACK_2BIT = 0,
    BITNET_PACK_TRIT5 = 1,
    BITNET_FORMAT_INT_RANGE_ = 0x7fffffff
} bitnet_format;

/* Kernel choice for bitnet_linear_variant (bitnet_linear picks by shape). */
typedef enum bitnet_kernel {
    BITNET_KERNEL_AUTO = 0,
    BITNET_KERNEL_REFERENCE = 1, /* one thread per output, any shape; the slow, obviously right one */
    BITNET_KERNEL_GEMV = 2,      /* weight-streaming decode kernels: M <= 64, on small layers up to 512 */
    BITNET_KERNEL_GEMM = 3,      /* LDS-tiled int8 MFMA prefill kernel, tile shape picked by shape */
    /* the prefill kernel with a fixed workgroup tile (tokens x weight rows): for tuning and tests */
    BITNET_KERNEL_GEMM_128x256 = 0x142,
    BITNET_KERNEL_GEMM_96x256 = 0x132,
    BITNET_KERNEL_GEMM_64x256 = 0x122,
    BITNET_KERNEL_GEMM_128x128 = 0x141,
    BITNET_KERNEL_GEMM_96x128 = 0x131,
    BITNET_KERNEL_GEMM_64x128 = 0x121,
    /* the same tiles contracted by eight waves in two K groups (each group half of the K steps, integer accumulators
       added through LDS: same result): the form for grids that leave a CU with one workgroup */
    BITNET_KERNEL_GEMM_96x128_K2 = 0x1B1,
    BITNET_KERNEL_GEMM_64x256_K2 = 0x1A2,
    /* eight waves in two row groups on one token tile: tiles of 512 weight rows whose activation stages both groups
       read (less traffic into the CU per multiply); one workgroup per CU */
    BITNET_KERNEL_GEMM_128x512 = 0x14A,
    /* bitnet_linear_ws only: the K steps split over 2, 4 or 8 workgroups per tile (prefill kernel; where the batched-decode kernels serve the shape,
       the batched-decode kernels) */
    BITNET_KERNEL_GEMM_SPLITK_2 = 0x202,
    BITNET_KERNEL_GEMM_SPLITK_4 = 0x204,
    BITNET_KERNEL_GEMM_SPLITK_8 = 0x208,
    BITNET_KERNEL_INT_RANGE_ = 0x7fffffff
} bitnet_kernel;

/* Library version, major*10000 + minor*100 + patch.  Also the version of the packed layouts. */
int bitnet_version(void);

/* Human-readable name of a status code; never NULL; static storage. */
const char* bitnet_status_string(bitnet_status s);

/* Bytes of the packed buffer for an N x K matrix in format f, written to *bytes (host). */
bitnet_status bitnet_packed_bytes(int64_t N, int64_t K, bitnet_format f, size_t* bytes);

/* Bytes of scratch bitnet_quantize_weights needs (host out).  Independent of the format. */
bitnet_status bitnet_quantize_weights_workspace(int64_t N, int64_t K, size_t* bytes);

/*
 * Eq. (1)-(3): W -> packed ternary codes + gamma.
 *   W          [N][K], dtype F32 or BF16, 4-byte (F32) / 2-byte (BF16) aligned
 *   packed     out, bitnet_packed_bytes() bytes, 16-byte aligned; padding codes are written as 0
 *   gamma      out, 1 float (device)
 *   workspace  scratch of at least bitnet_quantize_weights_workspace() bytes, 16-byte aligned;
 *              contents on entry are ignored, contents on exit are unspecified
 * Two launches on `stream` for the 2-bit format: |W| partial sums (double-double), then the
 * ternarize-and-pack pass, whose workgroups first fold the partial sums to gamma (the 5-trit format keeps
 * that reduction as a launch of its own).  A 16-byte aligned W takes the vector path of the |W| sum.
 * One gamma per call: a fused QKV or gate/up matrix passed as one tensor gets one scale.
 */
bitnet_status bitnet_quantize_weights(const void* W, bitnet_dtype w_dtype, int64_t N, int64_t K,
                                      bitnet_format f, void* packed, float* gamma,
                                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * bitnet_quantize_weights without a workspace argument and without any allocation, for callers that cannot
 * allocate device memory: code running under HIP-graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The block partial sums of the |W| reduction go to a static 32 KiB array in device memory that belongs to
 * the library (one copy per GPU, held until the process ends) instead of a caller's buffer; kernels, launch shapes and
 * results are those of bitnet_quantize_weights, bit for bit.
 *   W, packed, gamma, stream   as for bitnet_quantize_weights
 *   Limit: the partial sums of the shape must fit the static array (BITNET_ERR_WORKSPACE otherwise; true of every
 *   shape the library accepts today, whose need is a fixed 32 KiB).
 * Every call on a GPU uses that GPU's one array: calls that may overlap on one GPU (different streams, no ordering
 * between them) race on it and must use bitnet_quantize_weights with workspaces of their own.  Nothing in the array
 * has to be cleared between calls: the first kernel overwrites every entry the second one reads.
 */
bitnet_status bitnet_quantize_weights_static(const void* W, bitnet_dtype w_dtype, int64_t N, int64_t K,
                                             bitnet_format f, void* packed, float* gamma, void* stream);

/*
 * Eq. (3) for a matrix whose rows are spread over several devices (or quantized in several pieces): gamma is the
 * mean of |W| over the WHOLE matrix, so each holder of a row shard first reports its share of the sum, the shares
 * are exchanged (G pairs of doubles; between GPUs an all-gather of 16 bytes each), and every holder then quantizes
 * its rows with the gamma of the whole.  Codes and gamma are bit-identical to one bitnet_quantize_weights call on the
 * whole matrix: the shares are exact (double-double) sums, so neither the split nor the order of the pairs shows.
 *
 * bitnet_abs_sum: sum[0] + sum[1] = sum_ij |W_ij| over these N rows, as a normalised double-double pair.
 *   W          [N][K], F32 or BF16, element-aligned
 *   sum        out, 2 doubles (device), 8-byte aligned
 *   workspace  as for bitnet_quantize_weights (same size query)
 *
 * bitnet_quantize_weights_sharded: Eq. (1)-(2) and the packing of bitnet_quantize_weights for these N rows, with
 * gamma = fp32((sum of the nsums pairs) / (total_rows * K)).
 *   sums        nsums consecutive (hi, lo) pairs (device), e.g. the gathered outputs of bitnet_abs_sum; 1 <= nsums <= 256
 *   total_rows  rows of the whole matrix (>= N)
 *   packed      out, bitnet_packed_bytes(N, K, f) bytes: the packed layout of the shard's own [N][K] matrix
 *   gamma       out, 1 float (device): the gamma of the whole matrix
 * One launch for the 2-bit format (the packing pass folds the pairs itself), two for the 5-trit format.  No workspace.
 */
bitnet_status bitnet_abs_sum(const void* W, bitnet_dtype w_dtype, int64_t N, int64_t K, double* sum, void* workspace,
                             size_t workspace_bytes, void* stream);
bitnet_status bitnet_quantize_weights_sharded(const void* W, bitnet_dtype w_dtype, int64_t N, int64_t K, bitnet_format f,
                                              const double* sums, int nsums, int64_t total_rows, void* packed,
                                              float* gamma, void* stream);

/*
 * Section 2, activation quantization: x -> int8 codes + one scale per token.
 *   x    [M][K], dtype F32 or BF16, element-aligned (16-byte aligned rows take the vector path)
 *   xq   out [M][K] int8
 *   sx   out [M] float: the clamped absmax, i.e. x ~ x_q * sx / 127
 */
bitnet_status bitnet_quantize_acts(const void* x, bitnet_dtype x_dtype, int64_t M, int64_t K,
                                   int8_t* xq, float* sx, void* stream);

/*
 * Producers of int8 activations.  Section 2 ("LLaMA-alike components") names RMSNorm and SwiGLU as the
 * operations around BitLinear; these two entry points fuse the activation quantization above into them,
 * so a block hands int8 codes and scales from layer to layer and bitnet_linear never waits for a separate
 * quantization launch.  Every rounding step is fixed (stated below), so x_q and the scale are exactly
 * reproducible.
 *
 * bitnet_rmsnorm_quantize: per token, ms = mean_k x^2 (exact in fp64), r = (float)(1 / sqrt(ms + eps))
 * computed in fp64, z = (x * r) * g in fp32 (g == NULL: no gain, z = x * r), then sx / xq from z as in
 * bitnet_quantize_acts.
 *   x    [M][K], dtype F32 or BF16, element-aligned (16- / 8-byte aligned rows with K % 4 == 0 and
 *        K <= 65536 stay in registers between the passes; other shapes re-read x)
 *   g    [K] float (device) or NULL
 *   eps  added to the mean square; >= 0
 *   xq   out [M][K] int8;  sx  out [M] float
 *
 * bitnet_swiglu_quantize: gu is [M][2 F] (the output of a merged gate/up projection), per element
 * h = (gate / (1 + exp(-gate))) * up with gate = gu[m][f], up = gu[m][F + f]; exp is evaluated in fp32 as
 * 2^n * p(r), n = round(-gate * log2 e), r = -gate - n ln 2 (two-constant reduction), p the degree-6
 * Taylor polynomial in Horner form, arguments clamped to [-87, 88]; add, divide and multiply are single
 * fp32 operations.  Then sh / hq from h as in bitnet_quantize_acts.
 *   gu   [M][2 F], dtype F32 or BF16, element-aligned
 *   hq   out [M][F] int8;  sh  out [M] float
 */
bitnet_status bitnet_rmsnorm_quantize(const void* x, bitnet_dtype x_dtype, const float* g, float eps,
                                      int64_t M, int64_t K, int8_t* xq, float* sx, void* stream);
bitnet_status bitnet_swiglu_quantize(const void* gu, bitnet_dtype gu_dtype, int64_t M, int64_t F,
                                     int8_t* hq, float* sh, void* stream);

/*
 * The BitLinear product and rescale (Section 2: BitLinear replaces nn.Linear; Section 1: the product of ternary weights
 * and 8-bit activations needs integer addition only): y = (x_q . Wt^T) * gamma * s_x / 127, the integer sum exact in
 * int32, gamma of Eq. (3) and the per-token s_x undone in floating point.
 *   xq, sx   as written by bitnet_quantize_acts
 *   packed   as written by bitnet_quantize_weights for the same (N, K, f); 16-byte aligned
 *   gamma    1 float (device)
 *   y        out [M][N]; y_dtype F32, BF16 (round-to-nearest-even of the fp32 value) or I32 (the raw
 *            accumulator, no scaling); element-aligned
 * The kernel is chosen by shape: the weight-streaming decode kernels for M <= 64 (and up to 256 tokens, with
 * K >= 5120 up to 512, on layers small enough that 256 workgroups of token tiles cover them: up to 4096-12288 output
 * features), the MFMA GEMM above, the reference kernel when xq is not 16-byte aligned or K is not a multiple of 16.
 */
bitnet_status bitnet_linear(const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                            int64_t M, int64_t N, int64_t K, bitnet_format f,
                            void* y, bitnet_dtype y_dtype, void* stream);

/* Same, with the kernel forced (tests and benchmarks).  BITNET_ERR_KERNEL if it cannot run the shape. */
bitnet_status bitnet_linear_variant(const int8_t* xq, const float* sx, const void* packed,
                                    const float* gamma, int64_t M, int64_t N, int64_t K,
                                    bitnet_format f, void* y, bitnet_dtype y_dtype,
                                    bitnet_kernel which, void* stream);

/*
 * Which kernel and launch shape bitnet_linear (workspace_bytes == 0) or bitnet_linear_ws (with a workspace of that
 * size) takes for a shape.  Host only: nothing is launched and no device is needed.  For operators who want to see
 * why a shape runs the way it does, and for tests of the selection rules (Sections 1-2 fix what is computed; how the
 * launch is shaped is this library's choice).  Pointers are assumed aligned as the fast kernels require.
 *   text  out, host: "kernel=<family> params=<template parameters> grid=<x>x<y> block=<threads> lds=<bytes>
 *         splits=<n>", zero-terminated; BITNET_ERR_WORKSPACE if text_bytes is too small (128 is enough)
 *   families and their parameters:
 *     decode                 M <= 4: row blocks per wave, K waves, row slots, prefetch depth, x_q source (0 global, 1 LDS)
 *     batched_decode         5 ... 512 tokens: token tiles of 16, row blocks per wave, row slots, K groups, prefetch
 *     batched_decode_loader  depth, LDS lookahead (the second form has a wave that only copies activations)
 *     prefill                tile tokens, tile rows, and 2 as a third parameter for the eight-wave form with two
 *                            K groups (512 tile rows: the eight-wave form with two row groups); grid y = split-K factor
 *     reference, trit5_decode, trit5_reference: no parameters
 *   5-trit weights, more than 16 tokens and a workspace that holds the 2-bit copy (bitnet_linear_workspace_format):
 *   the plan of the 2-bit launch that follows the repacking pass, with " repack=trit5_to_2bit" appended
 */
bitnet_status bitnet_linear_describe(int64_t M, int64_t N, int64_t K, bitnet_format f, size_t workspace_bytes,
                                     char* text, size_t text_bytes);

/*
 * The same for the entry points that quantize x inside the decode launch (Section 2: per-token activation
 * quantization; "LLaMA-alike components": RMSNorm, SwiGLU): which instantiation of the decode kernel a call of
 * `entry` with these sizes would launch.  Host only, nothing is launched.  With it every launch a benchmark or a
 * serving loop makes can be listed and matched against the forms the parity tests reach.
 *   entry    which entry point; BITNET_ENTRY_LINEAR is bitnet_linear_describe
 *   x_dtype  F32 or BF16 (the kernel is instantiated per input type); ignored for BITNET_ENTRY_LINEAR
 *   N, K     as the entry point takes them: for BITNET_ENTRY_SWIGLU_LINEAR_FUSED K is its F, for the two
 *            BITNET_ENTRY_FFN_GATE_UP_* N is its F (the packed matrix has 2 F rows)
 *   text     as bitnet_linear_describe; the fifth decode parameter is the activation source: 0 int8 from global
 *            memory, 1 int8 staged in LDS, 2 / 3 bf16 / fp32 x quantized in the kernel, 4 / 5 RMSNorm first,
 *            6 / 7 SwiGLU first; family "decode_pair" is the gate/up launch with the gate in its epilogue
 * BITNET_ERR_KERNEL where the entry point would refuse the shape.
 */
typedef enum bitnet_entry {
    BITNET_ENTRY_LINEAR = 0,
    BITNET_ENTRY_LINEAR_FUSED = 1,
    BITNET_ENTRY_RMSNORM_LINEAR_FUSED = 2,
    BITNET_ENTRY_SWIGLU_LINEAR_FUSED = 3,
    BITNET_ENTRY_FFN_GATE_UP = 4,            /* bitnet_ffn_gate_up_fused with norm == 0 */
    BITNET_ENTRY_FFN_GATE_UP_NORM = 5,       /* ... with norm != 0 */
    BITNET_ENTRY_INT_RANGE_ = 0x7fffffff
} bitnet_entry;
bitnet_status bitnet_entry_describe(bitnet_entry entry, bitnet_dtype x_dtype, int64_t M, int64_t N, int64_t K,
                                    bitnet_format f, size_t workspace_bytes, char* text, size_t text_bytes);

/*
 * bitnet_linear with a scratch buffer.  Between decode and large prefill -- a few hundred tokens on layers with few
 * output features -- even the smallest tiles of the prefill kernel give the 256 CUs too few workgroups, each walking
 * all of K.  With a workspace the K steps of a tile are split over 2, 4 or 8 workgroups that store int32 partial
 * accumulators there; a second launch adds them (exact, independent of the split) and rescales.  Chosen by the same
 * cost model as the tile shape, only where it pays: long K, few tiles (measured on MI355X, M = 128: 11008 -> 4096 in
 * 18.1 instead of 25.4 us, 28672 -> 8192 in 40.7 instead of 70.9 us; nothing to gain at K = 4096 or from 512 tokens
 * on).  The batched-decode kernels can split the same way when forced, but never do by themselves:
 * tiling the tokens over workgroups serves their small-layer cases better without a second launch.  Results are
 * bit-identical to bitnet_linear / bitnet_linear_segmented.
 *   gamma_per_block  0: one gamma; otherwise one per 16-row block (as bitnet_linear_segmented)
 *   which            BITNET_KERNEL_AUTO, any selector of bitnet_linear_variant (the workspace is then unused), or
 *                    BITNET_KERNEL_GEMM_SPLITK_n to force n splits (BITNET_ERR_WORKSPACE if the buffer is too small
 *                    or K has fewer than n steps of 256 columns); the split then runs on the kernel family the
 *                    automatic choice takes for the shape: batched decode from 5 tokens on where it serves it, else the prefill kernel
 *   workspace        device memory, 16-byte aligned, or NULL (then this is bitnet_linear); contents are scratch:
 *                    nothing is expected in it and nothing of value is left; calls that share it must not overlap
 *   workspace_bytes  its size; bitnet_linear_workspace reports the size with which every split the model may want fits
 *                    (0 where split-K is never considered: shapes the decode kernels serve, or 512 or more tiles
 *                    of 64 x 128)
 */
bitnet_status bitnet_linear_workspace(int64_t M, int64_t N, int64_t K, size_t* bytes);
bitnet_status bitnet_linear_ws(const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                               int gamma_per_block, int64_t M, int64_t N, int64_t K, bitnet_format f,
                               void* y, bitnet_dtype y_dtype, bitnet_kernel which, void* workspace,
                               size_t workspace_bytes, void* stream);

/*
 * The 5-trit format at prefill sizes (Section 3: storage below 2 bits per weight).  The MFMA prefill kernel and the
 * batched-decode kernels read the 2-bit layout, whose fields are MFMA operand bytes after one shift and one AND; base-3
 * digits need a table look-up per byte, which costs more issue slots than the product leaves free.  So weights kept in
 * HBM in the 5-trit format are repacked to the 2-bit layout once per call -- 0.45 bytes of traffic per weight -- rather
 * than decoded once per tile:
 *
 * bitnet_repack_weights: the same code matrix in the other format, on the device (either direction; the result is
 * byte-identical to what bitnet_quantize_weights writes in that format).
 *   packed_in / packed_out  bitnet_packed_bytes() bytes of their formats, 16-byte aligned, not overlapping
 *   f_in != f_out           (BITNET_ERR_FORMAT otherwise)
 *
 * bitnet_linear_ws with f == BITNET_PACK_TRIT5, which == BITNET_KERNEL_AUTO, one gamma, more than 16 tokens, K a multiple
 * of 16 and a workspace of at least bitnet_linear_workspace_format() bytes does this by itself: it repacks into the
 * head of the workspace and runs the 2-bit path on the copy with the rest of the workspace.  With a smaller workspace,
 * and through bitnet_linear, 5-trit weights are walked 16 tokens at a time by the decode kernel as before.
 *
 * bitnet_linear_workspace_format: bitnet_linear_workspace for a given weight format.
 */
bitnet_status bitnet_repack_weights(const void* packed_in, bitnet_format f_in, int64_t N, int64_t K, void* packed_out,
                                    bitnet_format f_out, void* stream);
bitnet_status bitnet_linear_workspace_format(int64_t M, int64_t N, int64_t K, bitnet_format f, size_t* bytes);

/*
 * Decode path in one launch: activation quantization fused into the weight-streaming kernel, x -> y.
 * Same arithmetic as bitnet_quantize_acts followed by bitnet_linear, with bit-identical x_q and s_x:
 * every workgroup re-derives them for all M tokens into LDS (x is small and cache-resident at decode
 * sizes); nothing is written besides y.
 *   x   [M][K], dtype F32 or BF16, 16-byte aligned
 *   Limits: M <= 16, K a multiple of 16 and M * 256 * ceil(K / 256) + 512 <= 65536 bytes of LDS
 *   (M = 1 up to K = 65024, M = 4 up to K = 16128); otherwise BITNET_ERR_KERNEL and nothing is launched.
 * Meant for M = 1, where it saves a launch (3B-class layers on MI355X: 3.6-6.8 us against 5.1-7.5 us for the
 * two calls).  Because every workgroup repeats the quantization of all M tokens, bitnet_quantize_acts followed
 * by bitnet_linear is the faster route from about M = 3 on (measured: 8.7 us against 12.4 us on a 3200 ->
 * 17280 layer at M = 4); a producer that already emits int8 (bitnet_rmsnorm_quantize, bitnet_swiglu_quantize)
 * avoids the question.
 */
bitnet_status bitnet_linear_fused(const void* x, bitnet_dtype x_dtype, const void* packed,
                                  const float* gamma, int64_t M, int64_t N, int64_t K,
                                  bitnet_format f, void* y, bitnet_dtype y_dtype, void* stream);

/*
 * The same with RMSNorm in front (Section 2, "LLaMA-alike components": RMSNorm precedes the attention and the
 * feed-forward BitLinear layers): y = BitLinear(RMSNorm(x)) in one launch, x -> y.  Same arithmetic as
 * bitnet_rmsnorm_quantize followed by bitnet_linear, with bit-identical x_q and s_x; every workgroup re-derives
 * them into LDS, nothing is written besides y.  At decode (M = 1) it replaces two launches of a dependent chain.
 *   x    [M][K], dtype F32 or BF16, 16-byte aligned
 *   g    [K] float (device), 16-byte aligned, or NULL for no gain
 *   eps  added to the mean square; >= 0 (BITNET_ERR_SHAPE otherwise)
 *   Limits as for bitnet_linear_fused.  2-bit format only.
 * Measured at M = 1 on MI355X (3200 -> 9600 / 3200 -> 17280 / 8192 -> 57344): 6.5 / 8.2 / 24.7 us against 9.2 / 10.6 /
 * 27.0 us for bitnet_rmsnorm_quantize + bitnet_linear.
 * bitnet_rmsnorm_linear_fused_segmented: with one gamma per 16-row block, as bitnet_linear_fused_segmented.
 */
bitnet_status bitnet_rmsnorm_linear_fused(const void* x, bitnet_dtype x_dtype, const float* g, float eps,
                                          const void* packed, const float* gamma, int64_t M, int64_t N,
                                          int64_t K, bitnet_format f, void* y, bitnet_dtype y_dtype,
                                          void* stream);
bitnet_status bitnet_rmsnorm_linear_fused_segmented(const void* x, bitnet_dtype x_dtype, const float* g,
                                                    float eps, const void* packed, const float* gamma_rb,
                                                    int64_t M, int64_t N, int64_t K, bitnet_format f,
                                                    void* y, bitnet_dtype y_dtype, void* stream);

/*
 * ... and with SwiGLU in front (Section 2, "LLaMA-alike components": the down projection of the feed-forward block
 * consumes silu(gate) * up): y = BitLinear(SwiGLU(gu)) in one launch.  Same arithmetic as bitnet_swiglu_quantize
 * followed by bitnet_linear, with bit-identical h_q and s_h; nothing is written besides y.
 *   gu   [M][2 F] (gate | up, the output of a merged gate/up projection), dtype F32 or BF16, 16-byte aligned
 *   F    columns of the product (the K of bitnet_linear); packed holds an [N][F] matrix
 *   Limits as for bitnet_linear_fused with K = F.  2-bit format only.
 * Every workgroup repeats the gating of all F elements (an exponential and a division each), so this pays only
 * while F is small against the weight stream: measured at M = 1 on MI355X, 8.1 us against 8.7 us for the two calls
 * at F = 8640 (N = 3200), 9.2 against 9.5 us at F = 11008 (N = 4096), but 53 against 22 us at F = 28672 (N = 8192)
 * -- there bitnet_swiglu_quantize followed by bitnet_linear is the route.
 */
bitnet_status bitnet_swiglu_linear_fused(const void* gu, bitnet_dtype gu_dtype, const void* packed,
                                         const float* gamma, int64_t M, int64_t N, int64_t F,
                                         bitnet_format f, void* y, bitnet_dtype y_dtype, void* stream);

/*
 * The front half of the feed-forward block in one decode launch (Section 2, "LLaMA-alike components": SwiGLU):
 * [y_gate | y_up] = BitLinear(pre(x)) over a merged gate | up matrix, and h = silu(y_gate) * y_up is what gets
 * stored -- the gate is applied where its two operands meet, once per element, and the 2 F projection outputs
 * never travel through memory.  y_gate and y_up are the fp32 values bitnet_linear would store; silu as in
 * bitnet_swiglu_quantize (same fixed-step exponential, one IEEE division).
 *   x        [M][K], dtype F32 or BF16, 16-byte aligned
 *   norm     0: pre = per-token absmax quantization (as bitnet_linear_fused);
 *            1: pre = RMSNorm then quantization (as bitnet_rmsnorm_linear_fused), with g ([K] floats, 16-byte
 *            aligned, or NULL) and eps >= 0; g and eps are ignored when norm == 0
 *   packed   the [2 F][K] matrix, gate rows first; F a multiple of 16 (BITNET_ERR_SHAPE otherwise)
 *   gamma    one float, or with gamma_per_block != 0 one per 16-row block (2 F / 16 floats, e.g. from
 *            bitnet_quantize_weights_segmented with the segments {F, F})
 *   h        out [M][F], dtype F32 or BF16 (BITNET_ERR_DTYPE for I32)
 *   Limits as for bitnet_linear_fused.  2-bit format only.
 * The down projection then takes h through bitnet_linear_fused.
 */
bitnet_status bitnet_ffn_gate_up_fused(const void* x, bitnet_dtype x_dtype, int norm, const float* g, float eps,
                                       const void* packed, const float* gamma, int gamma_per_block,
                                       int64_t M, int64_t F, int64_t K, bitnet_format f, void* h,
                                       bitnet_dtype h_dtype, void* stream);

/*
 * One scale per segment of rows.  Eq. (3) gives every weight matrix its own gamma; when several
 * matrices are stored as one (merged Q|K|V or gate|up projections) these entry points keep one gamma per
 * original matrix instead of one for the merged tensor.
 *
 * bitnet_quantize_weights_segmented: rows are split into nseg consecutive segments of seg_rows[i] rows
 * (host array; every segment but the last a multiple of 16 rows; the sum is N).  Each segment gets its own
 * gamma (Eq. (3) over its rows) and its codes (Eq. (1)-(2) with that gamma), packed into one buffer with
 * the layout of the whole [N][K] matrix.
 *   gamma_rb   out, ceil(N / 16) floats (device): the gamma of the segment that each 16-row block belongs to
 *   workspace  as for bitnet_quantize_weights; used by one segment after the other in stream order
 * 2-bit format only (BITNET_ERR_FORMAT otherwise).
 *
 * bitnet_linear_segmented / bitnet_linear_fused_segmented: as bitnet_linear_variant / bitnet_linear_fused
 * with y[m][n] = acc * gamma_rb[n / 16] * s_x[m] / 127.  `which` as in bitnet_linear_variant
 * (BITNET_KERNEL_AUTO picks by shape).
 */
bitnet_status bitnet_quantize_weights_segmented(const void* W, bitnet_dtype w_dtype, int64_t N, int64_t K,
                                                int nseg, const int64_t* seg_rows, bitnet_format f,
                                                void* packed, float* gamma_rb, void* workspace,
                                                size_t workspace_bytes, void* stream);
bitnet_status bitnet_linear_segmented(const int8_t* xq, const float* sx, const void* packed,
                                      const float* gamma_rb, int64_t M, int64_t N, int64_t K,
                                      bitnet_format f, void* y, bitnet_dtype y_dtype, bitnet_kernel which,
                                      void* stream);
bitnet_status bitnet_linear_fused_segmented(const void* x, bitnet_dtype x_dtype, const void* packed,
                                            const float* gamma_rb, int64_t M, int64_t N, int64_t K,
                                            bitnet_format f, void* y, bitnet_dtype y_dtype, void* stream);

/*
 * Test helper: packed -> codes [N][K] int8 in {-1, 0, +1} (padding dropped).  The only supported
 * way to read codes back besides decoding the documented layout by hand.
 */
bitnet_status bitnet_unpack_weights(const void* packed, int64_t N, int64_t K, bitnet_format f,
                                    int8_t* codes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BITNET_H */

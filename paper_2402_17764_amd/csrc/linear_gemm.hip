// Prefill BitLinear kernel for gfx950: the ternary-by-int8 product on int8 MFMA (M > 64).
//
// Computes acc[m][n] = sum_k x_q[m][k] * Wt[n][k] exactly in int32 and y = acc * gamma * s_x[m] / 127
// (Sections 1-2 of arXiv 2402.17764).  At these M the cost is the contraction itself, so the kernel is
// organised around keeping v_mfma_i32_32x32x32_i8 issuing:
//
//   * a workgroup of four waves owns a 128 x 256 output tile (tokens x weight rows), each wave a 128 x 64
//     piece held as 4 x 2 accumulator fragments of 32 x 32 (96 x 256 tiles with 3 x 2 fragments for shapes
//     that would otherwise leave CUs idle); two workgroups share a CU, so every SIMD has two waves that are
//     not tied to the same barrier: one workgroup's loads, decode and barrier waits run under the other's
//     MFMAs (a single wave does not overlap its own VALU work with its MFMAs);
//   * activations (the A operand) are copied global -> LDS with 128-bit LDS-direct loads, two stages of
//     128 rows x 256 bytes; the 16-byte chunks of a row are XOR-swizzled with the row index so that the
//     ds_read_b128 of 16 consecutive rows hit all 64 banks;
//   * weights (the B operand) never touch LDS: the packed layout already stores, for every 16-row block,
//     the 64 codes a lane needs as one 16-byte quad, so each lane loads its own quads straight from
//     global memory one K step ahead and expands one 32-bit word (16 codes) into the four operand
//     registers of an MFMA with a shift and an AND per register -- (w << (6 - 2 i)) & 0xC0C0C0C0 leaves
//     64 * code in every byte, and the factor 64 is divided out with the output scale at the end;
//   * inside a K step the eight 32-column slices are software pipelined: the LDS reads and the decode
//     of slice t + 1 are issued among the 16 MFMAs of slice t;
//   * one barrier per K step of 256 columns (64 MFMAs per wave between barriers);
//   * for grids that leave a CU with a single workgroup (a few hundred tokens on a layer with few rows), a form with
//     eight waves: two groups of four, each contracting half of the K steps through activation stages of its own, the
//     second group's accumulators added through LDS at the end -- the two waves per SIMD that two workgroups per CU
//     provide elsewhere, without a second launch;
//   * for grids of many 128 x 256 tiles whose count suits the chip, a form with eight waves in two row groups on one token
//     tile (128 x 512): both groups read the same activation stages, so the CU fetches a third less per MFMA than two
//     separate workgroups do -- the K loop's losses are waves held at the issue of their loads while the vector-memory
//     queues are full, and they shrink with the bytes a CU pulls in;
//   * the epilogue rescales in registers, transposes each 32 x 64 fragment row through LDS and writes
//     whole 16-byte pieces of output rows;
//   * tile order: consecutive workgroups take consecutive token tiles of the same weight tile, so the
//     eight XCDs (workgroups are dealt to them round-robin) each keep re-using the token tile that is
//     already in their L2 while the weight tile is shared through the memory-side cache.
//
// Lane l of a wave supplies, for the B operand, weight row (l & 31) of a 32-row fragment and the 16
// columns selected by (l >> 5); for the A operand token (l & 31), same columns.  (With the operands the other
// way round a lane would hold runs of four consecutive outputs of one token, a cheaper epilogue -- but the K
// loop then runs 10 % slower on MI355X, measured, so the activations stay first.)
#include "bitnet_device.hpp"
#include "bitnet_internal.hpp"

namespace bitnet {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// tokens per workgroup tile: kFM fragments of 32; 4 (128 tokens) is the default, 3 (96 tokens) exists for shapes
// whose 128-token tiles would leave many of the 512 workgroup slots (256 CUs x 2) empty
constexpr int kGemmThreads = 256;
// kFN: 32-row weight fragments per wave; the four waves sit side by side along the weight rows, so a workgroup tile
// has 128 * kFN of them.  2 is the default; 1 (narrow tiles) doubles the number of workgroups for shapes whose wide
// tiles would leave most CUs idle, at the same decode work per MFMA (that depends on the tile height only).
constexpr int kGemmPitch32 = 64 * 4 + 32;      // epilogue row pitch, 4-byte outputs: rows r and r+4 in different bank halves
constexpr int kGemmPitch16 = 64 * 2 + 32;      // same for bf16 outputs
constexpr int gemm_stage_bytes(int fm) { return fm * 32 * 256; }            // one K step of activations
// float scale[32 * fm] sits behind the two stages and behind the epilogue's staging area (four waves x 32 rows),
// which reuses the stages while the scales are still read
// ... and behind the area through which a second K group (kg == 2) hands over its accumulators: fm * fn * 16 registers
// of 256 threads
constexpr int gemm_max3(int a, int b, int c) { return a > b ? (a > c ? a : c) : (b > c ? b : c); }
// ... and, with two row groups (ng == 2: eight waves on one token tile), behind eight waves' staging areas
constexpr int gemm_scale_offset(int fm, int fn, int kg, int ng = 1) {
    return gemm_max3(kg * 2 * gemm_stage_bytes(fm), 4 * ng * 32 * kGemmPitch32, (kg - 1) * fm * fn * 16 * 4 * kGemmThreads);
}
constexpr int gemm_lds_bytes(int fm, int fn, int kg, int ng = 1) { return gemm_scale_offset(fm, fn, kg, ng) + fm * 32 * 4; }

__device__ inline uint32_t gemm_quad_word(const uint4& q, int j) { return j == 0 ? q.x : j == 1 ? q.y : j == 2 ? q.z : q.w; }

// one register of the decoded B operand: columns 4 i .. 4 i + 3 of the word, as 64 * code per byte; km is
// 0xC0C0C0C0, or 0 for lanes whose quad lies past a partial last K step
__device__ inline int gemm_decode_reg(uint32_t w, int i, uint32_t km) { return (int)((w << (6 - 2 * i)) & km); }

struct GemmOutCtx {
    char* lds;
    const float* scale_lds;
    void* y;
    const float* gamma;
    int gstride, RB;
    int M;
    int64_t N;
    int row0, bn, wave, lane, vec_store;
    int slot;               // which staging area: the wave's number in the workgroup
};

// A lane holds, per 32 x 32 fragment, 16 tokens (8 (v >> 2) + 4 (lane >> 5) + (v & 3)) of weight row
// (lane & 31).  Each wave stages one fragment row (32 tokens x 64 weight rows) in its own LDS region,
// then its lanes read 16-byte pieces along the token rows and store them.  The region is private to the
// wave, whose LDS accesses complete in order: no workgroup barrier is needed.  The decode factor 64 is
// divided out of the scale (exact: a power of two) instead of being shifted out of every accumulator.
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
__device__ inline uint32_t pack_bf16x2(float lo, float hi) {          // round to nearest even, one instruction
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((v2f){lo, hi}, v2bf));
}

template <OutType kOut, int kFM, int kFN>
__device__ inline void gemm_epilogue(v16i (&acc)[kFM][kFN], const GemmOutCtx& c) {
    constexpr bool is16 = kOut == OutType::BF16;
    constexpr int esz = is16 ? 2 : 4;
    constexpr int pitch = is16 ? kGemmPitch16 : kGemmPitch32;
    constexpr int lanes_per_row = 32 * kFN * esz / 16;              // 16-byte pieces of a staged row: 4, 8 or 16
    constexpr int rows_per_pass = 64 / lanes_per_row;
    const int am = c.lane & 31, kg = c.lane >> 5;
    const int wn = c.wave;
    char* stage_out = c.lds + c.slot * (32 * kGemmPitch32);
    const int64_t n_wave = (int64_t)c.bn * (128 * kFN) + wn * (32 * kFN);
    // with one gamma per row block the lane's weight row (am of fragment fn) picks its own; otherwise the
    // factor is 1 and the staged scale already carries gamma
    float gfn[kFN];
#pragma unroll
    for (int fn = 0; fn < kFN; ++fn) {
        const int rb = min((int)((n_wave + fn * 32 + am) / kRowsPerBlock), c.RB - 1);
        gfn[fn] = c.gstride ? c.gamma[rb] : 1.0f;
    }
    const int piece = c.lane % lanes_per_row;
    const int64_t n = n_wave + piece * (16 / esz);
#pragma unroll
    for (int fm = 0; fm < kFM; ++fm) {
#pragma unroll
        for (int v = 0; v < 16; v += 2) {                           // tokens rl and rl + 1
            const int rl = 8 * (v >> 2) + 4 * kg + (v & 3);
            float sc[2] = {0.0f, 0.0f};
            if (kOut != OutType::I32) {
                sc[0] = c.scale_lds[fm * 32 + rl] * 0.015625f;
                sc[1] = c.scale_lds[fm * 32 + rl + 1] * 0.015625f;
            }
#pragma unroll
            for (int fn = 0; fn < kFN; ++fn) {
                char* p = stage_out + rl * pitch + (fn * 32 + am) * esz;
                const int a0 = acc[fm][fn][v], a1 = acc[fm][fn][v + 1];
                if (kOut == OutType::I32) {
                    *reinterpret_cast<int32_t*>(p) = a0 >> 6;
                    *reinterpret_cast<int32_t*>(p + pitch) = a1 >> 6;
                } else {
                    const float f0 = (float)a0 * (gfn[fn] * sc[0]), f1 = (float)a1 * (gfn[fn] * sc[1]);
                    if (kOut == OutType::F32) {
                        *reinterpret_cast<float*>(p) = f0;
                        *reinterpret_cast<float*>(p + pitch) = f1;
                    } else {
                        const uint32_t pk = pack_bf16x2(f0, f1);
                        *reinterpret_cast<uint16_t*>(p) = (uint16_t)pk;
                        *reinterpret_cast<uint16_t*>(p + pitch) = (uint16_t)(pk >> 16);
                    }
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int r0 = 0; r0 < 32; r0 += rows_per_pass) {
            const int rl = r0 + c.lane / lanes_per_row;
            const int m = c.row0 + fm * 32 + rl;
            const uint4 val = *reinterpret_cast<const uint4*>(stage_out + rl * pitch + piece * 16);
            if (m < c.M && n < c.N) {
                char* dst = static_cast<char*>(c.y) + ((int64_t)m * c.N + n) * esz;
                if (c.vec_store && n + 16 / esz <= c.N) {
                    *reinterpret_cast<uint4*>(dst) = val;
                } else if (is16) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const uint32_t u = (e >> 1) == 0 ? val.x : (e >> 1) == 1 ? val.y : (e >> 1) == 2 ? val.z : val.w;
                        if (n + e < c.N) reinterpret_cast<uint16_t*>(dst)[e] = (uint16_t)(u >> (16 * (e & 1)));
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint32_t u = e == 0 ? val.x : e == 1 ? val.y : e == 2 ? val.z : val.w;
                        if (n + e < c.N) reinterpret_cast<uint32_t*>(dst)[e] = u;
                    }
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// One output tile of 32 * kFM tokens (first token row0) x 128 * kFN * kNG weight rows (tile bn), by kKG * kNG groups of
// four waves: kKG > 1 splits the K steps over the groups, kNG > 1 the weight rows (one of the two is 1).
template <int kFM, int kFN, int kKG, int kNG>
__device__ __forceinline__ void gemm_tile(
        const int8_t* __restrict__ xq, const float* __restrict__ sx, const uint4* __restrict__ packed,
        const float* __restrict__ gamma, int gstride, int M, int64_t N, int64_t K, int Kq, int RB, int row0, int bn,
        int step0, int step1 /* the K steps of 256 columns this workgroup contracts: all of them, or one split */,
        void* __restrict__ y, OutType yt, int vec_store) {
#if defined(__HIP_DEVICE_COMPILE__)      // the buffer-resource builtins exist in the device pass only
    extern __shared__ uint4 smem[];
    constexpr int kGemmBM = 32 * kFM;
    constexpr int kGemmStageBytes = gemm_stage_bytes(kFM);
    constexpr int kCopies = 2 * kFM / kNG;          // 1 KiB wave-loads (4 token rows) per wave and stage
    static_assert(kKG == 1 || kNG == 1, "groups split either the K steps or the weight rows");
    char* lds = reinterpret_cast<char*>(smem);
    float* scale_lds = reinterpret_cast<float*>(lds + gemm_scale_offset(kFM, kFN, kKG, kNG));

    const int lane = threadIdx.x & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: LDS-DMA targets need no per-step broadcast
    const int grp = kKG > 1 ? wave_all >> 2 : 0;        // K group: four waves that contract their own run of K steps
    const int wave = wave_all & 3;                      // the wave's place in its group
    const int wn = wave;
    char* glds = lds + grp * 2 * kGemmStageBytes;       // the group's two activation stages
    // Row groups: both contract every K step from the same activation stages (each of the eight waves copies an
    // eighth of a stage), the second on the next 128 * kFN weight rows -- half the activation traffic into the CU
    // per MFMA of two separate workgroups.
    const int copier = kNG > 1 ? wave_all : wave;
    bn = bn * kNG + (kNG > 1 ? wave_all >> 2 : 0);
    const int steps = (Kq + 3) >> 2;
    const int full_steps = (int)(K >> 8);           // steps whose 256 columns all exist
    const int tail_quads = 16 * (Kq - 4 * (steps - 1));
    const int64_t wstride = (int64_t)RB * 64;

    // ---- per-token output scale gamma * s_x / 127, once per tile ------------------------------------
    if (threadIdx.x < kGemmBM) {
        const int m = min(row0 + (int)threadIdx.x, M - 1);
        scale_lds[threadIdx.x] = gstride ? sx[m] / kQb : (gamma[0] * sx[m]) / kQb;
    }

    // ---- A operand, global -> LDS: this wave copies rows 8*kFM*wave .. +8*kFM-1 of the tile, 4 rows per load.
    // Lane i of a load writes LDS slot i: row (i >> 4) of the group, chunk slot (i & 15); the chunk that
    // belongs in slot c' of row m is c' ^ (m & 15).  Offsets are relative to the tile's first row.
    const int cp_row = lane >> 4, cp_slot = lane & 15;
    const int8_t* xtile = xq + (int64_t)row0 * K;
    const int rows_here = min(kGemmBM, M - row0);                   // rows past M: clamped, never stored
    uint32_t xoff[kCopies];
#pragma unroll
    for (int t = 0; t < kCopies; ++t) {
        const int row = copier * (4 * kCopies) + t * 4 + cp_row;
        xoff[t] = (uint32_t)min(row, rows_here - 1) * (uint32_t)K + (uint32_t)((cp_slot ^ (row & 15)) << 4);
    }
    // ---- A operand, LDS -> registers
    const int am = lane & 31, kg = lane >> 5;
    const int a_row_base = am * 256;                                 // + fm * 8192
    // ---- B operand: fragment fn covers row blocks 2*fn, 2*fn+1 of this wave's 2 * kFN
    const int brow = lane & 15, bsel = (lane >> 4) & 1;
    uint32_t woff[kFN][2];                                      // byte offsets of the lane's quads inside a whole step
#pragma unroll
    for (int fn = 0; fn < kFN; ++fn)
#pragma unroll
        for (int h = 0; h < 2; ++h)
            woff[fn][h] = ((uint32_t)min(bn * (8 * kFN) + wn * (2 * kFN) + fn * 2 + bsel, RB - 1) * 64u + (uint32_t)((kg + 2 * h) * 16 + brow)) * 16u;

    v16i acc[kFM][kFN];
#pragma unroll
    for (int fm = 0; fm < kFM; ++fm)
#pragma unroll
        for (int fn = 0; fn < kFN; ++fn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[fm][fn][v] = 0;

    // Per K step both operands are addressed as "scalar base of the step + fixed per-lane byte offset".  For
    // the activations that is a raw buffer whose base advances with the step (scalar arithmetic only) and whose
    // size shrinks with it, so the hardware range check still ends at the last byte of the tile's x_q rows
    // (reads past it return zero; in the partial last step the columns past K meet zero codes, whatever they
    // hold).
    const int64_t xbytes = (int64_t)rows_here * K;
    auto copy_x = [&](int step, int stage) {
        const int64_t left = xbytes - (int64_t)step * 256;
        const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<int8_t*>(xtile + (int64_t)step * 256), 0, (int)min(left, (int64_t)0x7FFFFFFF), 0x00020000);
        char* dst_stage = glds + stage * kGemmStageBytes;
#pragma unroll
        for (int t = 0; t < kCopies; ++t)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, (__attribute__((address_space(3))) void*)(dst_stage + (copier * (4 * kCopies) + t * 4) * 256),
                                                     16, xoff[t], 0, 0, 0);
    };
    // For the weights a raw buffer per step as well: one whole step of the packed layout (RB KiB), the lane's
    // byte offset in it as the vector offset -- no 64-bit address arithmetic per load.
    auto load_w = [&](uint4 (&wq)[kFN][2], int step) {
        const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint4*>(packed + (int64_t)step * wstride), 0, (int)(wstride * 16), 0x00020000);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int fn = 0; fn < kFN; ++fn) {
                const v4i q = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, (int)woff[fn][h], 0, 0));
                wq[fn][h] = make_uint4((uint32_t)q.x, (uint32_t)q.y, (uint32_t)q.z, (uint32_t)q.w);
            }
    };
    // the partial last step: its chunks hold fewer quads; lanes past them are clamped here and masked in compute()
    auto load_w_tail = [&](uint4 (&wq)[kFN][2], int step) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int ln = min((kg + 2 * h) * 16 + brow, tail_quads - 1);
#pragma unroll
            for (int fn = 0; fn < kFN; ++fn) {
                const int rb = min(bn * (8 * kFN) + wn * (2 * kFN) + fn * 2 + bsel, RB - 1);
                wq[fn][h] = packed[(int64_t)step * wstride + (int64_t)rb * tail_quads + ln];
            }
        }
    };

    // One K step: 8 slices of 32 columns, slice (h, j) uses word j of quad h; the LDS reads and the
    // decode for slice t + 1 are placed among the MFMAs of slice t.
    auto compute = [&](const uint4 (&wq)[kFN][2], const uint32_t (&km)[2], int stage) {
        const char* src = glds + stage * kGemmStageBytes + a_row_base;
        const int sw = am & 15;
        v4i a[2][kFM], b[2][kFN];
        auto read_a = [&](v4i (&dst)[kFM], int t) {
            const int chunk = 8 * (t >> 2) + 4 * kg + (t & 3);
#pragma unroll
            for (int fm = 0; fm < kFM; ++fm)
                dst[fm] = *reinterpret_cast<const v4i*>(src + fm * 8192 + ((chunk ^ sw) << 4));
        };
        auto word_of = [&](int fn, int t) { return gemm_quad_word(wq[fn][t >> 2], t & 3); };
        read_a(a[0], 0);
#pragma unroll
        for (int fn = 0; fn < kFN; ++fn) {
            const uint32_t w = word_of(fn, 0);
#pragma unroll
            for (int i = 0; i < 4; ++i) b[0][fn][i] = gemm_decode_reg(w, i, km[0]);
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int cur = t & 1, nxt = cur ^ 1;
            __builtin_amdgcn_sched_barrier(0);          // slices stay in order: no hoisting of later LDS reads
            if (t < 7) read_a(a[nxt], t + 1);
            __builtin_amdgcn_sched_barrier(0);          // ... and no sinking: the reads lead their use by a whole slice
            constexpr int kMfmas = kFM * kFN, kRegs = 4 * kFN;
#pragma unroll
            for (int q = 0; q < kMfmas; ++q) {
                const int fm = q / kFN, fn = q % kFN;
                acc[fm][fn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[cur][fm], b[cur][fn], acc[fm][fn], 0, 0, 0);
                if (t < 7) {                                        // the next slice's decode, spread over the MFMAs
#pragma unroll
                    for (int d = q * kRegs / kMfmas; d < (q + 1) * kRegs / kMfmas; ++d)
                        b[nxt][d >> 2][d & 3] = gemm_decode_reg(word_of(d >> 2, t + 1), d & 3, km[(t + 1) >> 2]);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // One loop body for every step: operands of step s + 1 are requested right before step s is
    // consumed (activations into the other LDS stage, weights into the other of two register sets), and the
    // barrier at the top of the next step both publishes them and retires the stage that was just read.  The
    // loop is unrolled by two so that the two register sets swap roles by name: copying the landed quads into
    // a working set cost 32 moves per step.
    uint4 wa[kFN][2], wb[kFN][2];
    const uint32_t keep_t0 = (kg * 16 + brow) < tail_quads ? 0xC0C0C0C0u : 0u;
    const uint32_t keep_t1 = ((kg + 2) * 16 + brow) < tail_quads ? 0xC0C0C0C0u : 0u;
    // This group's run of K steps.  Every group walks the same number of loop iterations, `per_group`, so that all
    // waves of the workgroup meet at the same barriers; a group whose run is shorter (or empty) idles through the rest.
    const int per_group = (step1 - step0 + kKG - 1) / kKG;
    const int my0 = step0 + grp * per_group, my1 = min(step1, my0 + per_group);
    auto issue = [&](uint4 (&into)[kFN][2], int step) {
        copy_x(step, (step - my0) & 1);
        if (step < full_steps) load_w(into, step); else load_w_tail(into, step);
    };
    auto one_step = [&](uint4 (&wcur)[kFN][2], uint4 (&wnxt)[kFN][2], int s) {
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (s < my1) {
            // lanes past a partial last step get a zero decode constant
            const uint32_t all = s >= full_steps ? 0u : 0xC0C0C0C0u;   // uniform
            const uint32_t km[2] = {keep_t0 | all, keep_t1 | all};
            if (s + 1 < my1) issue(wnxt, s + 1);
            compute(wcur, km, (s - my0) & 1);
        }
    };
    if (my0 < my1) issue(wa, my0);
    int it = 0;
#pragma unroll 1
    for (; it + 1 < per_group; it += 2) {
        one_step(wa, wb, my0 + it);
        one_step(wb, wa, my0 + it + 1);
    }
    if (it < per_group) one_step(wa, wb, my0 + it);
    __syncthreads();                                    // every wave is done with the activation stages

    if (kKG > 1) {
        // Fold the K groups: group 1 parks its accumulators in LDS (over the stages), group 0 adds them -- integer
        // sums, the same result as one group walking all of K.  Group 1 leaves after the last barrier; what follows
        // synchronises inside single waves only.
        int* fold = reinterpret_cast<int*>(lds);
        const int t = threadIdx.x & (kGemmThreads - 1);
        if (grp == 1) {
#pragma unroll
            for (int fm = 0; fm < kFM; ++fm)
#pragma unroll
                for (int fn = 0; fn < kFN; ++fn)
#pragma unroll
                    for (int v = 0; v < 16; ++v) fold[((fm * kFN + fn) * 16 + v) * kGemmThreads + t] = acc[fm][fn][v];
        }
        __syncthreads();
        if (grp == 0) {
#pragma unroll
            for (int fm = 0; fm < kFM; ++fm)
#pragma unroll
                for (int fn = 0; fn < kFN; ++fn)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[fm][fn][v] += fold[((fm * kFN + fn) * 16 + v) * kGemmThreads + t];
        }
        __syncthreads();                                // the fold area is free: the epilogue stages through it
        if (grp != 0) return;
    }

    // ---- epilogue: one instantiation per output type, chosen once ---------------------------------------
    const GemmOutCtx ctx{lds, scale_lds, y, gamma, gstride, RB, M, N, row0, bn, wave, lane, vec_store, kNG > 1 ? wave_all : wave};
    if (yt == OutType::BF16) gemm_epilogue<OutType::BF16, kFM, kFN>(acc, ctx);
    else if (yt == OutType::F32) gemm_epilogue<OutType::F32, kFM, kFN>(acc, ctx);
    else gemm_epilogue<OutType::I32, kFM, kFN>(acc, ctx);
#endif
}

// Consecutive workgroups take consecutive token tiles of the same weight tile (see the header).  Workgroups per
// CU: what the registers and the LDS stages allow (two with the tall wide tiles, up to four with 64-token tiles);
// one for the eight-wave form, which exists for grids that give a CU one workgroup anyway.
constexpr int gemm_blocks_per_cu(int fm, int fn) { return fn == 1 ? (fm == 2 ? 4 : fm == 3 ? 3 : 2) : (fm == 2 ? 3 : 2); }

// blockIdx.y selects a split of the K steps (split-K: every split stores its int32 partial accumulators, [M][N] each,
// one after the other at y; a second kernel adds them up and rescales).  One split: the whole product, stored as yt.
template <int kFM, int kFN, int kKG = 1, int kNG = 1>
__global__ __launch_bounds__(kGemmThreads * kKG * kNG, kKG * kNG > 1 ? 1 : gemm_blocks_per_cu(kFM, kFN)) void linear_gemm_2bit(
        const int8_t* __restrict__ xq, const float* __restrict__ sx, const uint4* __restrict__ packed,
        const float* __restrict__ gamma, int gstride, int M, int64_t N, int64_t K, int Kq, int RB, int tiles_m,
        int steps_per_split, void* __restrict__ y, OutType yt, int vec_store) {
    const int b = blockIdx.x;
    const int steps = (Kq + 3) >> 2;
    const int step0 = blockIdx.y * steps_per_split;
    const int step1 = min(steps, step0 + steps_per_split);
    void* yp = static_cast<char*>(y) + (int64_t)blockIdx.y * M * N * 4;        // blockIdx.y > 0 only with int32 partials
    gemm_tile<kFM, kFN, kKG, kNG>(xq, sx, packed, gamma, gstride, M, N, K, Kq, RB, (b % tiles_m) * (32 * kFM), b / tiles_m, step0, step1,
                        yp, yt, vec_store);
}

// split-K, second kernel: y[m][n] = (sum over the splits of the partial accumulators) * gamma * s_x[m] / 127, four
// consecutive outputs per thread.  Integer sums: exact and independent of the number of splits.
__global__ __launch_bounds__(256) void gemm_splitk_reduce(const int32_t* __restrict__ part, int splits, const float* __restrict__ sx,
                                                          const float* __restrict__ gamma, int gstride, int prefill_assoc,
                                                          int64_t M, int64_t N, void* __restrict__ y, OutType yt) {
    const int64_t quads_per_row = (N + 3) >> 2;
    const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (q >= M * quads_per_row) return;
    const int64_t m = q / quads_per_row, n0 = (q - m * quads_per_row) * 4;
    int acc[4] = {0, 0, 0, 0};
    for (int p = 0; p < splits; ++p) {
        const int32_t* src = part + ((int64_t)p * M + m) * N + n0;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (n0 + e < N) acc[e] += src[e];
    }
    const float sxm = yt == OutType::I32 ? 0.0f : sx[m];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (n0 + e >= N) continue;
        const int64_t o = m * N + n0 + e;
        if (yt == OutType::I32) { static_cast<int32_t*>(y)[o] = acc[e]; continue; }
        // the same association as the one-launch epilogue of the kernel that wrote the partials (the prefill kernel
        // with per-block gamma: gamma * (s_x / 127); otherwise (gamma * s_x) / 127), so that splitting never changes
        // a bit of the output
        const float gm = gamma[gstride ? (n0 + e) / kRowsPerBlock : 0];
        const float scale = (gstride && prefill_assoc) ? gm * (sxm / kQb) : (gm * sxm) / kQb;
        const float v = (float)acc[e] * scale;
        if (yt == OutType::F32) static_cast<float*>(y)[o] = v;
        else static_cast<uint16_t*>(y)[o] = f32_to_bf16(v);
    }
}

hipError_t launch_splitk_reduce(const int32_t* part, int splits, const float* sx, const float* gamma, int gstride,
                                int prefill_assoc, int64_t M, int64_t N, void* y, OutType yt, hipStream_t stream) {
    const int64_t quads = M * ceil_div(N, 4);
    hipLaunchKernelGGL(gemm_splitk_reduce, dim3((unsigned)ceil_div(quads, 256)), dim3(256), 0, stream, part, splits, sx, gamma,
                       gstride, prefill_assoc, M, N, y, yt);
    return hipGetLastError();
}

bool gemm_supports(int64_t M, int64_t N, int64_t K, const void* xq) {
    // per-lane activation offsets are 32-bit and relative to the tile's first row (128 * K fits for every K the
    // library accepts); one K step of the packed weights (1 KiB per 16-row block) is addressed as one raw buffer
    return M >= 1 && K % 16 == 0 && reinterpret_cast<uintptr_t>(xq) % 16 == 0 && ceil_div(N, kRowsPerBlock) < ((int64_t)1 << 21);
}

template <int kFM, int kFN, int kKG = 1, int kNG = 1>
static hipError_t launch_gemm_tiles(const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                                    int gstride, int64_t M, int64_t N, int64_t K, void* y, OutType yt,
                                    hipStream_t stream, int splits = 1, void* workspace = nullptr, LaunchPlan* plan = nullptr) {
    if (!plan) {
        static RaisedFlags raised = {};
        const hipError_t e = raise_dynamic_lds(reinterpret_cast<const void*>(linear_gemm_2bit<kFM, kFN, kKG, kNG>), gemm_lds_bytes(kFM, kFN, kKG, kNG), raised);
        if (e != hipSuccess) return e;
    }
    const int Kq = (int)ceil_div(K, kColsPerQuad);
    const int RB = (int)ceil_div(N, kRowsPerBlock);
    const int tiles_m = (int)ceil_div(M, 32 * kFM);
    const int64_t tiles_n = ceil_div(N, 128 * kFN * kNG);
    const int steps = (int)ceil_div(K, 256);
    if (splits > steps) splits = steps;
    const int sps = (int)ceil_div(steps, splits);
    splits = (int)ceil_div(steps, sps);                 // no empty split
    const bool split = splits > 1;
    void* out = split ? workspace : y;
    const OutType ot = split ? OutType::I32 : yt;
    const size_t esz = ot == OutType::BF16 ? 2 : 4;
    const int vec_store = (reinterpret_cast<uintptr_t>(out) % 16 == 0) && ((N * esz) % 16 == 0);
    if (plan) {
        if (kNG > 1) plan->set("prefill", {32 * kFM, 128 * kFN * kNG}, (unsigned)(tiles_m * tiles_n), (unsigned)splits, kGemmThreads * kNG, gemm_lds_bytes(kFM, kFN, 1, kNG), splits);
        else if (kKG > 1) plan->set("prefill", {32 * kFM, 128 * kFN, kKG}, (unsigned)(tiles_m * tiles_n), (unsigned)splits, kGemmThreads * kKG, gemm_lds_bytes(kFM, kFN, kKG), splits);
        else plan->set("prefill", {32 * kFM, 128 * kFN}, (unsigned)(tiles_m * tiles_n), (unsigned)splits, kGemmThreads, gemm_lds_bytes(kFM, kFN, 1), splits);
        return hipSuccess;
    }
    hipLaunchKernelGGL((linear_gemm_2bit<kFM, kFN, kKG, kNG>), dim3((unsigned)(tiles_m * tiles_n), (unsigned)splits), dim3(kGemmThreads * kKG * kNG),
                       gemm_lds_bytes(kFM, kFN, kKG, kNG), stream, xq, sx, static_cast<const uint4*>(packed), gamma, gstride, (int)M, N, K, Kq, RB,
                       tiles_m, sps, out, ot, vec_store);
    if (split)
        return launch_splitk_reduce(static_cast<const int32_t*>(workspace), splits, sx, gamma, gstride, 1, M, N, y, yt, stream);
    return hipGetLastError();
}

// tile shape forced by the caller (tuning and tests); fm in 2 .. 4, fn in 1 .. 2; kg 1, or 2 (two K groups per workgroup:
// 96 x 128 and 64 x 256 tiles only, one launch only), or 3 (two row groups per workgroup, 32 fm x 512 tiles: fn == 2
// and fm == 4 only); splits > 1: split-K through `workspace` (splits * M * N int32)
hipError_t launch_linear_gemm_2bit_shape(int fm, int fn, int kg, const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                                         int gstride, int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream,
                                         int splits, void* workspace, LaunchPlan* plan) {
#define GEMM_SHAPE(FM_, FN_, KG_) if (fm == FM_ && fn == FN_ && kg == KG_) return launch_gemm_tiles<FM_, FN_, KG_ == 2 ? 2 : 1, KG_ == 3 ? 2 : 1>(xq, sx, packed, gamma, gstride, M, N, K, y, yt, stream, splits, workspace, plan)
    if (kg != 1 && splits > 1) return hipErrorInvalidValue;           // the eight-wave forms: one launch only
    GEMM_SHAPE(2, 1, 1); GEMM_SHAPE(3, 1, 1); GEMM_SHAPE(4, 1, 1); GEMM_SHAPE(2, 2, 1); GEMM_SHAPE(3, 2, 1); GEMM_SHAPE(4, 2, 1);
    GEMM_SHAPE(3, 1, 2); GEMM_SHAPE(2, 2, 2);
    GEMM_SHAPE(4, 2, 3);
#undef GEMM_SHAPE
    return hipErrorInvalidValue;
}

size_t splitk_workspace_bytes(int64_t M, int64_t N, int splits) { return (size_t)splits * (size_t)M * (size_t)N * 4; }

hipError_t launch_linear_gemm_2bit(const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                                   int gstride, int64_t M, int64_t N, int64_t K, void* y, OutType yt,
                                   hipStream_t stream, void* workspace, size_t workspace_bytes, int force_splits,
                                   LaunchPlan* plan) {
    // Tile shape (32 * fm tokens x 128 * fn weight rows) from a cost model fitted to measurements on MI355X
    // (nine LLaMA-family shapes, M = 65 ... 2048, every tile shape).  In microseconds, per K step of 256 columns:
    //   * a workgroup that has its CU to itself is latency bound and takes kAlone per step, a little more as the
    //     chip fills up (tiles are not dealt perfectly evenly);
    //   * a CU that holds n tiles is throughput bound at n * kSaturated per step; per unit of work the three wide
    //     shapes cost the same there and the narrow ones 12-18 % more, so the narrow shapes win exactly where the
    //     wide ones would leave most CUs idle (N <= 8192, or a few hundred tokens);
    //   * kFixed covers launch, prologue and epilogue.
    // Ties within 4 % go to the larger tile (less decode work and fewer activation re-reads per output).
    // Examples (13B o projection, N = K = 5120): M = 512 runs 96 x 128 tiles in 19.6 us (64 x 256: 23.6 us,
    // 128 x 256: 36 us); M = 2048 stays on 96 x 256 tiles.  (Up to 256 tokens such small layers go to the
    // batched-decode kernels instead, which tile the tokens over workgroups.)
    // Where one launch of four-wave workgroups gives no CU more than one of them, the 96 x 128 and 64 x 256 tiles also
    // exist with eight waves in two K groups (13B O / down at 512 tokens: 19.1 -> 17.9 us, 40.2 -> 36.6 us; 8192 rows,
    // K = 28672, 300 tokens: 99 -> 75 us): ceil(steps / 2) iterations of kPair[] us each and a fold, in kPairFixed; a CU
    // holds one such workgroup, so they are candidates only while the tiles fit the chip in one round.
    // With a workspace the K steps may also be split over 2, 4 or 8 workgroups per tile (each stores int32 partial
    // accumulators, a second launch adds them and rescales): the same model with steps / splits per workgroup and
    // tiles * splits workgroups, plus the second launch (a few microseconds and the partials' traffic).  It pays where
    // even the smallest tiles leave CUs idle and K is long.
    struct Shape { int fm, fn; double alone, saturated, fixed; };
    static const Shape kShapes[6] = {{4, 2, 1.48, 1.45, 5.4}, {3, 2, 1.15, 1.10, 4.7}, {2, 2, 0.94, 0.74, 4.4},
                                     {4, 1, 0.94, 0.86, 3.5}, {3, 1, 0.715, 0.613, 3.4}, {2, 1, 0.594, 0.43, 3.2}};
    struct PairShape { int fm, fn; double per_iteration, fixed; };
    static const PairShape kPair[2] = {{3, 1, 0.95, 7.0}, {2, 2, 1.10, 7.0}};
    const int64_t steps_total = ceil_div(K, 256);
    int best = 0, best_splits = 1, best_kg = 1;
    double best_cost = 0.0;
    for (int sp = 1; sp <= 8; sp *= 2) {
        if (force_splits > 0 && sp != force_splits) continue;
        if (sp > 1 && (!workspace || workspace_bytes < splitk_workspace_bytes(M, N, sp) || sp > steps_total)) continue;
        const double steps = (double)ceil_div(steps_total, (int64_t)sp);
        const double second = sp > 1 ? 4.5 + (double)(sp + 1) * (double)M * (double)N * 4.0 / 3.0e6 : 0.0;   // launch + partials at 3 TB/s
        for (int c = 0; c < 6; ++c) {                   // largest tile first
            const Shape& sh = kShapes[c];
            const int64_t tiles = ceil_div(M, 32 * sh.fm) * ceil_div(N, 128 * sh.fn) * sp;
            const double fill = (double)tiles / 256.0;
            const double alone = sh.alone * (1.0 + 0.2 * (fill < 1.0 ? fill * fill : 1.0));
            const double shared = (double)ceil_div(tiles, (int64_t)256) * sh.saturated;
            const double cost = sh.fixed + steps * (alone > shared ? alone : shared) + second;
            if ((sp == 1 && c == 0) || (force_splits > 0 && sp == force_splits && c == 0) || cost < 0.96 * best_cost) {
                best = c; best_splits = sp; best_kg = 1; best_cost = cost;
            }
        }
    }
    int fm = kShapes[best].fm, fn = kShapes[best].fn;
    if (force_splits <= 0) {
        for (int c = 0; c < 2; ++c) {
            const PairShape& sh = kPair[c];
            const int64_t tiles = ceil_div(M, 32 * sh.fm) * ceil_div(N, 128 * sh.fn);
            if (tiles > 256 || steps_total < 2) continue;
            const double fill = (double)tiles / 256.0;
            const double cost = sh.fixed + (double)ceil_div(steps_total, (int64_t)2) * sh.per_iteration * (1.0 + 0.2 * fill * fill);
            if (cost < 0.96 * best_cost) { fm = sh.fm; fn = sh.fn; best_splits = 1; best_kg = 2; best_cost = cost; }
        }
    }
    // Two row groups on one token tile (128 x 512, eight waves, one workgroup per CU): 2.70 us per K step, against 2.9 for
    // two 128 x 256 workgroups on a CU, because the CU fetches the activations once for both.  Rounds are whole here --
    // a CU cannot take half a tile while the last round drains -- so it wins where the count of tiles suits 256 CUs
    // (13B-class QKV at 2048 tokens, 480 tiles: 127 -> 116 us) and loses where it does not (gate/up there, 864 tiles:
    // 200 -> 220 us); not considered while its tiles fill less than 7/8 of the CUs, where four-wave workgroups spread over more
    // of them (240 tiles: 65 -> 62.5 us; 216 tiles: 58 -> 59 us; 192 tiles: 42 -> 46 us).
    if (force_splits <= 0) {
        const int64_t tiles = ceil_div(M, 128) * ceil_div(N, 512);
        const double cost = 6.0 + (double)steps_total * (double)ceil_div(tiles, (int64_t)256) * 2.70;
        if (tiles >= 224 && cost < 0.96 * best_cost) { fm = 4; fn = 2; best_splits = 1; best_kg = 3; best_cost = cost; }
    }
    return launch_linear_gemm_2bit_shape(fm, fn, best_kg, xq, sx, packed, gamma, gstride, M, N, K, y, yt, stream, best_splits, workspace, plan);
}

}  // namespace bitnet

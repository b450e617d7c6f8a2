// Weight-streaming BitLinear kernels for batched decode (4 < M <= 64) on gfx950: the same packed layout, decode
// and v_mfma_i32_16x16x64_i8 contraction as the decode kernel (linear_gemv.hip), with the activations of a K step
// staged once per group of waves through LDS.  acc[m][n] = sum_k x_q[m][k] * Wt[n][k] exactly in int32 and
// y = acc * gamma * s_x[m] / 127 (Sections 1-2 of arXiv 2402.17764).
#include "gemv_common.hpp"

namespace bitnet {

// ---------------------------------------------------------------------------------------------------
// 4 < M <= 64: the skinny kernel
// ---------------------------------------------------------------------------------------------------
// Between decode and prefill the weights are still streamed once from HBM, but every wave now needs
// 16 * kMT tokens x 256 bytes of activations for each K step (kMT = 1, 2 or 4 tiles of 16 tokens), more
// than the 1 KiB of weights a row block contributes.  A workgroup is kS groups of kW waves:
//   * a group owns a contiguous range of K steps and walks it in lock-step; the x_q rows of a step are
//     copied global -> LDS once per group with buffer loads (XOR-swizzled 16-byte chunks, read back with
//     conflict-free ds_read_b128), kLx steps ahead, through a ring of kLx + 1 stages;
//   * each wave owns kR row blocks, prefetches their quads kD steps ahead in registers and uses one
//     activation operand read from LDS for all kR of them (LDS bandwidth, not HBM, is the next limit:
//     16 * kMT / kR KiB of LDS reads per KiB of weights);
//   * the groups' partial accumulators are folded through LDS in a fixed order at the end.
// The workgroup covers kW * kR row blocks for all of K, so the host picks kR and kW to make the number
// of workgroups fit the CUs, and kS * kW * kR * kD KiB of weights are in flight per workgroup.
//
// Waiting: LDS-DMA completion is counted by vmcnt together with the weight loads, in issue order.  The
// prologue issues copies and weight loads in exactly the order of the loop body, so from the first
// step on the loads younger than this wave's copy for the current step number kSkinnyYounger, and an
// explicit s_waitcnt with that count retires the copy without draining the prefetch behind it.  The
// scheduling fences keep the compiler from moving loads across the counted wait; the barrier is the
// bare instruction because a fence-carrying barrier makes the compiler wait for every LDS-DMA load.
// The count holds only while the loop issues no other vector-memory instruction, i.e. while nothing spills:
// the build checks that every instantiation compiles without scratch memory.
template <int kMT, int kR, int kW, int kS, int kD, int kLx>
__global__ __launch_bounds__(kS * kW * kWave) void linear_skinny_2bit(
        const int8_t* __restrict__ xq_all, const float* __restrict__ sx_all, const uint4* __restrict__ packed,
        const float* __restrict__ gamma, int gstride, int M_all /* blockIdx.z selects a tile of 16 * kMT tokens */,
        int64_t N, int64_t K, int Kq, int RB, int spg,
        int steps_per_split /* blockIdx.y selects a run of K steps (split-K: int32 partials, [M][N] each, one after the
                               other at yv); one split: all steps */,
        void* __restrict__ yv, OutType yt) {
#if defined(__HIP_DEVICE_COMPILE__)      // the buffer-resource builtins exist in the device pass only
    extern __shared__ uint4 smem[];
    constexpr int kRing = kLx + 1;                     // LDS stages per group
    constexpr int kStageBytes = kMT * 16 * 256;        // tokens staged per step x 256 columns
    constexpr int kGroupBytes = kRing * kStageBytes;
    constexpr int kCopies = kMT * 4;                   // 1 KiB wave-loads per stage (4 token rows each)
    constexpr int kC = kCopies / kW;                   // ... issued by each wave of the group
    constexpr int kYounger = kR + (kLx - 1) * (kC + kR);
    static_assert(kCopies % kW == 0, "every wave issues the same number of copies: no guard, no branch");
    static_assert(kLx >= 1 && kLx <= kD, "activations are never requested before the weights of their step");
    static_assert(kYounger < 64, "vmcnt is six bits");
    static_assert((kS - 1) * kW * kR * kMT * 1024 <= kS * kGroupBytes, "the fold reuses the activation ring");
    char* lds = reinterpret_cast<char*>(smem);

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: LDS-DMA targets need no broadcast
    const int ks = wave / kW, wv = wave - ks * kW;     // K group, wave within the group
    const int r = lane & 15, g = lane >> 4;
    const int steps = (Kq + 3) >> 2;
    const int tail_quads = 16 * (Kq - 4 * (steps - 1));
    const int step0 = blockIdx.y * steps_per_split, step1 = min(steps, step0 + steps_per_split);
    // this workgroup's tokens: tile blockIdx.z of 16 * kMT (the launcher may tile M finer than it has to: with few row
    // blocks several workgroups that each stage a quarter of x_q move less through the L2 than one that stages all)
    const int m0 = blockIdx.z * (16 * kMT);
    const int M = min(M_all - m0, 16 * kMT);
    const int8_t* xq = xq_all + (int64_t)m0 * K;
    const float* sx = sx_all + m0;
    void* y = static_cast<char*>(yv) + (int64_t)blockIdx.y * M_all * N * 4 + (int64_t)m0 * N * (yt == OutType::BF16 ? 2 : 4);
    const int s_begin = step0 + ks * spg;                              // this group's steps: s_begin + [0, n_here)
    const int n_here = max(0, min(spg, step1 - s_begin));
    const int rbw = (blockIdx.x * kW + wv) * kR;
    const int64_t wstride = (int64_t)RB * 64;
    char* glds = lds + ks * kGroupBytes;

    // activation copy: lane i of a load fills slot i = (row i >> 4 of a group of four, chunk slot i & 15);
    // the chunk stored in slot c' of token m is c' ^ (m & 15).  The whole byte offset travels in the vector
    // offset, which the hardware range check covers: reads past the end of x_q return zero.
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t*>(xq), 0, (int)min((int64_t)M * K, (int64_t)0x7FFFFFFF), 0x00020000);
    uint32_t xoff[kC];
#pragma unroll
    for (int t = 0; t < kC; ++t) {
        const int row = (wv + t * kW) * 4 + (lane >> 4);
        xoff[t] = (uint32_t)min(row, M - 1) * (uint32_t)K + (uint32_t)(((lane & 15) ^ (row & 15)) << 4) +
                  (uint32_t)s_begin * 256u;
    }
    auto copy_x = [&](int i, int stage) {                              // local step i of this group
#pragma unroll
        for (int t = 0; t < kC; ++t)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                xrsrc, (__attribute__((address_space(3))) void*)(glds + stage * kStageBytes + (wv + t * kW) * 1024),
                16, xoff[t] + (uint32_t)i * 256u, 0, 0, 0);
    };

    // weight quads: one K step of the packed layout as a raw buffer (scalar base per step) plus a 32-bit byte
    // offset per lane; a row block's chunk is 64 quads in a whole step, tail_quads in a partial last one, and
    // lanes past it are clamped here and masked in compute()
    int rbc[kR];
    uint32_t woff_full[kR], woff_tail[kR];
#pragma unroll
    for (int a = 0; a < kR; ++a) {
        rbc[a] = min(rbw + a, RB - 1);
        woff_full[a] = ((uint32_t)rbc[a] * 64u + (uint32_t)lane) * 16u;
        woff_tail[a] = ((uint32_t)rbc[a] * (uint32_t)tail_quads + (uint32_t)min(lane, tail_quads - 1)) * 16u;
    }
    auto load_w = [&](uint4 (&w)[kR], int i) {
        const int sl = min(s_begin + i, steps - 1);                    // past the end: redirected, masked below
        const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint4*>(packed + (int64_t)sl * wstride), 0, (int)(wstride * 16), 0x00020000);
        const bool tail = sl == steps - 1;
#pragma unroll
        for (int a = 0; a < kR; ++a) {
            const v4i q = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, (int)(tail ? woff_tail[a] : woff_full[a]), 0, 0));
            w[a] = make_uint4((uint32_t)q.x, (uint32_t)q.y, (uint32_t)q.z, (uint32_t)q.w);
        }
    };

    v4i acc[kR][kMT];
#pragma unroll
    for (int a = 0; a < kR; ++a)
#pragma unroll
        for (int t = 0; t < kMT; ++t) acc[a][t] = (v4i){0, 0, 0, 0};

    auto compute = [&](const uint4 (&w)[kR], int i, int stage) {
        const int cq = s_begin + i == steps - 1 ? tail_quads : 64;
        const uint32_t km = (i < n_here && lane < cq) ? 0xC0C0C0C0u : 0u;     // padded steps contribute nothing
        const char* src = glds + stage * kStageBytes + r * 256;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v4i A[kR];
#pragma unroll
            for (int a = 0; a < kR; ++a) A[a] = decode_word_masked(quad_word(w[a], j), km);
            const int slot = ((4 * g + j) ^ r) << 4;
#pragma unroll
            for (int t = 0; t < kMT; ++t) {
                const v4i X = *reinterpret_cast<const v4i*>(src + t * 4096 + slot);
#pragma unroll
                for (int a = 0; a < kR; ++a)
                    acc[a][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[a], X, acc[a][t], 0, 0, 0);
            }
        }
    };

    // The output scales are requested before anything else (loaded after the fold they would add a cache round
    // trip to the tail of the kernel); being the oldest loads in flight they never disturb the counted waits.
    float gm[kR] = {}, sxm[kMT] = {};
    if (ks == 0) {                                                     // the group that writes the output
#pragma unroll
        for (int a = 0; a < kR; ++a) gm[a] = gamma[gstride * rbc[a]];
#pragma unroll
        for (int t = 0; t < kMT; ++t) sxm[t] = yt == OutType::I32 ? 0.0f : sx[min(16 * t + r, M - 1)];
    }
    issue_fence();

    // Prologue: the issue pattern of steps -kD ... -1 of the loop below.  Where the loop would copy a
    // step before the first, step 0 is copied (again) so that the count of loads in flight is the same.
    uint4 wst[kD][kR];
#pragma unroll
    for (int p = 0; p < kD; ++p) {
        constexpr int kLead = kD - kLx;
        const int xs = p >= kLead ? p - kLead : 0;
        copy_x(xs, xs % kRing);
        issue_fence();                                                 // the counted wait relies on this issue order
        load_w(wst[p], p);
        issue_fence();
    }

    // Steps are walked in groups of kD so that the register stages are indexed statically; the count is
    // padded to a whole group with steps whose weights are masked to zero, so the body has no guards.
    const int padded = (spg + kD - 1) / kD * kD;                      // >= kD: the loop runs at least once
    int i0 = 0;
    do {
#pragma unroll
        for (int d = 0; d < kD; ++d) {
            const int i = i0 + d;
            // loads issued after this wave's copy for step i: kR weight loads, then for each of the next
            // kLx - 1 steps kC copies and kR weight loads
            // (imm: vmcnt[3:0] | expcnt 7 << 4 | lgkmcnt 15 << 8 | vmcnt[5:4] << 14)
            issue_fence();
            __builtin_amdgcn_s_waitcnt((kYounger & 15) | 0x0F70 | ((kYounger >> 4) << 14));
            __builtin_amdgcn_s_barrier();                              // stage i is complete, stage i - 1 is free
            issue_fence();
            copy_x(i + kLx, (i + kLx) % kRing);
            issue_fence();                                             // copies first: the wait above counts on it
            compute(wst[d], i, i % kRing);
            load_w(wst[d], i + kD);                                    // after the last use: reloaded in place
        }
        i0 += kD;
    } while (i0 < padded);
    issue_fence();

    if constexpr (kS > 1) {
        // fold the K groups: groups 1 ... kS - 1 park their accumulators in LDS, group 0 adds them in order
        __builtin_amdgcn_s_waitcnt(0);                                 // copies past the end have landed
        __syncthreads();
        v4i* fold = reinterpret_cast<v4i*>(lds);
        if (ks > 0) {
#pragma unroll
            for (int a = 0; a < kR; ++a)
#pragma unroll
                for (int t = 0; t < kMT; ++t)
                    fold[((((ks - 1) * kW + wv) * kR + a) * kMT + t) * kWave + lane] = acc[a][t];
        }
        __syncthreads();
        if (ks > 0) return;
        for (int q = 0; q < kS - 1; ++q)
#pragma unroll
            for (int a = 0; a < kR; ++a)
#pragma unroll
                for (int t = 0; t < kMT; ++t)
                    acc[a][t] += fold[(((q * kW + wv) * kR + a) * kMT + t) * kWave + lane];
    }

#pragma unroll
    for (int t = 0; t < kMT; ++t) {
        const int m = 16 * t + r;                                      // MFMA output column = token
        if (m >= M) continue;
#pragma unroll
        for (int a = 0; a < kR; ++a) {
            const float scale = (gm[a] * sxm[t]) / kQb;
            const int64_t n0 = (int64_t)(rbw + a) * 16 + 4 * g;
            if (n0 < N) store_row4(y, yt, (int64_t)m * N + n0, n0, N, acc[a][t], scale);
        }
    }
#endif
}

// ---------------------------------------------------------------------------------------------------
// The skinny kernel with a loader wave (larger token tiles)
// ---------------------------------------------------------------------------------------------------
// With 32 or 64 tokens the LDS ring of the kernel above holds two or three steps of activations at most, and
// because LDS-DMA copies and weight loads retire through one in-order counter, waiting for a step's copy also
// drains every weight load issued before it: no more than kLx steps of weights are ever in flight, and the
// waves spend 40-60 % of their cycles in s_waitcnt (measured).  Here the two streams get separate waves:
//   * one loader wave per workgroup issues all LDS-DMA copies (every K group's stage of a step), waits for
//     them with an exact count -- its counter sees nothing but copies -- and publishes each step at the barrier;
//   * the kS * kW compute waves never wait for a copy: their counter tracks weight quads only, so the
//     compiler's own waits leave kD - 1 steps of weights in flight per wave.
// Everything else (K groups, kR row blocks per wave, swizzled LDS tiles, fold) is as above.
template <int kMT, int kR, int kW, int kS, int kD, int kLx>
__global__ __launch_bounds__((kS * kW + 1) * kWave) void linear_skinny_ws_2bit(
        const int8_t* __restrict__ xq_all, const float* __restrict__ sx_all, const uint4* __restrict__ packed,
        const float* __restrict__ gamma, int gstride, int M_all, int64_t N, int64_t K, int Kq, int RB, int spg,
        int steps_per_split /* as in linear_skinny_2bit */, void* __restrict__ yv, OutType yt) {
#if defined(__HIP_DEVICE_COMPILE__)      // the buffer-resource builtins exist in the device pass only
    extern __shared__ uint4 smem[];
    constexpr int kRing = kLx + 1;                     // LDS stages per group
    constexpr int kStageBytes = kMT * 16 * 256;        // tokens staged per step x 256 columns
    constexpr int kGroupBytes = kRing * kStageBytes;
    constexpr int kCopies = kMT * 4;                   // 1 KiB wave-loads per stage (4 token rows each)
    constexpr int kYounger = (kLx - 1) * kS * kCopies; // copies issued after those of the step being awaited
    static_assert(kLx >= 1 && kYounger < 64, "vmcnt is six bits");
    static_assert((kS - 1) * kW * kR * kMT * 1024 <= kS * kGroupBytes, "the fold reuses the activation ring");
    char* lds = reinterpret_cast<char*>(smem);

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 15, g = lane >> 4;
    const int steps = (Kq + 3) >> 2;
    const int tail_quads = 16 * (Kq - 4 * (steps - 1));
    const int padded = (spg + kD - 1) / kD * kD;       // barriers per wave: the same for both roles
    const int step0 = blockIdx.y * steps_per_split, step1 = min(steps, step0 + steps_per_split);
    // this workgroup's tokens: tile blockIdx.z of 16 * kMT (the launcher may tile M finer than it has to: with few row
    // blocks several workgroups that each stage a quarter of x_q move less through the L2 than one that stages all)
    const int m0 = blockIdx.z * (16 * kMT);
    const int M = min(M_all - m0, 16 * kMT);
    const int8_t* xq = xq_all + (int64_t)m0 * K;
    const float* sx = sx_all + m0;
    void* y = static_cast<char*>(yv) + (int64_t)blockIdx.y * M_all * N * 4 + (int64_t)m0 * N * (yt == OutType::BF16 ? 2 : 4);

    v4i acc[kR][kMT];
#pragma unroll
    for (int a = 0; a < kR; ++a)
#pragma unroll
        for (int t = 0; t < kMT; ++t) acc[a][t] = (v4i){0, 0, 0, 0};
    int ks = 0, wv = 0, rbw = 0;
    float gm[kR] = {}, sxm[kMT] = {};                                  // output scales, requested ahead of the weights

    if (wave == kS * kW) {
        // ---- loader: lane i of a copy fills slot i = (row i >> 4 of a group of four token rows, chunk slot
        // i & 15); the chunk stored in slot c' of token m is c' ^ (m & 15).  Reads past x_q return zero.
        const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<int8_t*>(xq), 0, (int)min((int64_t)M * K, (int64_t)0x7FFFFFFF), 0x00020000);
        uint32_t xoff[kCopies];
#pragma unroll
        for (int t = 0; t < kCopies; ++t) {
            const int row = t * 4 + (lane >> 4);
            xoff[t] = (uint32_t)min(row, M - 1) * (uint32_t)K + (uint32_t)(((lane & 15) ^ (row & 15)) << 4);
        }
        auto copy_x = [&](int i, int stage) {                          // local step i of every group
#pragma unroll
            for (int q = 0; q < kS; ++q) {
                const uint32_t col = (uint32_t)(step0 + q * spg + i) * 256u;
#pragma unroll
                for (int t = 0; t < kCopies; ++t)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        xrsrc, (__attribute__((address_space(3))) void*)(lds + q * kGroupBytes + stage * kStageBytes + t * 1024),
                        16, xoff[t] + col, 0, 0, 0);
            }
        };
#pragma unroll
        for (int p = 0; p < kLx; ++p) {
            copy_x(p, p % kRing);
            issue_fence();                                             // step by step: the counted wait relies on it
        }
        for (int i = 0; i < padded; ++i) {
            issue_fence();
            __builtin_amdgcn_s_waitcnt((kYounger & 15) | 0x0F70 | ((kYounger >> 4) << 14));   // step i has landed
            __builtin_amdgcn_s_barrier();                              // publish it; stage i - 1 is free
            issue_fence();
            copy_x(i + kLx, (i + kLx) % kRing);
        }
        issue_fence();
    } else {
        // ---- compute waves
        ks = wave / kW;
        wv = wave - ks * kW;
        rbw = (blockIdx.x * kW + wv) * kR;
        const int s_begin = step0 + ks * spg;                          // this group's steps: s_begin + [0, n_here)
        const int n_here = max(0, min(spg, step1 - s_begin));
        const int64_t wstride = (int64_t)RB * 64;
        const char* glds = lds + ks * kGroupBytes;
        int rbc[kR];
        uint32_t woff_full[kR], woff_tail[kR];
#pragma unroll
        for (int a = 0; a < kR; ++a) {
            rbc[a] = min(rbw + a, RB - 1);
            woff_full[a] = ((uint32_t)rbc[a] * 64u + (uint32_t)lane) * 16u;
            woff_tail[a] = ((uint32_t)rbc[a] * (uint32_t)tail_quads + (uint32_t)min(lane, tail_quads - 1)) * 16u;
        }
        auto load_w = [&](uint4 (&w)[kR], int i) {
            const int sl = min(s_begin + i, steps - 1);                // past the end: redirected, masked below
            const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<uint4*>(packed + (int64_t)sl * wstride), 0, (int)(wstride * 16), 0x00020000);
            const bool tail = sl == steps - 1;
#pragma unroll
            for (int a = 0; a < kR; ++a) {
                const v4i q = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, (int)(tail ? woff_tail[a] : woff_full[a]), 0, 0));
                w[a] = make_uint4((uint32_t)q.x, (uint32_t)q.y, (uint32_t)q.z, (uint32_t)q.w);
            }
        };
        auto compute = [&](const uint4 (&w)[kR], int i, int stage) {
            const int cq = s_begin + i == steps - 1 ? tail_quads : 64;
            const uint32_t km = (i < n_here && lane < cq) ? 0xC0C0C0C0u : 0u; // padded steps contribute nothing
            const char* src = glds + stage * kStageBytes + r * 256;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v4i A[kR];
#pragma unroll
                for (int a = 0; a < kR; ++a) A[a] = decode_word_masked(quad_word(w[a], j), km);
                const int slot = ((4 * g + j) ^ r) << 4;
#pragma unroll
                for (int t = 0; t < kMT; ++t) {
                    const v4i X = *reinterpret_cast<const v4i*>(src + t * 4096 + slot);
#pragma unroll
                    for (int a = 0; a < kR; ++a)
                        acc[a][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[a], X, acc[a][t], 0, 0, 0);
                }
            }
        };
        if (ks == 0) {                                                 // the group that writes the output
#pragma unroll
            for (int a = 0; a < kR; ++a) gm[a] = gamma[gstride * rbc[a]];
#pragma unroll
            for (int t = 0; t < kMT; ++t) sxm[t] = yt == OutType::I32 ? 0.0f : sx[min(16 * t + r, M - 1)];
        }
        uint4 wst[kD][kR];
#pragma unroll
        for (int d = 0; d < kD; ++d) load_w(wst[d], d);
        int i0 = 0;
        do {
#pragma unroll
            for (int d = 0; d < kD; ++d) {
                const int i = i0 + d;
                __builtin_amdgcn_s_barrier();                          // stage i is complete
                compute(wst[d], i, i % kRing);
                load_w(wst[d], i + kD);                                // after the last use: reloaded in place
            }
            i0 += kD;
        } while (i0 < padded);
    }

    // fold the K groups (every wave meets the barriers; the loader has nothing to add)
    __builtin_amdgcn_s_waitcnt(0);                                     // copies past the end have landed
    __syncthreads();
    if constexpr (kS > 1) {
        v4i* fold = reinterpret_cast<v4i*>(lds);
        if (wave < kS * kW && ks > 0) {
#pragma unroll
            for (int a = 0; a < kR; ++a)
#pragma unroll
                for (int t = 0; t < kMT; ++t)
                    fold[((((ks - 1) * kW + wv) * kR + a) * kMT + t) * kWave + lane] = acc[a][t];
        }
        __syncthreads();
        if (wave >= kS * kW || ks > 0) return;
        for (int q = 0; q < kS - 1; ++q)
#pragma unroll
            for (int a = 0; a < kR; ++a)
#pragma unroll
                for (int t = 0; t < kMT; ++t)
                    acc[a][t] += fold[(((q * kW + wv) * kR + a) * kMT + t) * kWave + lane];
    } else {
        if (wave >= kS * kW) return;
    }

#pragma unroll
    for (int t = 0; t < kMT; ++t) {
        const int m = 16 * t + r;                                      // MFMA output column = token
        if (m >= M) continue;
#pragma unroll
        for (int a = 0; a < kR; ++a) {
            const float scale = (gm[a] * sxm[t]) / kQb;
            const int64_t n0 = (int64_t)(rbw + a) * 16 + 4 * g;
            if (n0 < N) store_row4(y, yt, (int64_t)m * N + n0, n0, N, acc[a][t], scale);
        }
    }
#endif
}

// ---------------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------------
constexpr int64_t kSkinnyMaxTokens = 512;      // beyond 64 tokens only where one round of workgroups exists (few row blocks)

// Token tile (16 * kmt tokens per workgroup, grid z walks the tiles) and row blocks per workgroup (rpw = kW * kR).
//   * One round of workgroups: the activation rings take 48-128 KB of LDS, so a CU often holds a single workgroup
//     and any beyond 256 run as a second round (600 workgroups of one row block: 9.3 us where 150 of four take
//     5.5 us); and where several do fit, a CU streams at a fixed rate however many it holds, so 288 workgroups leave
//     32 CUs with twice the work of the others (13B gate / up at 8 tokens: 14.0 us with six row blocks per workgroup,
//     9.5 us with eight).  So: the fewest row blocks per workgroup that give at most 256 workgroups; beyond 4096
//     row blocks sixteen, the most a form has.
//   * With few row blocks the traffic that counts is x_q through the L2s: every workgroup stages all K columns of
//     its tokens, 16 kmt K bytes against 4 K per row block of weights.  One tile of 64 tokens per workgroup and 256
//     workgroups of one row block move 17408 K bytes; four tiles of 16 tokens and 64 x 4 workgroups of four row
//     blocks move 8192 K (7B down projection at 64 tokens: 15.4 -> 10.0 us; 13B down at 48: 19.9 -> 11.2 us).  Up to
//     1024 row blocks the tile is therefore the one with the least such traffic among the one-round launches.
//   * The same tiling carries these kernels past 64 tokens: up to 256 tokens, where a one-round launch with at most
//     eight row blocks per workgroup exists (layers of up to 512-768 row blocks), they beat the prefill kernel, whose
//     tiles leave most CUs idle there (7B down at 128 tokens: 13.6 us against 35.9 us, 20.7 us with split-K; 70B O
//     at 256: 22.7 against 28.0 us).  Tiles of 32 tokens while six row blocks per workgroup suffice, else of 64:
//     the measured best on 30 of 36 cases.  From 257 to 512 tokens the advantage remains only where K is long
//     (K >= 5120: 7B down at 512 tokens 28.3 against 36.0 us; with K = 3200 the prefill kernel is 1.4x faster there).
// Returns false where these kernels should not run (above 64 tokens and no such launch); kmt and rpw are valid anyway.
static bool skinny_shape(int64_t M, int64_t RBc, int* kmt_out, int* rpw_out) {
    const int kmt_full = M <= 16 ? 1 : M <= 32 ? 2 : 4;            // the smallest tile that holds all tokens (64 at most)
    int kmt = kmt_full, rpw = 16;
    bool ok = true;
    auto one_round = [&](int t) {
        for (const int c : {1, 2, 4, 6, 8})
            if (ceil_div(RBc, c) * ceil_div(M, 16 * t) <= 256) return c;
        return 0;
    };
    if (M > 64) {
        const int c2 = one_round(2), c4 = one_round(4);
        if (c2 && c2 <= 6) { kmt = 2; rpw = c2; }
        else if (c4) { kmt = 4; rpw = c4; }
        else ok = false;
    } else {
        for (const int c : {8, 6, 4, 2, 1})
            if (ceil_div(RBc, c) <= 256) rpw = c;
        if (RBc <= 1024 && kmt_full > 1) {
            int64_t best = 0, best_wgs = 0;
            for (const int t : {1, 2, 4}) {
                if (t > kmt_full) break;
                const int c = one_round(t);                     // the most workgroups that still make one round
                if (!c) continue;
                const int64_t wgs = ceil_div(RBc, c) * ceil_div(M, 16 * t), traffic = wgs * (16 * t + 4 * c);
                // equal traffic: more workgroups, then the larger tile (its form splits K over more waves)
                if (best == 0 || traffic < best || (traffic == best && wgs >= best_wgs)) {
                    best = traffic; best_wgs = wgs; kmt = t; rpw = c;
                }
            }
        }
    }
    *kmt_out = kmt; *rpw_out = rpw;
    return ok;
}

bool gemv_supports(int64_t M, int64_t N, int64_t K, const void* xq) {
    // x_q offsets are 32-bit; one K step of the packed weights (1 KiB per 16-row block) is addressed as one raw buffer
    if (!(M >= 1 && M <= kSkinnyMaxTokens && K % 16 == 0 && reinterpret_cast<uintptr_t>(xq) % 16 == 0 &&
          M * K < ((int64_t)1 << 31) && ceil_div(N, kRowsPerBlock) < ((int64_t)1 << 21)))
        return false;
    if (M > 256 && K < 5120) return false;          // a short K: the prefill kernel's few workgroups are done quickly
    int kmt, rpw;
    return skinny_shape(M, ceil_div(N, kRowsPerBlock), &kmt, &rpw);
}

template <int kMT, int kR, int kW, int kS, int kD, int kLx>
static hipError_t launch_skinny(const int8_t* xq, const float* sx, const void* packed, const float* gamma, int gstride,
                                int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream,
                               int splits, void* workspace, LaunchPlan* plan) {
    constexpr size_t lds = (size_t)kS * (kLx + 1) * kMT * 16 * 256;
    static_assert(lds <= 160 * 1024, "activation rings must fit the LDS of a CU");
    static_assert(kS * kW <= 16, "at most 1024 threads per workgroup");
    auto* kern = linear_skinny_2bit<kMT, kR, kW, kS, kD, kLx>;
    if (lds > 65536 && !plan) {
        static RaisedFlags raised = {};
        const hipError_t e = raise_dynamic_lds(reinterpret_cast<const void*>(kern), (int)lds, raised);
        if (e != hipSuccess) return e;
    }
    const int Kq = (int)ceil_div(K, kColsPerQuad);
    const int RB = (int)ceil_div(N, kRowsPerBlock);
    const int steps = (int)ceil_div(K, 256);
    if (splits > steps) splits = steps;
    const int sps = (int)ceil_div(steps, splits);
    splits = (int)ceil_div(steps, sps);                 // no empty split
    const int spg = (int)ceil_div(sps, kS);
    const bool split = splits > 1;                      // then int32 partials go to the workspace and a second launch adds them
    dim3 grid((unsigned)ceil_div(RB, kW * kR), (unsigned)splits, (unsigned)ceil_div(M, 16 * kMT));
    if (plan) {
        plan->set("batched_decode", {kMT, kR, kW, kS, kD, kLx}, grid.x * grid.z, grid.y, kS * kW * kWave, lds, splits);
        return hipSuccess;
    }
    hipLaunchKernelGGL(kern, grid, dim3(kS * kW * kWave), lds, stream, xq, sx, static_cast<const uint4*>(packed), gamma,
                       gstride, (int)M, N, K, Kq, RB, spg, sps, split ? workspace : y, split ? OutType::I32 : yt);
    if (split)
        return launch_splitk_reduce(static_cast<const int32_t*>(workspace), splits, sx, gamma, gstride, 0, M, N, y, yt, stream);
    return hipGetLastError();
}

template <int kMT, int kR, int kW, int kS, int kD, int kLx>
static hipError_t launch_skinny_ws(const int8_t* xq, const float* sx, const void* packed, const float* gamma, int gstride,
                                   int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream,
                                  int splits, void* workspace, LaunchPlan* plan) {
    constexpr size_t lds = (size_t)kS * (kLx + 1) * kMT * 16 * 256;
    static_assert(lds <= 160 * 1024, "activation rings must fit the LDS of a CU");
    static_assert(kS * kW + 1 <= 16, "at most 1024 threads per workgroup");
    auto* kern = linear_skinny_ws_2bit<kMT, kR, kW, kS, kD, kLx>;
    if (lds > 65536 && !plan) {
        static RaisedFlags raised = {};
        const hipError_t e = raise_dynamic_lds(reinterpret_cast<const void*>(kern), (int)lds, raised);
        if (e != hipSuccess) return e;
    }
    const int Kq = (int)ceil_div(K, kColsPerQuad);
    const int RB = (int)ceil_div(N, kRowsPerBlock);
    const int steps = (int)ceil_div(K, 256);
    if (splits > steps) splits = steps;
    const int sps = (int)ceil_div(steps, splits);
    splits = (int)ceil_div(steps, sps);                 // no empty split
    const int spg = (int)ceil_div(sps, kS);
    const bool split = splits > 1;                      // then int32 partials go to the workspace and a second launch adds them
    dim3 grid((unsigned)ceil_div(RB, kW * kR), (unsigned)splits, (unsigned)ceil_div(M, 16 * kMT));
    if (plan) {
        plan->set("batched_decode_loader", {kMT, kR, kW, kS, kD, kLx}, grid.x * grid.z, grid.y, (kS * kW + 1) * kWave, lds, splits);
        return hipSuccess;
    }
    hipLaunchKernelGGL(kern, grid, dim3((kS * kW + 1) * kWave), lds, stream, xq, sx, static_cast<const uint4*>(packed), gamma,
                       gstride, (int)M, N, K, Kq, RB, spg, sps, split ? workspace : y, split ? OutType::I32 : yt);
    if (split)
        return launch_splitk_reduce(static_cast<const int32_t*>(workspace), splits, sx, gamma, gstride, 0, M, N, y, yt, stream);
    return hipGetLastError();
}
// Split-K of the batched-decode kernels: blockIdx.y takes a run of K steps, int32 partials go to the workspace and the
// prefill kernel's second launch adds them.  It exists as a forced variant only: what it was built for -- few row
// blocks and a long K, where every workgroup pulls all of x_q through its LDS -- is served better by tiling the tokens
// over workgroups (launch_linear_gemv_2bit below), which cuts the same traffic without a second launch (64 tokens,
// 22016 -> 4096: 29.1 us as one tile, 21.5 us with four splits, 15.9 us with four token tiles).
int skinny_splitk_splits(int64_t M, int64_t N, int64_t K) {
    (void)M; (void)N; (void)K;
    return 1;
}

hipError_t launch_linear_gemv_2bit(const int8_t* xq, const float* sx, const void* packed,
                                   const float* gamma, int gstride, int64_t M, int64_t N, int64_t K, void* y,
                                   OutType yt, hipStream_t stream, void* workspace, size_t workspace_bytes,
                                   int force_splits, LaunchPlan* plan) {
    const int64_t RB = ceil_div(N, kRowsPerBlock);
    // Up to four tokens, and up to eight on layers of fewer than 1024 row blocks, the M <= 16 kernel (each wave reads
    // its own x_q) is the faster one: at eight tokens 3B down 6.1 -> 5.1 us, 7B QKV 6.0 -> 5.5 us, 70B O 6.8 -> 6.1 us;
    // at sixteen the kernels below win on every layer measured.  A forced split-K stays on the kernels that have one.
    if (M <= 4 || (M <= 8 && RB < 1024 && force_splits == 0))
        return launch_linear_gemv16_2bit(xq, sx, packed, gamma, gstride, M, N, K, y, yt, stream, plan);
    // More tokens: the activations of a step outweigh the weights a wave reads with them, so they
    // are staged once per group of waves (skinny kernel), 16 * kMT >= M tokens per step.
    int splits = 1;
    if (force_splits > 0) splits = force_splits;
    else if (workspace && workspace_bytes >= splitk_workspace_bytes(M, N, skinny_splitk_splits(M, N, K)))
        splits = skinny_splitk_splits(M, N, K);
    // a split leaves each workgroup 1 / splits of K, so it can own that many more row blocks at the same running time:
    // the kernel form is chosen as for a layer with splits times the rows (fewer, larger workgroups that each stage
    // a fraction of x_q, instead of every workgroup staging all of it)
    const int64_t RBc = RB * splits;
#define SKINNY(...) \
    return launch_skinny<__VA_ARGS__>(xq, sx, packed, gamma, gstride, M, N, K, y, yt, stream, splits, workspace, plan)
#define SKINNY_WS(...) \
    return launch_skinny_ws<__VA_ARGS__>(xq, sx, packed, gamma, gstride, M, N, K, y, yt, stream, splits, workspace, plan)
    // The kernel forms per size come from sweeps over the 3B ... 70B LLaMA family shapes (31 forms, 8 ... 256 tokens).
    int kmt, rpw;
    skinny_shape(M, RBc, &kmt, &rpw);
    if (kmt == 1) {
        if (rpw == 16)     SKINNY(1, 4, 4, 2, 2, 2);
        else if (rpw == 8) SKINNY(1, 2, 4, 2, 2, 2);
        else if (rpw == 6) SKINNY(1, 3, 2, 4, 2, 2);
        else if (rpw == 4) SKINNY(1, 2, 2, 4, 2, 2);
        else if (rpw == 2) {
            // eight K groups, unless their shares pad much worse than four groups' would (20 steps: 8 x 4 against 4 x 6)
            const int64_t steps = ceil_div(ceil_div(K, 256), splits);
            const int64_t walk8 = 8 * (ceil_div(ceil_div(steps, 8), 2) * 2), walk4 = 4 * (ceil_div(ceil_div(steps, 4), 2) * 2);
            if (walk8 * 20 >= walk4 * 25) SKINNY(1, 1, 2, 4, 2, 2);
            else SKINNY(1, 1, 2, 8, 2, 2);
        }
        else               SKINNY(1, 1, 1, 8, 2, 2);
    } else if (kmt == 2) {
        // from six row blocks on, the form with a loader wave (weights 3 steps deep in flight per wave)
        if (rpw == 16)     SKINNY_WS(2, 4, 4, 1, 4, 3);
        else if (rpw == 8) SKINNY_WS(2, 2, 4, 1, 4, 3);
        else if (rpw == 6) SKINNY_WS(2, 2, 3, 2, 4, 3);
        else if (rpw == 4) SKINNY(2, 2, 2, 4, 2, 2);
        else if (rpw == 2) SKINNY(2, 1, 2, 4, 2, 2);
        else               SKINNY(2, 1, 1, 4, 2, 2);
    } else {
        if (rpw == 16)     SKINNY_WS(4, 4, 4, 1, 4, 2);
        else if (rpw == 8) SKINNY_WS(4, 2, 4, 1, 4, 2);
        else if (rpw == 6) SKINNY_WS(4, 2, 3, 1, 4, 2);
        else if (rpw == 4) SKINNY_WS(4, 2, 2, 2, 4, 2);
        else if (rpw == 2) SKINNY(4, 2, 1, 4, 2, 1);
        else               SKINNY(4, 1, 1, 4, 2, 1);
    }
#undef SKINNY
#undef SKINNY_WS
}

}  // namespace bitnet

// Prefill BitLinear kernel for gfx950: the ternary-by-int8 product on int8 MFMA (M > 64).
//
// Computes acc[m][n] = sum_k x_q[m][k] * Wt[n][k] exactly in int32 and y = acc * gamma * s_x[m] / 127
// (Sections 1-2 of arXiv 2402.17764).  At these M the cost is the contraction itself, so the kernel is
// organised around keeping v_mfma_i32_32x32x32_i8 issuing:
//
//   * a workgroup of four waves owns a 256 x 256 output tile, each wave a 128 x 128 quarter held as
//     4 x 4 accumulator fragments of 32 x 32 (256 accumulator registers per lane);
//   * activations (the A operand) are copied global -> LDS with 128-bit LDS-direct loads, two stages of
//     256 rows x 256 bytes; the 16-byte chunks of a row are XOR-swizzled with the row index so that the
//     ds_read_b128 of 16 consecutive rows hit all 64 banks;
//   * weights (the B operand) never touch LDS: the packed layout already stores, for every 16-row block,
//     the 64 codes a lane needs as one 16-byte quad, so each lane loads its own quads straight from
//     global memory one K step ahead and expands one 32-bit word (16 codes) into the four operand
//     registers of an MFMA with a shift and an AND per register -- (w << (6 - 2 i)) & 0xC0C0C0C0 leaves
//     64 * code in every byte, and the factor 64 is shifted out of the accumulator at the end;
//   * one barrier per K step of 256 columns (128 MFMAs per wave between barriers);
//   * tile order: consecutive workgroups take consecutive token tiles of the same weight tile, so the
//     eight XCDs (workgroups are dealt to them round-robin) each keep re-using the token tile that is
//     already in their L2 while the weight tile is shared through the memory-side cache.
//
// Lane l of a wave supplies, for the B operand, weight row (l & 31) of a 32-row fragment and the 16
// columns selected by (l >> 5); for the A operand token (l & 31), same columns.
#include "bitnet_device.hpp"
#include "bitnet_internal.hpp"

namespace bitnet {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kGemmBM = 256;                   // tokens per workgroup tile
constexpr int kGemmBN = 256;                   // weight rows per workgroup tile
constexpr int kGemmThreads = 256;
constexpr int kGemmStageBytes = kGemmBM * 256; // one K step of activations
constexpr int kGemmLdsBytes = 2 * kGemmStageBytes;

__device__ inline v4i gemm_decode_word(uint32_t w) {
    v4i a;
    a.x = (int)((w << 6) & 0xC0C0C0C0u);
    a.y = (int)((w << 4) & 0xC0C0C0C0u);
    a.z = (int)((w << 2) & 0xC0C0C0C0u);
    a.w = (int)(w & 0xC0C0C0C0u);
    return a;
}

__device__ inline uint32_t gemm_quad_word(const uint4& q, int j) { return j == 0 ? q.x : j == 1 ? q.y : j == 2 ? q.z : q.w; }

__global__ __launch_bounds__(kGemmThreads, 1) void linear_gemm_2bit(
        const int8_t* __restrict__ xq, const float* __restrict__ sx, const uint4* __restrict__ packed,
        const float* __restrict__ gamma, int M, int64_t N, int64_t K, int Kq, int RB, int tiles_m,
        void* __restrict__ y, OutType yt) {
    extern __shared__ uint4 smem[];
    char* lds = reinterpret_cast<char*>(smem);

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int bm = blockIdx.x % tiles_m;            // token tile varies fastest (see header)
    const int bn = blockIdx.x / tiles_m;
    const int steps = (Kq + 3) >> 2;
    const int tail_quads = 16 * (Kq - 4 * (steps - 1));
    const int64_t wstride = (int64_t)RB * 64;

    // ---- A operand, global -> LDS: this wave copies rows 64*wave .. +63 of the tile, 4 rows per load
    // lane i of a load writes LDS slot i: row (i >> 4) of the group, chunk slot (i & 15); the chunk that
    // belongs in slot c' of row m is c' ^ (m & 15)
    const int cp_row = lane >> 4, cp_slot = lane & 15;
    // ---- A operand, LDS -> registers
    const int am = lane & 31, kg = lane >> 5;
    // ---- B operand: fragment fn covers row blocks 2*fn, 2*fn+1 of this wave's 8
    const int brow = lane & 15, bsel = (lane >> 4) & 1;
    int rbc[4];
#pragma unroll
    for (int fn = 0; fn < 4; ++fn) rbc[fn] = min(bn * 16 + wn * 8 + fn * 2 + bsel, RB - 1);

    v16i acc[4][4];
#pragma unroll
    for (int fm = 0; fm < 4; ++fm)
#pragma unroll
        for (int fn = 0; fn < 4; ++fn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[fm][fn][v] = 0;

    auto copy_x = [&](int step, int stage) {
        char* dst_stage = lds + stage * kGemmStageBytes;
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const int row = wave * 64 + t * 4 + cp_row;                      // row inside the tile
            const int m = min(bm * kGemmBM + row, M - 1);                   // rows past M: clamped, never stored
            const int chunk = cp_slot ^ (row & 15);
            const int64_t col = min((int64_t)step * 256 + chunk * 16, K - 16);   // past-the-end columns meet zero codes
            const int8_t* src = xq + (int64_t)m * K + col;
            char* dst = dst_stage + (wave * 64 + t * 4) * 256;              // wave-uniform; lane i lands at +16 i
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
        }
    };
    auto load_w = [&](uint4 (&wq)[4][2], int step) {
        const int cq = step == steps - 1 ? tail_quads : 64;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int g = kg + 2 * h;
            const int ln = min(g * 16 + brow, cq - 1);
#pragma unroll
            for (int fn = 0; fn < 4; ++fn) wq[fn][h] = packed[(int64_t)step * wstride + (int64_t)rbc[fn] * cq + ln];
        }
    };
    auto compute = [&](const uint4 (&wq)[4][2], int step, int stage) {
        const int cq = step == steps - 1 ? tail_quads : 64;
        const char* src_stage = lds + stage * kGemmStageBytes;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t keep = ((kg + 2 * h) * 16 + brow) < cq ? 0xFFFFFFFFu : 0u;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int chunk = 8 * h + 4 * kg + j;
                v4i a[4], b[4];
#pragma unroll
                for (int fm = 0; fm < 4; ++fm) {
                    const int row = wm * 128 + fm * 32 + am;
                    a[fm] = *reinterpret_cast<const v4i*>(src_stage + row * 256 + ((chunk ^ (row & 15)) << 4));
                }
#pragma unroll
                for (int fn = 0; fn < 4; ++fn) b[fn] = gemm_decode_word(gemm_quad_word(wq[fn][h], j) & keep);
#pragma unroll
                for (int fm = 0; fm < 4; ++fm)
#pragma unroll
                    for (int fn = 0; fn < 4; ++fn)
                        acc[fm][fn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[fm], b[fn], acc[fm][fn], 0, 0, 0);
            }
        }
    };

    uint4 w0[4][2], w1[4][2];
    copy_x(0, 0);
    load_w(w0, 0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    int s = 0;
    for (; s + 2 <= steps; s += 2) {
        // even step: operands of step s + 1 go to stage 1 / w1 while step s is consumed from stage 0 / w0
        copy_x(s + 1, 1);
        load_w(w1, s + 1);
        compute(w0, s, 0);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (s + 2 < steps) {
            copy_x(s + 2, 0);
            load_w(w0, s + 2);
        }
        compute(w1, s + 1, 1);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    }
    if (s < steps) compute(w0, s, 0);

    // ---- epilogue: lane holds, per fragment, 16 tokens (8 (v >> 2) + 4 (l >> 5) + (v & 3)) of one weight row
    const float gm = gamma[0];
#pragma unroll
    for (int fm = 0; fm < 4; ++fm) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = bm * kGemmBM + wm * 128 + fm * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
            if (m >= M) continue;
            const float scale = yt == OutType::I32 ? 0.0f : (gm * sx[m]) / kQb;
#pragma unroll
            for (int fn = 0; fn < 4; ++fn) {
                const int64_t n = (int64_t)bn * kGemmBN + wn * 128 + fn * 32 + am;
                if (n >= N) continue;
                const int a = acc[fm][fn][v] >> 6;                           // drop the decode factor 64 (exact)
                const int64_t idx = (int64_t)m * N + n;
                if (yt == OutType::I32) static_cast<int32_t*>(y)[idx] = a;
                else if (yt == OutType::F32) static_cast<float*>(y)[idx] = (float)a * scale;
                else static_cast<uint16_t*>(y)[idx] = f32_to_bf16((float)a * scale);
            }
        }
    }
}

bool gemm_supports(int64_t M, int64_t N, int64_t K, const void* xq) {
    (void)N;
    return M >= 1 && K % 16 == 0 && reinterpret_cast<uintptr_t>(xq) % 16 == 0;
}

hipError_t launch_linear_gemm_2bit(const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                                   int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_gemm_2bit),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLdsBytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int Kq = (int)ceil_div(K, kColsPerQuad);
    const int RB = (int)ceil_div(N, kRowsPerBlock);
    const int tiles_m = (int)ceil_div(M, kGemmBM);
    const int64_t tiles_n = ceil_div(N, kGemmBN);
    dim3 grid((unsigned)(tiles_m * tiles_n));
    hipLaunchKernelGGL(linear_gemm_2bit, grid, dim3(kGemmThreads), kGemmLdsBytes, stream, xq, sx,
                       static_cast<const uint4*>(packed), gamma, (int)M, N, K, Kq, RB, tiles_m, y, yt);
    return hipGetLastError();
}

}  // namespace bitnet

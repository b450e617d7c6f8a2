// Weight-streaming BitLinear kernel for decode and batched decode (M <= 64) on gfx950.
//
// Computes acc[m][n] = sum_k x_q[m][k] * Wt[n][k] exactly in int32 and y = acc * gamma * s_x[m] / 127
// (Sections 1-2 of arXiv 2402.17764).  At these M the cost is moving the packed weights out of HBM,
// so the kernel is organised around that stream:
//
//   * one 128-bit load per lane fetches one quad (64 codes of one row); a wavefront's 64 lanes fetch
//     four whole 16-row x 64-column tiles = 1 KiB of contiguous memory per load instruction;
//   * a 32-bit word of 2-bit two's-complement codes becomes four int8 MFMA operand registers with one
//     shift and one AND each: (w << (6 - 2 i)) & 0xC0C0C0C0 leaves 64 * code in every byte, so no
//     multiply and no sign fix-up is spent on decoding; the factor 64 is shifted out of the int32
//     accumulator at the end (exact, |64 * 127 * K| < 2^31);
//   * the contraction itself runs on v_mfma_i32_16x16x64_i8 with the 16 weight rows as the A operand
//     and up to 16 tokens as the B operand; the matrix pipe is otherwise idle in a bandwidth-bound
//     kernel, and M = 1 ... 16 cost the same;
//   * the waves of a workgroup split K between them and fold their partial accumulators through LDS
//     in a fixed order (integer adds: exact and deterministic).
//
// Lane l of a wave supplies row (l & 15) and the columns of quad (l >> 4) of the current step; the
// activation operand of lane l is token (l & 15), same columns, so every product pairs the same k.
#include "bitnet_device.hpp"
#include "bitnet_internal.hpp"

namespace bitnet {

typedef int v4i __attribute__((ext_vector_type(4)));

__device__ inline v4i decode_word(uint32_t w) {
    v4i a;
    a.x = (int)((w << 6) & 0xC0C0C0C0u);
    a.y = (int)((w << 4) & 0xC0C0C0C0u);
    a.z = (int)((w << 2) & 0xC0C0C0C0u);
    a.w = (int)(w & 0xC0C0C0C0u);
    return a;
}

__device__ inline v4i as_v4i(const uint4& u) {
    v4i a;
    a.x = (int)u.x; a.y = (int)u.y; a.z = (int)u.z; a.w = (int)u.w;
    return a;
}

// kR  row blocks (16 rows each) per workgroup, all handled by every wave
// kMT token tiles of 16
// kW  waves per workgroup; wave w takes K steps w, w + kW, ...
template <int kR, int kMT, int kW>
__global__ __launch_bounds__(kW * kWave) void linear_gemv_2bit(const int8_t* __restrict__ xq, const float* __restrict__ sx,
                                                                const uint4* __restrict__ packed,
                                                                const float* __restrict__ gamma, int M, int64_t N, int64_t K,
                                                                int Kq, int RB, void* __restrict__ y, OutType yt) {
    __shared__ v4i fold[kW][kR * kMT][kWave];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int r = lane & 15;
    const int g = lane >> 4;
    const int rb0 = blockIdx.x * kR;
    const int steps = (Kq + 3) >> 2;

    v4i acc[kR][kMT];
#pragma unroll
    for (int a = 0; a < kR; ++a)
#pragma unroll
        for (int t = 0; t < kMT; ++t) acc[a][t] = (v4i){0, 0, 0, 0};

    const uint4 zero4 = make_uint4(0, 0, 0, 0);

    for (int step = wave; step < steps; step += kW) {
        const int kq = 4 * step + g;
        const bool kq_ok = kq < Kq;

        uint4 wq[kR];
#pragma unroll
        for (int a = 0; a < kR; ++a) {
            wq[a] = zero4;
            if (kq_ok && rb0 + a < RB) wq[a] = packed[((int64_t)(rb0 + a) * Kq + kq) * 16 + r];
        }
        uint4 xv[kMT][4];
#pragma unroll
        for (int t = 0; t < kMT; ++t) {
            const int m = 16 * t + r;
            const int64_t kbase = (int64_t)kq * 64;
            const uint4* xp = reinterpret_cast<const uint4*>(xq + (int64_t)m * K + kbase);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                xv[t][j] = zero4;
                if (m < M && kbase + 16 * j + 16 <= K) xv[t][j] = xp[j];
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int a = 0; a < kR; ++a) {
                const uint32_t word = j == 0 ? wq[a].x : j == 1 ? wq[a].y : j == 2 ? wq[a].z : wq[a].w;
                const v4i A = decode_word(word);
#pragma unroll
                for (int t = 0; t < kMT; ++t)
                    acc[a][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A, as_v4i(xv[t][j]), acc[a][t], 0, 0, 0);
            }
        }
    }

    // fold the K slices of the kW waves
#pragma unroll
    for (int a = 0; a < kR; ++a)
#pragma unroll
        for (int t = 0; t < kMT; ++t) fold[wave][a * kMT + t][lane] = acc[a][t];
    __syncthreads();

    const float gm = gamma[0];
    for (int tile = wave; tile < kR * kMT; tile += kW) {
        v4i s = fold[0][tile][lane];
#pragma unroll
        for (int w = 1; w < kW; ++w) {
            const v4i o = fold[w][tile][lane];
            s.x += o.x; s.y += o.y; s.z += o.z; s.w += o.w;
        }
        const int a = tile / kMT, t = tile % kMT;
        const int m = 16 * t + r;                               // MFMA output: column = lane & 15 = token
        const int64_t n0 = (int64_t)(rb0 + a) * 16 + 4 * g;     // rows 4 g .. 4 g + 3 of the row block
        if (m >= M || n0 >= N) continue;
        const int v[4] = {s.x >> 6, s.y >> 6, s.z >> 6, s.w >> 6};   // drop the decode factor 64 (exact)
        const int64_t base = (int64_t)m * N + n0;
        if (yt == OutType::I32) {
            int32_t* yo = static_cast<int32_t*>(y);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (n0 + e < N) yo[base + e] = v[e];
        } else {
            const float scale = (gm * sx[m]) / kQb;
            if (yt == OutType::F32) {
                float* yo = static_cast<float*>(y);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (n0 + e < N) yo[base + e] = (float)v[e] * scale;
            } else {
                uint16_t* yo = static_cast<uint16_t*>(y);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (n0 + e < N) yo[base + e] = f32_to_bf16((float)v[e] * scale);
            }
        }
    }
}

bool gemv_supports(int64_t M, int64_t N, int64_t K, const void* xq) {
    (void)N;
    return M >= 1 && M <= 64 && K % 16 == 0 && reinterpret_cast<uintptr_t>(xq) % 16 == 0;
}

template <int kR, int kMT, int kW>
static void launch_one(const int8_t* xq, const float* sx, const void* packed, const float* gamma, int64_t M,
                       int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream) {
    const int Kq = (int)ceil_div(K, kColsPerQuad);
    const int RB = (int)ceil_div(N, kRowsPerBlock);
    dim3 grid((unsigned)ceil_div(RB, kR));
    hipLaunchKernelGGL((linear_gemv_2bit<kR, kMT, kW>), grid, dim3(kW * kWave), 0, stream, xq, sx,
                       static_cast<const uint4*>(packed), gamma, (int)M, N, K, Kq, RB, y, yt);
}

hipError_t launch_linear_gemv_2bit(const int8_t* xq, const float* sx, const void* packed,
                                   const float* gamma, int64_t M, int64_t N, int64_t K, void* y,
                                   OutType yt, hipStream_t stream) {
    const int64_t RB = ceil_div(N, kRowsPerBlock);
    if (M <= 16) {
        // few row blocks: keep one per workgroup so the grid still covers the chip
        if (RB < 2048)      launch_one<1, 1, 8>(xq, sx, packed, gamma, M, N, K, y, yt, stream);
        else if (RB < 4096) launch_one<2, 1, 8>(xq, sx, packed, gamma, M, N, K, y, yt, stream);
        else                launch_one<4, 1, 8>(xq, sx, packed, gamma, M, N, K, y, yt, stream);
    } else if (M <= 32) {
        launch_one<4, 2, 4>(xq, sx, packed, gamma, M, N, K, y, yt, stream);
    } else {
        launch_one<2, 4, 4>(xq, sx, packed, gamma, M, N, K, y, yt, stream);
    }
    return hipGetLastError();
}

}  // namespace bitnet

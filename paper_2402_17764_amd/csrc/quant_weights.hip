// Absmean ternary weight quantization (Eq. (1)-(3) of arXiv 2402.17764) for gfx950.
//
//   pass 1  abs_sum_partials : grid-stride |W| sum, double-double per thread, fixed-shape tree
//                              inside the block, one (hi, lo) pair per block into the workspace
//   pass 2  finish_gamma     : one block folds the partials in a fixed order, gamma = fp32(S / (N K))
//   pass 3  ternarize_pack   : re-reads W, takes the decision of Eq. (1)-(2) in fp32 and writes the
//                              packed buffer through LDS so that both the 4 B/weight read and the
//                              0.25 B/weight write are contiguous
//
// The whole path is HBM-bound at 8.25 B per weight (two reads of W, one packed write).
#include "bitnet_device.hpp"
#include "bitnet_internal.hpp"

namespace bitnet {

// ---------------------------------------------------------------------------------------------------
// pass 1
// ---------------------------------------------------------------------------------------------------
constexpr int kSumThreads = 256;

template <typename T> struct Vec4;
template <> struct Vec4<float> {
    using type = float4;
    __device__ static void widen(const float4& v, float (&o)[4]) { o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w; }
};
template <> struct Vec4<uint16_t> {
    using type = ushort4;
    __device__ static void widen(const ushort4& v, float (&o)[4]) {
        o[0] = bf16_to_f32(v.x); o[1] = bf16_to_f32(v.y); o[2] = bf16_to_f32(v.z); o[3] = bf16_to_f32(v.w);
    }
};
__device__ inline float widen1(float v) { return v; }
__device__ inline float widen1(uint16_t v) { return bf16_to_f32(v); }

template <typename T>
__global__ __launch_bounds__(kSumThreads) void abs_sum_partials(const T* __restrict__ W, int64_t count,
                                                                int vec_ok, double* __restrict__ partials) {
    using V = typename Vec4<T>::type;
    dd acc{0.0, 0.0};
    const int64_t tid = (int64_t)blockIdx.x * kSumThreads + threadIdx.x;
    const int64_t nthreads = (int64_t)gridDim.x * kSumThreads;
    int64_t done = 0;
    if (vec_ok) {
        const int64_t nvec = count / 4;
        const V* Wv = reinterpret_cast<const V*>(W);
        // four loads in flight per thread and four independent accumulators: the sums are exact, so the
        // split changes nothing but the bytes in flight and the length of the dependent chains
        dd part[4] = {{0.0, 0.0}, {0.0, 0.0}, {0.0, 0.0}, {0.0, 0.0}};
        int64_t i = tid;
        for (; i + 3 * nthreads < nvec; i += 4 * nthreads) {
            V v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = Wv[i + u * nthreads];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                float f[4];
                Vec4<T>::widen(v[u], f);
#pragma unroll
                for (int e = 0; e < 4; ++e) dd_add_double(part[e], (double)fabsf(f[e]));
            }
        }
        for (; i < nvec; i += nthreads) {
            float f[4];
            Vec4<T>::widen(Wv[i], f);
#pragma unroll
            for (int e = 0; e < 4; ++e) dd_add_double(part[e], (double)fabsf(f[e]));
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) dd_add_dd(acc, part[e]);
        done = nvec * 4;
    }
    for (int64_t i = done + tid; i < count; i += nthreads) dd_add_double(acc, (double)fabsf(widen1(W[i])));

    // fixed-shape tree over the block: the same pairs are always added in the same order
    __shared__ double sh_hi[kSumThreads];
    __shared__ double sh_lo[kSumThreads];
    sh_hi[threadIdx.x] = acc.hi;
    sh_lo[threadIdx.x] = acc.lo;
    __syncthreads();
    for (int s = kSumThreads / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) {
            dd a{sh_hi[threadIdx.x], sh_lo[threadIdx.x]};
            dd b{sh_hi[threadIdx.x + s], sh_lo[threadIdx.x + s]};
            dd_add_dd(a, b);
            sh_hi[threadIdx.x] = a.hi;
            sh_lo[threadIdx.x] = a.lo;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        partials[2 * blockIdx.x] = sh_hi[0];
        partials[2 * blockIdx.x + 1] = sh_lo[0];
    }
}

// ---------------------------------------------------------------------------------------------------
// pass 2
// ---------------------------------------------------------------------------------------------------
// gamma[0 .. nout-1] all receive the value (nout > 1: one copy per 16-row block of a segment)
__global__ __launch_bounds__(kSumThreads) void finish_gamma(const double* __restrict__ partials, int nparts,
                                                            int64_t count, float* __restrict__ gamma, int64_t nout) {
    dd acc{0.0, 0.0};
    for (int i = threadIdx.x; i < nparts; i += kSumThreads) {
        dd p{partials[2 * i], partials[2 * i + 1]};
        dd_add_dd(acc, p);
    }
    __shared__ double sh_hi[kSumThreads];
    __shared__ double sh_lo[kSumThreads];
    sh_hi[threadIdx.x] = acc.hi;
    sh_lo[threadIdx.x] = acc.lo;
    __syncthreads();
    for (int s = kSumThreads / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) {
            dd a{sh_hi[threadIdx.x], sh_lo[threadIdx.x]};
            dd b{sh_hi[threadIdx.x + s], sh_lo[threadIdx.x + s]};
            dd_add_dd(a, b);
            sh_hi[threadIdx.x] = a.hi;
            sh_lo[threadIdx.x] = a.lo;
        }
        __syncthreads();
    }
    const double S = sh_hi[0] + sh_lo[0];
    const float g = (float)(S / (double)count);     // Eq. (3); fp64 IEEE division, one rounding to fp32
    for (int64_t i = threadIdx.x; i < nout; i += kSumThreads) gamma[i] = g;
}

// ---------------------------------------------------------------------------------------------------
// pass 3, 2-bit format
// ---------------------------------------------------------------------------------------------------
// One workgroup of 16 waves owns one 16-row block; wave r streams row 16*rb + r.  Per step the wave
// reads 1024 consecutive columns (lane l, sub-step t: columns 256 t + 4 l .. +3, a 16-byte load for
// fp32), so reads are 1 KiB runs.  The four codes of a lane land in one word at bits 8 b + 2 i with
// i = l & 3; OR-ing the four lanes of a quad completes the word.  Words are staged in LDS in output
// order ([16 quads of K][16 rows][4 words] = 4 KiB) and written out as 256-byte runs, one per quad
// column, which land inside the 1 KiB (step, row block) chunks of the packed layout.
constexpr int kPackWaves = 16;
constexpr int kPackThreads = kPackWaves * kWave;          // 1024
constexpr int kPackColsPerStep = 1024;                    // 16 quads along K per workgroup step

// W, N: the rows being packed (a whole matrix, or one segment of it); they become row blocks rb_off ... of a
// packed matrix of RB row blocks in all.
template <typename T, bool kVec>
__global__ __launch_bounds__(kPackThreads) void ternarize_pack_2bit(const T* __restrict__ W, int64_t N, int64_t K,
                                                                    int64_t Kq /* quads per row */, int64_t RB,
                                                                    int64_t rb_off, const float* __restrict__ gamma,
                                                                    uint32_t* __restrict__ packed) {
    using V = typename Vec4<T>::type;
    __shared__ uint32_t stage[16 * 16 * 4];
    const int lane = threadIdx.x & (kWave - 1);
    const int r = threadIdx.x >> 6;                        // wave index = row inside the block
    const int64_t rb = blockIdx.x;
    const int64_t n = rb * kRowsPerBlock + r;
    const float d = gamma[0] + kEps;                       // gamma + eps, one fp32 add (Eq. (1))
    const float thr = ternary_threshold(d);                // |w| >= thr  <=>  RoundClip(w / d) = +-1
    const T* row = W + n * K;
    const int i = lane & 3;

    for (int64_t k0 = (int64_t)blockIdx.y * kPackColsPerStep; k0 < Kq * kColsPerQuad;
         k0 += (int64_t)gridDim.y * kPackColsPerStep) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int64_t k = k0 + 256 * t + 4 * lane;
            float f[4] = {0.f, 0.f, 0.f, 0.f};             // padding rows / columns quantize to code 0
            if (n < N) {
                if (kVec) {
                    if (k < K) Vec4<T>::widen(*reinterpret_cast<const V*>(row + k), f);
                } else {
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        if (k + b < K) f[b] = widen1(row[k + b]);
                }
            }
            uint32_t w = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) w |= ternary_code2_threshold(f[b], thr) << (8 * b + 2 * i);
            w = quad_or(w);
            if (i == 0) {
                const int quad = 4 * t + (lane >> 4);      // which of the 16 quads of this step
                const int j = (lane >> 2) & 3;             // word inside the quad
                stage[(quad * 16 + r) * 4 + j] = w;
            }
        }
        __syncthreads();
        // 16 quads x 16 rows x 4 words = 1024 words: one per thread, contiguous in the output
        {
            const int quad = threadIdx.x >> 6;
            const int64_t kq = k0 / kColsPerQuad + quad;
            if (kq < Kq) packed[quad_index_2bit(kq, rb + rb_off, 0, Kq, RB) * 4 + (threadIdx.x & 63)] = stage[threadIdx.x];
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------------
int quant_weights_num_partials() { return 2048; }

// Eq. (3): passes 1 and 2, shared by every packing format
hipError_t launch_absmean_gamma(const void* W, bool bf16, int64_t N, int64_t K, float* gamma, void* workspace,
                                hipStream_t stream, int64_t nout) {
    const int64_t count = N * K;
    double* partials = static_cast<double*>(workspace);
    int64_t want = ceil_div(count, (int64_t)kSumThreads * 16);
    int blocks = (int)(want < 1 ? 1 : (want > quant_weights_num_partials() ? quant_weights_num_partials() : want));
    const size_t esz = bf16 ? 2 : 4;
    const int vec_ok = (reinterpret_cast<uintptr_t>(W) % (4 * esz)) == 0;
    if (bf16)
        hipLaunchKernelGGL(abs_sum_partials<uint16_t>, dim3(blocks), dim3(kSumThreads), 0, stream,
                           static_cast<const uint16_t*>(W), count, vec_ok, partials);
    else
        hipLaunchKernelGGL(abs_sum_partials<float>, dim3(blocks), dim3(kSumThreads), 0, stream,
                           static_cast<const float*>(W), count, vec_ok, partials);
    hipLaunchKernelGGL(finish_gamma, dim3(1), dim3(kSumThreads), 0, stream, partials, blocks, count, gamma, nout);
    return hipGetLastError();
}

hipError_t launch_quantize_weights_2bit(const void* W, bool bf16, int64_t N, int64_t K, void* packed,
                                        float* gamma, void* workspace, hipStream_t stream, int64_t rb_off,
                                        int64_t rb_total, int64_t nout) {
    hipError_t err = launch_absmean_gamma(W, bf16, N, K, gamma, workspace, stream, nout);
    if (err != hipSuccess) return err;
    const size_t esz = bf16 ? 2 : 4;
    const int vec_ok = (reinterpret_cast<uintptr_t>(W) % (4 * esz)) == 0;

    const int64_t Kq = ceil_div(K, kColsPerQuad);
    const int64_t RB = ceil_div(N, kRowsPerBlock);                       // row blocks packed by this call
    const int64_t RBT = rb_total > 0 ? rb_total : RB;                      // ... of the whole packed matrix
    const int64_t steps = ceil_div(Kq * kColsPerQuad, kPackColsPerStep);
    // enough workgroups to fill the chip even for few row blocks: split K across blockIdx.y
    int64_t ysplit = 1;
    while (RB * ysplit < 1024 && ysplit * 2 <= steps) ysplit *= 2;
    const bool vec = vec_ok && (K % 4 == 0);
    dim3 grid((unsigned)RB, (unsigned)ysplit);
    uint32_t* out = static_cast<uint32_t*>(packed);
    if (bf16) {
        const uint16_t* w = static_cast<const uint16_t*>(W);
        if (vec) hipLaunchKernelGGL((ternarize_pack_2bit<uint16_t, true>), grid, dim3(kPackThreads), 0, stream, w, N, K, Kq, RBT, rb_off, gamma, out);
        else     hipLaunchKernelGGL((ternarize_pack_2bit<uint16_t, false>), grid, dim3(kPackThreads), 0, stream, w, N, K, Kq, RBT, rb_off, gamma, out);
    } else {
        const float* w = static_cast<const float*>(W);
        if (vec) hipLaunchKernelGGL((ternarize_pack_2bit<float, true>), grid, dim3(kPackThreads), 0, stream, w, N, K, Kq, RBT, rb_off, gamma, out);
        else     hipLaunchKernelGGL((ternarize_pack_2bit<float, false>), grid, dim3(kPackThreads), 0, stream, w, N, K, Kq, RBT, rb_off, gamma, out);
    }
    return hipGetLastError();
}

}  // namespace bitnet

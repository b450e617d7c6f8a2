// Reference-grade BitLinear product for gfx950: one thread per output element, a plain loop over K
// that adds, subtracts or skips each activation according to its ternary weight (Sections 1-2 of
// arXiv 2402.17764), then the rescale y = acc * gamma * s_x / 127.  It accepts every shape and
// alignment; the fast kernels are checked against the same oracle and take over where they apply.
// Also here: the unpack helper that turns the packed buffer back into int8 codes.
#include "bitnet_device.hpp"
#include "bitnet_internal.hpp"

namespace bitnet {

__device__ inline uint32_t load_word_2bit(const uint32_t* packed, int64_t Kq, int64_t RB, int64_t n, int64_t k) {
    const int64_t rb = n >> 4, kq = k >> 6, j = (k >> 4) & 3;
    return packed[quad_index_2bit(kq, rb, (int)(n & 15), Kq, RB) * 4 + j];
}

__device__ inline void store_out(void* y, OutType yt, int64_t idx, int32_t acc, float scale) {
    if (yt == OutType::I32) {
        static_cast<int32_t*>(y)[idx] = acc;
    } else {
        const float v = (float)acc * scale;
        if (yt == OutType::F32) static_cast<float*>(y)[idx] = v;
        else static_cast<uint16_t*>(y)[idx] = f32_to_bf16(v);
    }
}

__global__ __launch_bounds__(256) void linear_reference_2bit(const int8_t* __restrict__ xq, const float* __restrict__ sx,
                                                             const uint32_t* __restrict__ packed,
                                                             const float* __restrict__ gamma, int gstride, int64_t M,
                                                             int64_t N, int64_t K, int64_t Kq, int64_t RB, void* __restrict__ y,
                                                             OutType yt) {
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t m = blockIdx.y;
    if (n >= N) return;
    const int8_t* xr = xq + m * K;
    int32_t acc = 0;
    for (int64_t k0 = 0; k0 < K; k0 += 16) {
        const uint32_t w = load_word_2bit(packed, Kq, RB, n, k0);
        const int lim = (int)((K - k0) < 16 ? (K - k0) : 16);
        for (int c = 0; c < lim; ++c) {
            const int code = code_value((w >> code_shift(c)) & 3u);
            if (code > 0) acc += xr[k0 + c];
            else if (code < 0) acc -= xr[k0 + c];
        }
    }
    const float scale = (gamma[gstride * (n / kRowsPerBlock)] * sx[m]) / kQb;
    store_out(y, yt, m * N + n, acc, scale);
}

__global__ __launch_bounds__(256) void unpack_2bit(const uint32_t* __restrict__ packed, int64_t N, int64_t K, int64_t Kq,
                                                   int64_t RB, int8_t* __restrict__ codes) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= N * K) return;
    const int64_t n = idx / K, k = idx % K;
    const uint32_t w = load_word_2bit(packed, Kq, RB, n, k);
    codes[idx] = (int8_t)code_value((w >> code_shift((int)(k & 15))) & 3u);
}

hipError_t launch_linear_reference_2bit(const int8_t* xq, const float* sx, const void* packed,
                                        const float* gamma, int gstride, int64_t M, int64_t N, int64_t K, void* y,
                                        OutType yt, hipStream_t stream) {
    const int64_t Kq = ceil_div(K, kColsPerQuad);
    // gridDim.y is limited to 65535: walk M in slabs
    for (int64_t m0 = 0; m0 < M; m0 += 32768) {
        const int64_t mc = (M - m0) < 32768 ? (M - m0) : 32768;
        dim3 grid((unsigned)ceil_div(N, 256), (unsigned)mc);
        const size_t ysz = yt == OutType::BF16 ? 2 : 4;
        hipLaunchKernelGGL(linear_reference_2bit, grid, dim3(256), 0, stream, xq + m0 * K, sx + m0,
                           static_cast<const uint32_t*>(packed), gamma, gstride, mc, N, K, Kq, ceil_div(N, kRowsPerBlock),
                           static_cast<char*>(y) + m0 * N * ysz, yt);
    }
    return hipGetLastError();
}

hipError_t launch_unpack_2bit(const void* packed, int64_t N, int64_t K, int8_t* codes, hipStream_t stream) {
    const int64_t Kq = ceil_div(K, kColsPerQuad);
    hipLaunchKernelGGL(unpack_2bit, dim3((unsigned)ceil_div(N * K, 256)), dim3(256), 0, stream,
                       static_cast<const uint32_t*>(packed), N, K, Kq, ceil_div(N, kRowsPerBlock), codes);
    return hipGetLastError();
}

}  // namespace bitnet

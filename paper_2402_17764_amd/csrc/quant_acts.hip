// Per-token absmax quantization of activations to int8 (Section 2 of arXiv 2402.17764: activations
// are scaled per token into [-Q_b, Q_b], Q_b = 127, with no zero point).
//
// One workgroup per token.  The token is read once into registers (16-byte loads), the absmax is
// reduced with DPP / shuffle steps inside each wave and through LDS across waves, then the same
// registers are scaled, rounded (ties to even) and written as packed int8.  Tokens too long for the
// register budget, or rows that are not 16-byte aligned, take a two-sweep path that re-reads x.
#include "bitnet_device.hpp"
#include "bitnet_internal.hpp"

namespace bitnet {

constexpr int kActThreads = 256;
constexpr int kActWaves = kActThreads / kWave;
constexpr int kActMaxVec = 16;         // register-resident path: up to 16 x 16 bytes per thread

__device__ inline int quantize_one(float v, float inv) {
    float r = rintf(v * inv);                              // one fp32 multiply, ties to even
    r = fminf(kQb, fmaxf(-kQb, r));
    return (int)r;
}

__device__ inline float block_max_nonneg(float v, float* sh) {
    v = wave_max_nonneg(v);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) sh[wave] = v;
    __syncthreads();
    float m = sh[0];
#pragma unroll
    for (int w = 1; w < kActWaves; ++w) m = fmaxf(m, sh[w]);
    return m;
}

// ---- register-resident vector path ----------------------------------------------------------------
// fp32: a 16-byte load is 4 elements -> 4 int8 = one 32-bit store.
// bf16: a 16-byte load is 8 elements -> 8 int8 = one 64-bit store.
template <bool kBf16>
__global__ __launch_bounds__(kActThreads) void quantize_acts_vec(const void* __restrict__ xv, int64_t K,
                                                                 int8_t* __restrict__ xq, float* __restrict__ sx) {
    constexpr int kElems = kBf16 ? 8 : 4;
    __shared__ float sh[kActWaves];
    const int64_t m = blockIdx.x;
    const int nvec = (int)(K / kElems);
    const uint4* row = reinterpret_cast<const uint4*>(static_cast<const char*>(xv) + m * K * (kBf16 ? 2 : 4));
    uint4 raw[kActMaxVec];
    float amax = 0.0f;
#pragma unroll
    for (int v = 0; v < kActMaxVec; ++v) {
        const int idx = v * kActThreads + threadIdx.x;
        raw[v] = make_uint4(0, 0, 0, 0);
        if (idx < nvec) raw[v] = row[idx];
        const uint32_t u[4] = {raw[v].x, raw[v].y, raw[v].z, raw[v].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (kBf16) {
                amax = fmaxf(amax, fabsf(__uint_as_float(u[e] << 16)));
                amax = fmaxf(amax, fabsf(__uint_as_float(u[e] & 0xFFFF0000u)));
            } else {
                amax = fmaxf(amax, fabsf(__uint_as_float(u[e])));
            }
        }
    }
    amax = block_max_nonneg(amax, sh);
    const float s = fmaxf(amax, kEps);
    const float inv = kQb / s;                             // one IEEE division per token
    if (threadIdx.x == 0) sx[m] = s;

    int8_t* out = xq + m * K;
#pragma unroll
    for (int v = 0; v < kActMaxVec; ++v) {
        const int idx = v * kActThreads + threadIdx.x;
        if (idx >= nvec) continue;
        const uint32_t u[4] = {raw[v].x, raw[v].y, raw[v].z, raw[v].w};
        if (kBf16) {
            uint32_t lo = 0, hi = 0;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                lo |= ((uint32_t)quantize_one(__uint_as_float(u[e] << 16), inv) & 0xFFu) << (16 * e);
                lo |= ((uint32_t)quantize_one(__uint_as_float(u[e] & 0xFFFF0000u), inv) & 0xFFu) << (16 * e + 8);
                hi |= ((uint32_t)quantize_one(__uint_as_float(u[e + 2] << 16), inv) & 0xFFu) << (16 * e);
                hi |= ((uint32_t)quantize_one(__uint_as_float(u[e + 2] & 0xFFFF0000u), inv) & 0xFFu) << (16 * e + 8);
            }
            reinterpret_cast<uint2*>(out)[idx] = make_uint2(lo, hi);
        } else {
            uint32_t p = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) p |= ((uint32_t)quantize_one(__uint_as_float(u[e]), inv) & 0xFFu) << (8 * e);
            reinterpret_cast<uint32_t*>(out)[idx] = p;
        }
    }
}

// ---- any-shape path: two sweeps, element loads -----------------------------------------------------
template <bool kBf16>
__global__ __launch_bounds__(kActThreads) void quantize_acts_any(const void* __restrict__ xv, int64_t K,
                                                                 int8_t* __restrict__ xq, float* __restrict__ sx) {
    __shared__ float sh[kActWaves];
    const int64_t m = blockIdx.x;
    const float* rf = static_cast<const float*>(xv) + m * K;
    const uint16_t* rh = static_cast<const uint16_t*>(xv) + m * K;
    float amax = 0.0f;
    for (int64_t k = threadIdx.x; k < K; k += kActThreads)
        amax = fmaxf(amax, fabsf(kBf16 ? bf16_to_f32(rh[k]) : rf[k]));
    amax = block_max_nonneg(amax, sh);
    const float s = fmaxf(amax, kEps);
    const float inv = kQb / s;
    if (threadIdx.x == 0) sx[m] = s;
    int8_t* out = xq + m * K;
    for (int64_t k = threadIdx.x; k < K; k += kActThreads)
        out[k] = (int8_t)quantize_one(kBf16 ? bf16_to_f32(rh[k]) : rf[k], inv);
}

hipError_t launch_quantize_acts(const void* x, bool bf16, int64_t M, int64_t K, int8_t* xq, float* sx,
                                hipStream_t stream) {
    const int elems = bf16 ? 8 : 4;
    const bool aligned = (reinterpret_cast<uintptr_t>(x) % 16 == 0) && (K % elems == 0) &&
                         (reinterpret_cast<uintptr_t>(xq) % 8 == 0);
    const bool fits = K / elems <= (int64_t)kActMaxVec * kActThreads;
    dim3 grid((unsigned)M), block(kActThreads);
    if (aligned && fits) {
        if (bf16) hipLaunchKernelGGL(quantize_acts_vec<true>, grid, block, 0, stream, x, K, xq, sx);
        else      hipLaunchKernelGGL(quantize_acts_vec<false>, grid, block, 0, stream, x, K, xq, sx);
    } else {
        if (bf16) hipLaunchKernelGGL(quantize_acts_any<true>, grid, block, 0, stream, x, K, xq, sx);
        else      hipLaunchKernelGGL(quantize_acts_any<false>, grid, block, 0, stream, x, K, xq, sx);
    }
    return hipGetLastError();
}

}  // namespace bitnet

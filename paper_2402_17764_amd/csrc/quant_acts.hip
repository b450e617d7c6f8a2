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
constexpr int kActMaxVec = 16;         // register-resident path: up to 16 x 16 bytes per thread (256 or 1024 threads)

__device__ inline int quantize_one(float v, float inv) { return (int)(int8_t)(quantize_bits(v, inv) & 0xFFu); }

template <int kWaves = kActWaves>
__device__ inline float block_max_nonneg(float v, float* sh) {
    v = wave_max_nonneg(v);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) sh[wave] = v;
    __syncthreads();
    float m = sh[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) m = fmaxf(m, sh[w]);
    return m;
}

// ---- register-resident vector path ----------------------------------------------------------------
// fp32: a 16-byte load is 4 elements -> 4 int8 = one 32-bit store.
// bf16: a 16-byte load is 8 elements -> 8 int8 = one 64-bit store.
// kVecs 16-byte loads per thread hold the token (the launcher picks the smallest that covers K, which keeps the
// register count and with it the number of resident tokens per CU in proportion to K); 1024 threads for the rows
// 256 threads cannot hold.
template <bool kBf16, int kVecs, int kThreads>
__global__ __launch_bounds__(kThreads) void quantize_acts_vec(const void* __restrict__ xv, int64_t K,
                                                              int8_t* __restrict__ xq, float* __restrict__ sx) {
    constexpr int kElems = kBf16 ? 8 : 4;
    __shared__ float sh[kThreads / kWave];
    const int64_t m = blockIdx.x;
    const int nvec = (int)(K / kElems);
    const uint4* row = reinterpret_cast<const uint4*>(static_cast<const char*>(xv) + m * K * (kBf16 ? 2 : 4));
    uint4 raw[kVecs];
    float amax = 0.0f;
#pragma unroll
    for (int v = 0; v < kVecs; ++v) {
        const int idx = v * kThreads + threadIdx.x;
        raw[v] = make_uint4(0, 0, 0, 0);
        if (idx < nvec) raw[v] = row[idx];
    }
#pragma unroll
    for (int v = 0; v < kVecs; ++v) {
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
    amax = block_max_nonneg<kThreads / kWave>(amax, sh);
    const float s = fmaxf(amax, kEps);
    const float inv = kQb / s;                             // one IEEE division per token
    if (threadIdx.x == 0) sx[m] = s;

    int8_t* out = xq + m * K;
#pragma unroll
    for (int v = 0; v < kVecs; ++v) {
        const int idx = v * kThreads + threadIdx.x;
        if (idx >= nvec) continue;
        const uint32_t u[4] = {raw[v].x, raw[v].y, raw[v].z, raw[v].w};
        if (kBf16) {
            const uint32_t lo = pack4_quantized(__uint_as_float(u[0] << 16), __uint_as_float(u[0] & 0xFFFF0000u),
                                                __uint_as_float(u[1] << 16), __uint_as_float(u[1] & 0xFFFF0000u), inv);
            const uint32_t hi = pack4_quantized(__uint_as_float(u[2] << 16), __uint_as_float(u[2] & 0xFFFF0000u),
                                                __uint_as_float(u[3] << 16), __uint_as_float(u[3] & 0xFFFF0000u), inv);
            reinterpret_cast<uint2*>(out)[idx] = make_uint2(lo, hi);
        } else {
            reinterpret_cast<uint32_t*>(out)[idx] = pack4_quantized(__uint_as_float(u[0]), __uint_as_float(u[1]), __uint_as_float(u[2]),
                                                                    __uint_as_float(u[3]), inv);
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

// ---------------------------------------------------------------------------------------------------
// Producers of int8 activations: the operations that precede a BitLinear layer in a LLaMA-style block
// (Section 2, "LLaMA-alike components": RMSNorm, SwiGLU) with the activation quantization fused in,
// so that the normalised / gated activations never travel through HBM as bf16.
// ---------------------------------------------------------------------------------------------------
constexpr int kProdMaxChunks = 16;     // register-resident path: up to 16 chunks of 4 elements per thread (256 or 1024 threads)

// four consecutive elements of a row, widened to fp32 (k is a multiple of 4; the row is 16- / 8-byte aligned)
template <bool kBf16>
__device__ inline void load_chunk(const void* row, int64_t k, float (&f)[4]) {
    if (kBf16) {
        const uint2 u = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(row) + k);
        f[0] = __uint_as_float(u.x << 16);
        f[1] = __uint_as_float(u.x & 0xFFFF0000u);
        f[2] = __uint_as_float(u.y << 16);
        f[3] = __uint_as_float(u.y & 0xFFFF0000u);
    } else {
        const float4 v = *reinterpret_cast<const float4*>(static_cast<const float*>(row) + k);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
}
template <bool kBf16>
__device__ inline float load_elem(const void* row, int64_t k) {
    return kBf16 ? bf16_to_f32(static_cast<const uint16_t*>(row)[k]) : static_cast<const float*>(row)[k];
}

__device__ inline uint32_t pack4(const float (&v)[4], float inv) { return pack4_quantized(v[0], v[1], v[2], v[3], inv); }

// RMSNorm -> absmax int8.  Per token: ms = mean of squares (exact: squares of fp32 values are exact in
// fp64 and the sum is carried in double-double), r = (float)(1 / sqrt(ms + eps)) in fp64, z = (x * r) * g
// in fp32, then the per-token quantization of z.  kChunks > 0: the token stays in registers between the passes,
// kChunks chunks of four elements per thread (the launcher picks the smallest count that covers K); 0: three sweeps
// over memory, any K.  The gain is requested together with the token where it costs few registers (up to eight
// chunks: its latency would otherwise sit in the token's dependent chain) and loaded where
// it is used otherwise.
template <bool kBf16, int kChunks, int kThreads>
__global__ __launch_bounds__(kThreads) void rmsnorm_quantize_kernel(
        const void* __restrict__ xv, const float* __restrict__ g, float eps, int64_t K, int8_t* __restrict__ xq,
        float* __restrict__ sx) {
    constexpr int kWaves = kThreads / kWave;
    constexpr bool kVec = kChunks > 0, kHoldGain = kChunks > 0 && kChunks <= 8;
    __shared__ double sh_hi[kWaves], sh_lo[kWaves];
    __shared__ float sh[kWaves];
    const int64_t m = blockIdx.x;
    const void* row = static_cast<const char*>(xv) + m * K * (kBf16 ? 2 : 4);
    int8_t* out = xq + m * K;
    const int nchunks = (int)(K / 4);
    float v[kVec ? kChunks : 1][4], gv[kHoldGain ? kChunks : 1][4];

    // four interleaved double-double accumulators: the sums are exact, so splitting them changes nothing
    // but the length of the dependent chain
    dd acc{0.0, 0.0}, acc2{0.0, 0.0}, acc3{0.0, 0.0}, acc4{0.0, 0.0};
    if (kVec) {
#pragma unroll
        for (int i = 0; i < kChunks; ++i) {
            if (i * kThreads >= nchunks) continue;              // uniform: whole iterations past the row
            const int c = i * kThreads + threadIdx.x;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[i][e] = 0.0f;
            if (c < nchunks) {
                load_chunk<kBf16>(row, 4 * (int64_t)c, v[i]);
                if (kHoldGain && g) {                              // requested now, needed after the reduction
#pragma unroll
                    for (int e = 0; e < 4; ++e) gv[i][e] = g[4 * c + e];
                }
            }
        }
#pragma unroll
        for (int i = 0; i < kChunks; ++i) {
            if (i * kThreads >= nchunks) continue;
            dd_add_double(acc, (double)v[i][0] * (double)v[i][0]);
            dd_add_double(acc2, (double)v[i][1] * (double)v[i][1]);
            dd_add_double(acc3, (double)v[i][2] * (double)v[i][2]);
            dd_add_double(acc4, (double)v[i][3] * (double)v[i][3]);
        }
        dd_add_dd(acc, acc2);
        dd_add_dd(acc3, acc4);
        dd_add_dd(acc, acc3);
    } else {
        for (int64_t k = threadIdx.x; k < K; k += kThreads) {
            const double a = (double)load_elem<kBf16>(row, k);
            dd_add_double(acc, a * a);
        }
    }
    const double ms = block_sum_dd<kWaves>(acc, sh_hi, sh_lo) / (double)K;
    const float r = (float)(1.0 / sqrt(ms + (double)eps));

    float amax = 0.0f;
    if (kVec) {
#pragma unroll
        for (int i = 0; i < kChunks; ++i) {
            if (i * kThreads >= nchunks) continue;              // uniform: whole iterations past the row
            const int c = i * kThreads + threadIdx.x;
            if (c < nchunks) {
                float gl[4] = {1.0f, 1.0f, 1.0f, 1.0f};
                if (g) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) gl[e] = kHoldGain ? gv[i][e] : g[4 * c + e];
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float z = v[i][e] * r;
                    if (g) z = z * gl[e];
                    v[i][e] = z;
                    amax = fmaxf(amax, fabsf(z));
                }
            }
        }
    } else {
        for (int64_t k = threadIdx.x; k < K; k += kThreads) {
            float z = load_elem<kBf16>(row, k) * r;
            if (g) z = z * g[k];
            amax = fmaxf(amax, fabsf(z));
        }
    }
    amax = block_max_nonneg<kWaves>(amax, sh);
    const float s = fmaxf(amax, kEps);
    const float inv = kQb / s;
    if (threadIdx.x == 0) sx[m] = s;

    if (kVec) {
#pragma unroll
        for (int i = 0; i < kChunks; ++i) {
            if (i * kThreads >= nchunks) continue;              // uniform: whole iterations past the row
            const int c = i * kThreads + threadIdx.x;
            if (c < nchunks) reinterpret_cast<uint32_t*>(out)[c] = pack4(v[i], inv);
        }
    } else {
        for (int64_t k = threadIdx.x; k < K; k += kThreads) {
            float z = load_elem<kBf16>(row, k) * r;                // the same two multiplies: the same z
            if (g) z = z * g[k];
            out[k] = (int8_t)quantize_one(z, inv);
        }
    }
}

// SwiGLU gating -> absmax int8.  gu is [M][2F]: h = silu(gu[:, :F]) * gu[:, F:], then the per-token
// quantization of h.
template <bool kBf16, int kChunks, int kThreads>
__global__ __launch_bounds__(kThreads) void swiglu_quantize_kernel(
        const void* __restrict__ guv, int64_t F, int8_t* __restrict__ hq, float* __restrict__ sh_out) {
    constexpr int kWaves = kThreads / kWave;
    constexpr bool kVec = kChunks > 0;                             // as for rmsnorm_quantize_kernel
    __shared__ float sh[kWaves];
    const int64_t m = blockIdx.x;
    const void* gate = static_cast<const char*>(guv) + m * 2 * F * (kBf16 ? 2 : 4);
    const void* up = static_cast<const char*>(gate) + F * (kBf16 ? 2 : 4);
    int8_t* out = hq + m * F;
    const int nchunks = (int)(F / 4);
    float v[kVec ? kChunks : 1][4];

    float amax = 0.0f;
    if (kVec) {
#pragma unroll
        for (int i = 0; i < kChunks; ++i) {
            if (i * kThreads >= nchunks) continue;              // uniform: whole iterations past the row
            const int c = i * kThreads + threadIdx.x;
            if (c < nchunks) {
                float a[4], b[4];
                load_chunk<kBf16>(gate, 4 * (int64_t)c, a);
                load_chunk<kBf16>(up, 4 * (int64_t)c, b);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[i][e] = swiglu_one(a[e], b[e]);
                    amax = fmaxf(amax, fabsf(v[i][e]));
                }
            }
        }
    } else {
        for (int64_t f = threadIdx.x; f < F; f += kThreads)
            amax = fmaxf(amax, fabsf(swiglu_one(load_elem<kBf16>(gate, f), load_elem<kBf16>(up, f))));
    }
    amax = block_max_nonneg<kWaves>(amax, sh);
    const float s = fmaxf(amax, kEps);
    const float inv = kQb / s;
    if (threadIdx.x == 0) sh_out[m] = s;

    if (kVec) {
#pragma unroll
        for (int i = 0; i < kChunks; ++i) {
            if (i * kThreads >= nchunks) continue;              // uniform: whole iterations past the row
            const int c = i * kThreads + threadIdx.x;
            if (c < nchunks) reinterpret_cast<uint32_t*>(out)[c] = pack4(v[i], inv);
        }
    } else {
        for (int64_t f = threadIdx.x; f < F; f += kThreads)
            out[f] = (int8_t)quantize_one(swiglu_one(load_elem<kBf16>(gate, f), load_elem<kBf16>(up, f)), inv);
    }
}

// Few tokens: 1024 threads per token, so that the dependent chains of the gate (exponential, division) and
// of the exact sum interleave over four waves per SIMD; many tokens: 256, and the tokens fill the CUs.  Rows too
// long for 256 threads' registers take 1024 threads at any token count.
constexpr int kProdFewTokens = 64;

// chunks of four: rows must start on a chunk boundary of the input loads and of the 32-bit stores
static bool producer_vec_ok(const void* in, size_t esz, int64_t cols, const void* out) {
    return cols % 4 == 0 && cols <= (int64_t)kProdMaxChunks * 1024 * 4 &&
           reinterpret_cast<uintptr_t>(in) % (4 * esz) == 0 && reinterpret_cast<uintptr_t>(out) % 4 == 0;
}

// threads per token and register chunks per thread for a row of `cols` elements (chunks == 0: the sweeping form)
static void producer_shape(bool vec, int64_t M, int64_t cols, int* threads, int* chunks) {
    *threads = (M < kProdFewTokens || cols > (int64_t)kProdMaxChunks * 256 * 4) ? 1024 : 256;
    *chunks = 0;
    if (!vec) return;
    const int64_t need = ceil_div(cols, (int64_t)*threads * 4);
    *chunks = need <= 4 ? 4 : need <= 8 ? 8 : 16;
}

#define PRODUCER_PICK(B_)                                                                                        \
    do {                                                                                                         \
        if (threads == 1024) {                                                                                   \
            if (chunks == 4) GO(B_, 4, 1024); else if (chunks == 8) GO(B_, 8, 1024);                             \
            else if (chunks == 16) GO(B_, 16, 1024); else GO(B_, 0, 1024);                                       \
        } else {                                                                                                 \
            if (chunks == 4) GO(B_, 4, 256); else if (chunks == 8) GO(B_, 8, 256);                               \
            else if (chunks == 16) GO(B_, 16, 256); else GO(B_, 0, 256);                                         \
        }                                                                                                        \
    } while (0)

hipError_t launch_rmsnorm_quantize(const void* x, bool bf16, const float* g, float eps, int64_t M, int64_t K,
                                   int8_t* xq, float* sx, hipStream_t stream) {
    int threads, chunks;
    producer_shape(producer_vec_ok(x, bf16 ? 2 : 4, K, xq), M, K, &threads, &chunks);
    dim3 grid((unsigned)M), block(threads);
#define GO(B_, C_, T_) hipLaunchKernelGGL((rmsnorm_quantize_kernel<B_, C_, T_>), grid, block, 0, stream, x, g, eps, K, xq, sx)
    if (bf16) PRODUCER_PICK(true); else PRODUCER_PICK(false);
#undef GO
    return hipGetLastError();
}

hipError_t launch_swiglu_quantize(const void* gu, bool bf16, int64_t M, int64_t F, int8_t* hq, float* sh,
                                  hipStream_t stream) {
    int threads, chunks;
    producer_shape(producer_vec_ok(gu, bf16 ? 2 : 4, F, hq), M, F, &threads, &chunks);
    dim3 grid((unsigned)M), block(threads);
#define GO(B_, C_, T_) hipLaunchKernelGGL((swiglu_quantize_kernel<B_, C_, T_>), grid, block, 0, stream, gu, F, hq, sh)
    if (bf16) PRODUCER_PICK(true); else PRODUCER_PICK(false);
#undef GO
    return hipGetLastError();
}
#undef PRODUCER_PICK

hipError_t launch_quantize_acts(const void* x, bool bf16, int64_t M, int64_t K, int8_t* xq, float* sx,
                                hipStream_t stream) {
    const int elems = bf16 ? 8 : 4;
    const bool aligned = (reinterpret_cast<uintptr_t>(x) % 16 == 0) && (K % elems == 0) &&
                         (reinterpret_cast<uintptr_t>(xq) % 8 == 0);
    const int64_t nvec = K / elems;
    const int threads = nvec <= (int64_t)kActMaxVec * kActThreads ? kActThreads : 1024;
    const int64_t need = ceil_div(nvec, threads);
    dim3 grid((unsigned)M), block(threads);
#define GO(B_, V_, T_) hipLaunchKernelGGL((quantize_acts_vec<B_, V_, T_>), grid, block, 0, stream, x, K, xq, sx)
#define PICK(B_)                                                                                                 \
    do {                                                                                                         \
        if (threads == 1024) { if (need <= 8) GO(B_, 8, 1024); else if (!B_) GO(false, 16, 1024); }              \
        else if (need <= 2) GO(B_, 2, kActThreads);                                                              \
        else if (need <= 4) GO(B_, 4, kActThreads);                                                              \
        else if (need <= 8) GO(B_, 8, kActThreads);                                                              \
        else GO(B_, 16, kActThreads);                                                                            \
    } while (0)
    // (bf16 at 1024 threads and 16 loads per thread would spill: such rows, beyond 65536 elements, sweep instead)
    if (aligned && need <= ((threads == 1024 && bf16) ? 8 : kActMaxVec)) {
        if (bf16) PICK(true); else PICK(false);
    } else {
        block = dim3(kActThreads);
        if (bf16) hipLaunchKernelGGL(quantize_acts_any<true>, grid, block, 0, stream, x, K, xq, sx);
        else      hipLaunchKernelGGL(quantize_acts_any<false>, grid, block, 0, stream, x, K, xq, sx);
    }
#undef GO
#undef PICK
    return hipGetLastError();
}

}  // namespace bitnet

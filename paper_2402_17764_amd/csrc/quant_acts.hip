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
    if (kWaves == 1) return v;
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

// one 16-byte piece of a row widened to fp32: eight bf16 or four fp32 elements
template <bool kBf16>
__device__ inline void expand_vec(const uint4& q, float (&f)[kBf16 ? 8 : 4]) {
    const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (kBf16) {
            f[2 * e] = __uint_as_float(u[e] << 16);
            f[2 * e + 1] = __uint_as_float(u[e] & 0xFFFF0000u);
        } else {
            f[e] = __uint_as_float(u[e]);
        }
    }
}

// r = (float)(1 / sqrt(mean(x^2) + eps)) from the threads' double-double partial sums of squares.  Every wave adds
// up its lanes; wave 0 alone then adds the waves, divides and takes the root in fp64 -- a hundred dependent
// instructions that the other waves' SIMDs can give to other tokens meanwhile -- and hands r over through LDS.
template <int kWaves>
__device__ inline float rms_scale(dd v, int64_t K, float eps, double* sh_hi, double* sh_lo, float* shr) {
    const dd w = wave_sum_dd(v);
    if (kWaves == 1) return (float)(1.0 / sqrt((w.hi + w.lo) / (double)K + (double)eps));
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { sh_hi[wave] = w.hi; sh_lo[wave] = w.lo; }
    __syncthreads();
    if (wave == 0) {
        dd t{sh_hi[0], sh_lo[0]};
#pragma unroll
        for (int q = 1; q < kWaves; ++q) dd_add_dd(t, dd{sh_hi[q], sh_lo[q]});
        const double ms = (t.hi + t.lo) / (double)K;
        const float r = (float)(1.0 / sqrt(ms + (double)eps));
        if (threadIdx.x == 0) shr[0] = r;
    }
    __syncthreads();
    return shr[0];
}

// RMSNorm -> absmax int8.  Per token: ms = mean of squares (exact: squares of fp32 values are exact in
// fp64 and the sum is carried in double-double), r = (float)(1 / sqrt(ms + eps)) in fp64, z = (x * r) * g
// in fp32, then the per-token quantization of z.
//
// Register-resident form: the token is read once, kVecs 16-byte loads per thread (the launcher picks the smallest
// count that covers K), and stays in registers *as loaded* -- bf16 pairs are widened where they are used -- so that a
// workgroup needs few registers and a CU holds many tokens at different stages: the kernel does more arithmetic than
// memory traffic (nine fp64 operations per element for the exact sum), and only tokens in other phases can hide one
// token's loads and reductions.  z is kept in registers between the absmax and the rounding where that takes at most
// 32 of them and recomputed with the same two multiplications otherwise.
template <bool kBf16, int kVecs, int kThreads>
__global__ __launch_bounds__(kThreads) void rmsnorm_quantize_vec(
        const void* __restrict__ xv, const float* __restrict__ g, float eps, int64_t K, int8_t* __restrict__ xq,
        float* __restrict__ sx) {
    constexpr int kElems = kBf16 ? 8 : 4;
    constexpr int kWaves = kThreads / kWave;
    constexpr bool kKeepZ = kVecs * kElems <= 32;
    __shared__ double sh_hi[kWaves], sh_lo[kWaves];
    __shared__ float sh[kWaves + 1];                               // the waves' maxima; r of the token behind them
    const int64_t m = blockIdx.x;
    const int nvec = (int)(K / kElems);
    const uint4* row = reinterpret_cast<const uint4*>(static_cast<const char*>(xv) + m * K * (kBf16 ? 2 : 4));
    const float4* g4 = reinterpret_cast<const float4*>(g);
    uint4 raw[kVecs];
#pragma unroll
    for (int v = 0; v < kVecs; ++v) {
        const int idx = v * kThreads + threadIdx.x;
        raw[v] = make_uint4(0, 0, 0, 0);
        if (idx < nvec) raw[v] = row[idx];
    }

    // four interleaved double-double accumulators: the sums are exact, so splitting them changes nothing
    // but the length of the dependent chain (vectors past the row hold zeros and are skipped whole)
    dd acc[4] = {{0.0, 0.0}, {0.0, 0.0}, {0.0, 0.0}, {0.0, 0.0}};
#pragma unroll
    for (int v = 0; v < kVecs; ++v) {
        if (v * kThreads >= nvec) continue;                     // uniform
        float f[kElems];
        expand_vec<kBf16>(raw[v], f);
#pragma unroll
        for (int e = 0; e < kElems; ++e) dd_add_double(acc[e & 3], (double)f[e] * (double)f[e]);
    }
    dd_add_dd(acc[0], acc[1]);
    dd_add_dd(acc[2], acc[3]);
    dd_add_dd(acc[0], acc[2]);
    const float r = rms_scale<kWaves>(acc[0], K, eps, sh_hi, sh_lo, sh + kWaves);

    // z = (x * r) * g of one vector; the gain comes from the caches (every token reads the same K floats)
    auto scaled = [&](int v, int idx, float (&z)[kElems]) {
        expand_vec<kBf16>(raw[v], z);
        float gl[kElems];
        if (g) {
#pragma unroll
            for (int q = 0; q < kElems / 4; ++q) {
                const float4 t = g4[idx * (kElems / 4) + q];
                gl[4 * q] = t.x; gl[4 * q + 1] = t.y; gl[4 * q + 2] = t.z; gl[4 * q + 3] = t.w;
            }
        }
#pragma unroll
        for (int e = 0; e < kElems; ++e) {
            z[e] = z[e] * r;
            if (g) z[e] = z[e] * gl[e];
        }
    };

    float zk[kKeepZ ? kVecs : 1][kElems];
    float amax = 0.0f;
#pragma unroll
    for (int v = 0; v < kVecs; ++v) {
        const int idx = v * kThreads + threadIdx.x;
        if (v * kThreads >= nvec) continue;                     // uniform
        if (idx < nvec) {
            float z[kElems];
            scaled(v, idx, z);
#pragma unroll
            for (int e = 0; e < kElems; ++e) {
                amax = fmaxf(amax, fabsf(z[e]));
                if (kKeepZ) zk[v][e] = z[e];
            }
        }
    }
    amax = block_max_nonneg<kWaves>(amax, sh);
    const float s = fmaxf(amax, kEps);
    const float inv = kQb / s;
    if (threadIdx.x == 0) sx[m] = s;

    int8_t* out = xq + m * K;
#pragma unroll
    for (int v = 0; v < kVecs; ++v) {
        const int idx = v * kThreads + threadIdx.x;
        if (v * kThreads >= nvec) continue;                     // uniform
        if (idx >= nvec) continue;
        float z[kElems];
        if (kKeepZ) {
#pragma unroll
            for (int e = 0; e < kElems; ++e) z[e] = zk[v][e];
        } else {
            scaled(v, idx, z);                                  // the same two multiplications: the same z
        }
        if (kBf16) {
            reinterpret_cast<uint2*>(out)[idx] = make_uint2(pack4_quantized(z[0], z[1], z[2], z[3], inv),
                                                            pack4_quantized(z[4], z[5], z[6], z[7], inv));
        } else {
            reinterpret_cast<uint32_t*>(out)[idx] = pack4_quantized(z[0], z[1], z[2], z[3], inv);
        }
    }
}

// Any K and any alignment: three sweeps over the token in memory, element loads.
template <bool kBf16, int kThreads>
__global__ __launch_bounds__(kThreads) void rmsnorm_quantize_any(
        const void* __restrict__ xv, const float* __restrict__ g, float eps, int64_t K, int8_t* __restrict__ xq,
        float* __restrict__ sx) {
    constexpr int kWaves = kThreads / kWave;
    __shared__ double sh_hi[kWaves], sh_lo[kWaves];
    __shared__ float sh[kWaves + 1];                               // the waves' maxima; r of the token behind them
    const int64_t m = blockIdx.x;
    const void* row = static_cast<const char*>(xv) + m * K * (kBf16 ? 2 : 4);
    int8_t* out = xq + m * K;
    dd acc{0.0, 0.0};
    for (int64_t k = threadIdx.x; k < K; k += kThreads) {
        const double a = (double)load_elem<kBf16>(row, k);
        dd_add_double(acc, a * a);
    }
    const float r = rms_scale<kWaves>(acc, K, eps, sh_hi, sh_lo, sh + kWaves);
    float amax = 0.0f;
    for (int64_t k = threadIdx.x; k < K; k += kThreads) {
        float z = load_elem<kBf16>(row, k) * r;
        if (g) z = z * g[k];
        amax = fmaxf(amax, fabsf(z));
    }
    amax = block_max_nonneg<kWaves>(amax, sh);
    const float s = fmaxf(amax, kEps);
    const float inv = kQb / s;
    if (threadIdx.x == 0) sx[m] = s;
    for (int64_t k = threadIdx.x; k < K; k += kThreads) {
        float z = load_elem<kBf16>(row, k) * r;                    // the same two multiplies: the same z
        if (g) z = z * g[k];
        out[k] = (int8_t)quantize_one(z, inv);
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
    const int elems = bf16 ? 8 : 4;
    const int max_vecs = bf16 ? 8 : 16;                            // 64 token elements per thread at most
    const bool aligned = K % elems == 0 && reinterpret_cast<uintptr_t>(x) % 16 == 0 &&
                         reinterpret_cast<uintptr_t>(xq) % (bf16 ? 8 : 4) == 0 && reinterpret_cast<uintptr_t>(g) % 16 == 0;
    const int64_t nvec = K / elems;
    // few tokens: 1024 threads each, so that the dependent chains of the exact sum interleave over four waves per
    // SIMD; many tokens: 256, and the tokens fill the CUs (one or two waves per token were measured too: slower at
    // every size from 64 to 4096 tokens); rows that would need more than eight loads per thread at 256 threads
    // take 1024 at any count (sixteen loads cost occupancy: fp32 rows of 13824 run 5-15 % faster on 1024 threads)
    const int threads = (M < kProdFewTokens || nvec > (int64_t)8 * 256) ? 1024 : 256;
    const int64_t need = ceil_div(nvec, threads);
    dim3 grid((unsigned)M), block(threads);
#define GO(B_, V_, T_) hipLaunchKernelGGL((rmsnorm_quantize_vec<B_, V_, T_>), grid, block, 0, stream, x, g, eps, K, xq, sx)
#define PICK(B_, T_)                                                                                             \
    do {                                                                                                         \
        if (need <= 1) GO(B_, 1, T_); else if (need <= 2) GO(B_, 2, T_); else if (need <= 4) GO(B_, 4, T_);      \
        else if (need <= 8) GO(B_, 8, T_); else if (!B_ && T_ == 1024) GO(false, 16, 1024);                      \
    } while (0)
    if (aligned && need <= max_vecs) {
        if (bf16) { if (threads == 1024) PICK(true, 1024); else PICK(true, 256); }
        else      { if (threads == 1024) PICK(false, 1024); else PICK(false, 256); }
    } else {
        if (bf16) {
            if (threads >= 1024) hipLaunchKernelGGL((rmsnorm_quantize_any<true, 1024>), grid, block, 0, stream, x, g, eps, K, xq, sx);
            else                 hipLaunchKernelGGL((rmsnorm_quantize_any<true, 256>), grid, block, 0, stream, x, g, eps, K, xq, sx);
        } else {
            if (threads >= 1024) hipLaunchKernelGGL((rmsnorm_quantize_any<false, 1024>), grid, block, 0, stream, x, g, eps, K, xq, sx);
            else                 hipLaunchKernelGGL((rmsnorm_quantize_any<false, 256>), grid, block, 0, stream, x, g, eps, K, xq, sx);
        }
    }
#undef GO
#undef PICK
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

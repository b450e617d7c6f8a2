// Weight-streaming BitLinear kernel for decode (M <= 16; the batched-decode kernels for up to 64 tokens are in
// linear_skinny.hip) on gfx950, with the fused activation quantization and its pre-operations.
//
// They compute acc[m][n] = sum_k x_q[m][k] * Wt[n][k] exactly in int32 and
// y = acc * gamma * s_x[m] / 127 (Sections 1-2 of arXiv 2402.17764).  At these M the cost is moving
// the packed weights out of HBM, so the kernels are organised around that stream:
//
//   * one 128-bit load per lane fetches one quad (64 codes of one row); the 64 lanes of a wavefront
//     fetch one (step, row block) chunk = 1 KiB of contiguous memory per load instruction, and
//     because the packed layout is step-major, all waves working on the same step read one dense run;
//   * a 32-bit word of 2-bit two's-complement codes becomes four int8 MFMA operand registers with one
//     shift and one AND each: (w << (6 - 2 i)) & 0xC0C0C0C0 leaves 64 * code in every byte, so no
//     multiply and no sign fix-up is spent on decoding; the factor 64 is shifted out of the int32
//     accumulator at the end (exact, |64 * 127 * K| < 2^31);
//   * the contraction runs on v_mfma_i32_16x16x64_i8 with the 16 weight rows as the A operand and 16
//     tokens as the B operand; the matrix pipe is otherwise idle in a bandwidth-bound kernel, and
//     M = 1 ... 16 cost the same;
//   * the K loop has no branch and no guarded load: steps, row blocks and tokens beyond the matrix
//     are redirected to valid addresses and their weights ANDed with zero, so loads for the next
//     kD steps are always in flight under the current step's MFMAs;
//   * waves that split K fold their partial accumulators through LDS in a fixed order (integer adds:
//     exact and deterministic).
//
// Lane l of a wave supplies row (l & 15) and the columns of quad (l >> 4) of the current step; the
// activation operand of lane l is token (l & 15), same columns, so every product pairs the same k.
#include "gemv_common.hpp"

namespace bitnet {

// ---------------------------------------------------------------------------------------------------
// M <= 16 (the product on pre-quantized activations uses it up to M = 4, the fused entry point up to 16)
// ---------------------------------------------------------------------------------------------------
// Where the activation operand comes from.
enum XMode : int {
    kXGlobal = 0,      // int8 x_q read from global memory with every step
    kXLds = 1,         // int8 x_q copied once per workgroup into LDS
    kXFusedBf16 = 2,   // bf16 x: per-token absmax quantization done in the kernel, x_q lives only in LDS
    kXFusedF32 = 3,    // fp32 x, same
    kXNormBf16 = 4,    // bf16 x: RMSNorm (with an optional gain) and the quantization done in the kernel
    kXNormF32 = 5,     // fp32 x, same
    kXSwigluBf16 = 6,  // bf16 [gate | up] rows of 2 K elements: SwiGLU gating and the quantization done in the kernel
    kXSwigluF32 = 7    // fp32, same
};
// what the fused modes do to a token before its absmax quantization
enum PreOp : int { kPreNone = 0, kPreRmsNorm = 1, kPreSwiglu = 2 };

// uint4 slots in front of the x region: 16 floats of reduction scratch, 16 floats of s_x, 2 x 16 doubles for the
// double-double reduction of the RMSNorm modes
constexpr int kGemvLdsHeader = 32;

// In-kernel activation quantization for the fused modes (Section 2 of the paper: per-token absmax,
// Q_b = 127), the same arithmetic as the stand-alone activation kernel: s = max(absmax, 1e-5),
// inv = 127 / s, x_q = clip(rint(x * inv)).  Rows land in LDS zero padded to Kpad columns, s_x[m] in
// sxl[m].  Token 0 is fetched into registers before the weight prefetch is issued (so that waiting for
// it does not wait for the weights) and quantized from there; further tokens take two sweeps.
constexpr int kFusedRegVecs = 4;          // 16-byte vectors of token 0 a thread can hold
// ... and how many of them also get their RMSNorm gain prefetched (the rest read it after the reduction);
// the 1024-thread workgroups have 128 registers per lane and none to spare
constexpr int gain_reg_vecs(int threads) { return threads >= 1024 ? 0 : 2; }

template <bool kBf16>
__device__ inline float vec_absmax(const uint4& q, float amax) {
    const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (kBf16) {
            amax = fmaxf(amax, fabsf(__uint_as_float(u[e] << 16)));
            amax = fmaxf(amax, fabsf(__uint_as_float(u[e] & 0xFFFF0000u)));
        } else {
            amax = fmaxf(amax, fabsf(__uint_as_float(u[e])));
        }
    }
    return amax;
}

// Four values -> four int8 codes in one word (pack4_quantized: the stand-alone quantizers' own arithmetic).
__device__ inline uint32_t pack4_codes(float a, float b, float c, float d, float inv) { return pack4_quantized(a, b, c, d, inv); }

// one 16-byte vector of x -> its int8 codes, written to the token's LDS row (32-bit words)
template <bool kBf16>
__device__ inline void vec_quantize_store(const uint4& q, float inv, uint32_t* out, int v) {
    const uint32_t u[4] = {q.x, q.y, q.z, q.w};
    if (kBf16) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
            out[2 * v + h] = pack4_codes(__uint_as_float(u[2 * h] << 16), __uint_as_float(u[2 * h] & 0xFFFF0000u),
                                         __uint_as_float(u[2 * h + 1] << 16), __uint_as_float(u[2 * h + 1] & 0xFFFF0000u), inv);
    } else {
        out[v] = pack4_codes(__uint_as_float(u[0]), __uint_as_float(u[1]), __uint_as_float(u[2]), __uint_as_float(u[3]), inv);
    }
}

template <int kThreads>
__device__ inline float block_absmax_to_scale(float amax, float* red) {
    amax = wave_max_nonneg(amax);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = amax;
    __syncthreads();
    float mx = red[0];
#pragma unroll
    for (int w = 1; w < kThreads / kWave; ++w) mx = fmaxf(mx, red[w]);
    return fmaxf(mx, kEps);
}

// a 16-byte vector of x widened to fp32
template <bool kBf16>
__device__ inline void vec_expand(const uint4& q, float (&f)[kBf16 ? 8 : 4]) {
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

// kPre == kPreRmsNorm: the token first goes through RMSNorm, z = (x * r) * gain with
// r = (float)(1 / sqrt(mean(x^2) + eps)), the mean of squares exact (fp64 squares of fp32 values, double-double
// sums).  kPre == kPreSwiglu: the token is a [gate | up] row of 2 K elements and h = silu(gate) * up is what gets
// quantized.  Both are the arithmetic of the stand-alone producer kernels, so they give the same codes and scales
// (Section 2 of the paper, LLaMA-alike components: RMSNorm in front of the attention and feed-forward BitLinear
// layers, SwiGLU in front of the down projection).
template <bool kBf16, int kPre, int kThreads>
__device__ inline void fused_quantize_to_lds(const void* __restrict__ xv, const uint4 (&row0)[kFusedRegVecs],
                                             const uint4 (&up0)[kFusedRegVecs] /* SwiGLU: the up half of token 0 */,
                                             bool row0_in_regs,
                                             const float4 (&gain0)[2][kBf16 ? 2 : 1] /* gain of row0's first columns */,
                                             int M, int64_t K, int Kpad, const float* __restrict__ gain, float eps,
                                             float* red, float* sxl, uint4* xlds) {
    constexpr int kE = kBf16 ? 8 : 4;                 // elements per 16-byte vector
    constexpr int kWaves = kThreads / kWave;
    constexpr bool kNorm = kPre == kPreRmsNorm, kSwiglu = kPre == kPreSwiglu;
    const int nvec = (int)(K / kE);
    const int nvec_pad = Kpad / kE;
    const int64_t row_bytes = (kSwiglu ? 2 : 1) * K * (kBf16 ? 2 : 4);
    double* sh_hi = reinterpret_cast<double*>(red + 32);
    double* sh_lo = sh_hi + 16;
    for (int m = 0; m < M; ++m) {
        const uint4* row = reinterpret_cast<const uint4*>(static_cast<const char*>(xv) + (int64_t)m * row_bytes);
        uint32_t* out = reinterpret_cast<uint32_t*>(xlds) + (size_t)m * (Kpad >> 2);
        const bool regs = m == 0 && row0_in_regs;
        float r = 1.0f;
        if (kNorm) {
            // two interleaved accumulators: the sums are exact, so splitting them only shortens the dependent chain
            dd acc{0.0, 0.0}, acc2{0.0, 0.0};
            auto add_squares = [&](const uint4& q) {
                float f[kE];
                vec_expand<kBf16>(q, f);
#pragma unroll
                for (int e = 0; e < kE; e += 2) {
                    dd_add_double(acc, (double)f[e] * (double)f[e]);
                    dd_add_double(acc2, (double)f[e + 1] * (double)f[e + 1]);
                }
            };
            if (regs) {
#pragma unroll
                for (int v = 0; v < kFusedRegVecs; ++v)
                    if (v * kThreads + (int)threadIdx.x < nvec) add_squares(row0[v]);     // clamped duplicates do not count
            } else {
                for (int v = threadIdx.x; v < nvec; v += kThreads) add_squares(row[v]);
            }
            dd_add_dd(acc, acc2);
            const double ms = block_sum_dd<kWaves>(acc, sh_hi, sh_lo) / (double)K;
            r = (float)(1.0 / sqrt(ms + (double)eps));
        }
        // The values that get quantized, for one vector of columns (kNorm, kSwiglu): the same operations wherever
        // they are evaluated, so the same values.  slot >= 0: vector `slot` of the token held in registers.
        auto values = [&](const uint4& q, const uint4& qu, int v, int slot, float (&f)[kE]) {
            vec_expand<kBf16>(q, f);
            if (kNorm) {
#pragma unroll
                for (int e = 0; e < kE; ++e) f[e] = f[e] * r;
                if (gain) {
#pragma unroll
                    for (int h = 0; h < kE / 4; ++h) {
                        const float4 gq = (slot >= 0 && slot < gain_reg_vecs(kThreads)) ? gain0[slot][h]
                                                                                        : *reinterpret_cast<const float4*>(gain + (size_t)v * kE + 4 * h);
                        f[4 * h] = f[4 * h] * gq.x; f[4 * h + 1] = f[4 * h + 1] * gq.y;
                        f[4 * h + 2] = f[4 * h + 2] * gq.z; f[4 * h + 3] = f[4 * h + 3] * gq.w;
                    }
                }
            }
            if (kSwiglu) {
                float u[kE];
                vec_expand<kBf16>(qu, u);
#pragma unroll
                for (int e = 0; e < kE; ++e) f[e] = swiglu_one(f[e], u[e]);
            }
        };
        auto absmax_floats = [&](const float (&f)[kE], float amax) {
#pragma unroll
            for (int e = 0; e < kE; ++e) amax = fmaxf(amax, fabsf(f[e]));
            return amax;
        };
        auto store_floats = [&](const float (&f)[kE], int v, float inv) {
#pragma unroll
            for (int h = 0; h < kE / 4; ++h)
                out[(kE / 4) * v + h] = pack4_codes(f[4 * h], f[4 * h + 1], f[4 * h + 2], f[4 * h + 3], inv);
        };
        float hk[kSwiglu ? kFusedRegVecs : 1][kE];     // SwiGLU: the gated values of token 0 stay in registers
        float amax = 0.0f;
        if (regs) {
#pragma unroll
            for (int v = 0; v < kFusedRegVecs; ++v) {
                const int idx = v * kThreads + (int)threadIdx.x;
                if (kPre == kPreNone) {
                    amax = vec_absmax<kBf16>(row0[v], amax);        // clamped duplicates are harmless, cheaper than a branch
                } else if (idx < nvec) {
                    float f[kE];
                    values(row0[v], up0[v], idx, v, f);
                    amax = absmax_floats(f, amax);
                    if (kSwiglu) {
#pragma unroll
                        for (int e = 0; e < kE; ++e) hk[kSwiglu ? v : 0][e] = f[e];
                    }
                }
            }
        } else {
            for (int v = threadIdx.x; v < nvec; v += kThreads) {
                if (kPre == kPreNone) {
                    amax = vec_absmax<kBf16>(row[v], amax);
                } else {
                    float f[kE];
                    values(row[v], row[kSwiglu ? nvec + v : v], v, -1, f);
                    amax = absmax_floats(f, amax);
                }
            }
        }
        const float sc = block_absmax_to_scale<kThreads>(amax, red);
        const float inv = kQb / sc;                   // one IEEE division per token
        if (threadIdx.x == 0) sxl[m] = sc;
        if (regs) {
#pragma unroll
            for (int v = 0; v < kFusedRegVecs; ++v) {
                const int idx = v * kThreads + (int)threadIdx.x;
                if (idx < nvec) {
                    if (kPre == kPreNone) {
                        vec_quantize_store<kBf16>(row0[v], inv, out, idx);
                    } else if (kSwiglu) {
                        store_floats(hk[kSwiglu ? v : 0], idx, inv);
                    } else {
                        float f[kE];
                        values(row0[v], up0[v], idx, v, f);
                        store_floats(f, idx, inv);
                    }
                }
            }
        } else {
            for (int v = threadIdx.x; v < nvec; v += kThreads) {
                if (kPre == kPreNone) {
                    vec_quantize_store<kBf16>(row[v], inv, out, v);
                } else {
                    float f[kE];
                    values(row[v], row[kSwiglu ? nvec + v : v], v, -1, f);
                    store_floats(f, v, inv);
                }
            }
        }
        for (int v = nvec + threadIdx.x; v < nvec_pad; v += kThreads)                          // zero padding
            vec_quantize_store<kBf16>(make_uint4(0, 0, 0, 0), inv, out, v);
        __syncthreads();                              // red[] is reused by the next token; LDS rows complete
    }
}

// The same quantization with one wave per token, for several tokens of short rows (at most kWaveTokenVecs 16-byte vectors
// per lane: 4096 bf16 or 2048 fp32 elements): wave w takes tokens w, w + waves, ...; a token's absmax is a reduction
// inside the wave, so the tokens of different waves proceed side by side and the workgroup meets once at the end --
// where the block-wide form above pays two barriers and a trip to the L2 per token, one token after the other (1536
// columns, 16 tokens: 15.7 -> 6.9 us per launch).  Same arithmetic, same bits; the absmax is order-free.
constexpr int kWaveTokenVecs = 8;
template <bool kBf16, int kThreads>
__device__ inline void fused_quantize_wave_per_token(const void* __restrict__ xv, int M, int64_t K, int Kpad, float* sxl, uint4* xlds) {
    constexpr int kE = kBf16 ? 8 : 4;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int nvec = (int)(K / kE), nvec_pad = Kpad / kE;
    for (int m = wave; m < M; m += kThreads / kWave) {
        const uint4* row = reinterpret_cast<const uint4*>(static_cast<const char*>(xv) + (int64_t)m * K * (kBf16 ? 2 : 4));
        uint32_t* out = reinterpret_cast<uint32_t*>(xlds) + (size_t)m * (Kpad >> 2);
        uint4 q[kWaveTokenVecs];
        float amax = 0.0f;
#pragma unroll
        for (int v = 0; v < kWaveTokenVecs; ++v) {
            q[v] = row[min(v * kWave + lane, nvec - 1)];            // clamped duplicates do not change a maximum
            amax = vec_absmax<kBf16>(q[v], amax);
        }
        const float sc = fmaxf(wave_max_nonneg(amax), kEps);
        const float inv = kQb / sc;                                 // one IEEE division per token
        if (lane == 0) sxl[m] = sc;
#pragma unroll
        for (int v = 0; v < kWaveTokenVecs; ++v) {
            const int idx = v * kWave + lane;
            if (idx < nvec) vec_quantize_store<kBf16>(q[v], inv, out, idx);
        }
        for (int v = nvec + lane; v < nvec_pad; v += kWave) vec_quantize_store<kBf16>(make_uint4(0, 0, 0, 0), inv, out, v);
    }
    __syncthreads();
}

// kR    row blocks (16 rows each) per wave
// kS    waves that split K: wave ws takes steps ws, ws + kS, ...
// kW    row slots per workgroup (waves with different row blocks), workgroup = kS * kW waves
// kD    register prefetch depth in steps
// kX    XMode
// kPair the matrix is a merged gate | up projection of 2 * pair_off row blocks: a wave owns row block b of the gate half
//       and row block b of the up half (kR = 2) and the epilogue stores h = silu(y_gate) * y_up, [M][N] with
//       N = 16 * pair_off -- the SwiGLU of the feed-forward block applied where its two operands meet
template <int kR, int kS, int kW, int kD, int kX, bool kPair = false>
__global__ __launch_bounds__(kS * kW * kWave) void linear_gemv16_2bit(
        const void* __restrict__ xin /* x_q, or x for the fused modes */, const float* __restrict__ sx,
        const uint4* __restrict__ packed, const float* __restrict__ gamma, int gstride /* 0: one gamma, 1: one per row block */,
        int M, int64_t N, int64_t K, int Kq, int RB,
        int items /* K steps per wave, rounded up to a multiple of kD */, void* __restrict__ y, OutType yt,
        const float* __restrict__ gain /* RMSNorm modes: per-column gain or null */, float eps, int pair_off = 0) {
    static_assert(!kPair || kR == 2, "a gate row block and an up row block per wave");
    extern __shared__ uint4 smem[];
    constexpr int kThreads = kS * kW * kWave;
    constexpr bool kFromLds = kX != kXGlobal;
    constexpr bool kFused = kX >= kXFusedBf16;
    constexpr bool kNorm = kX == kXNormBf16 || kX == kXNormF32;
    constexpr bool kSwiglu = kX == kXSwigluBf16 || kX == kXSwigluF32;
    constexpr int kPre = kNorm ? kPreRmsNorm : kSwiglu ? kPreSwiglu : kPreNone;
    constexpr bool kInBf16 = kX == kXFusedBf16 || kX == kXNormBf16 || kX == kXSwigluBf16;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int r = lane & 15;
    const int g = lane >> 4;
    const int ws = wave % kS;
    const int ww = wave / kS;
    const int steps = (Kq + 3) >> 2;                   // K steps of 256 columns, the last may be partial
    const int tail_quads = 16 * (Kq - 4 * (steps - 1));   // quads in the last step's chunk (64 if whole)
    const int rbw = kPair ? (int)(blockIdx.x * kW + ww) : (int)(blockIdx.x * kW + ww) * kR;
    const int Kpad = steps * 256;
    const int8_t* xq = static_cast<const int8_t*>(xin);

    float* red = reinterpret_cast<float*>(smem);       // [16] reduction scratch (fused modes)
    float* sxl = red + 16;                             // [16] s_x of the fused modes; doubles for the RMSNorm sum follow
    uint4* xlds = smem + kGemvLdsHeader;               // x_q rows, Kpad bytes each; later the fold buffer

    const int64_t wstride = (int64_t)RB * 64;          // quads per whole step
    int rbc[kR];
#pragma unroll
    for (int a = 0; a < kR; ++a)                                   // row blocks past the matrix: clamped, never stored
        rbc[a] = kPair ? min(rbw, pair_off - 1) + a * pair_off : min(rbw + a, RB - 1);
    const int mrow = min(r, M - 1);
    const int8_t* xg = xq + (int64_t)mrow * K;
    const uint4* xl = xlds + mrow * (Kpad >> 4) + 4 * g;

    v4i acc[kR];
#pragma unroll
    for (int a = 0; a < kR; ++a) acc[a] = (v4i){0, 0, 0, 0};

    // One K step of operands.  Steps past the end are redirected to the last step and masked in mac();
    // in the last step only the first tail_quads lanes hold a quad, the others are clamped and masked.
    struct Stage { uint4 w[kR]; uint4 x[4]; };
    auto load = [&](Stage& s, int item) {
        const int sl = min(ws + item * kS, steps - 1);
        const int cq = sl == steps - 1 ? tail_quads : 64;
        const int ln = min(lane, cq - 1);
#pragma unroll
        for (int a = 0; a < kR; ++a) s.w[a] = load_streaming_b128(packed + ((int64_t)sl * wstride + (int64_t)rbc[a] * cq + ln));
        if (!kFromLds) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t col = min((int64_t)sl * 256 + 64 * g + 16 * j, K - 16);   // past-the-end columns meet zero codes
                s.x[j] = *reinterpret_cast<const uint4*>(xg + col);
            }
        }
    };
    auto mac = [&](Stage& s, int item) {
        const int step = ws + item * kS;
        const int sl = min(step, steps - 1);
        const int cq = sl == steps - 1 ? tail_quads : 64;
        const uint32_t km = (step < steps && lane < cq) ? 0xC0C0C0C0u : 0u;   // validity folded into the decode constant
        if (kFromLds) {
#pragma unroll
            for (int j = 0; j < 4; ++j) s.x[j] = xl[sl * 16 + j];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int a = 0; a < kR; ++a)
                acc[a] = __builtin_amdgcn_mfma_i32_16x16x64_i8(decode_word_masked(quad_word(s.w[a], j), km), as_v4i(s.x[j]),
                                                               acc[a], 0, 0, 0);
    };

    // fused modes: token 0 goes to registers first (cache hits, back long before the weights)
    uint4 row0[kFusedRegVecs], up0[kFusedRegVecs];
    float4 gain0[2][kInBf16 ? 2 : 1];
    bool row0_in_regs = false;
    if (kFused) {
        const int nvec = (int)(K / (kInBf16 ? 8 : 4));
        row0_in_regs = nvec <= kFusedRegVecs * kThreads;
        if (row0_in_regs) {
#pragma unroll
            for (int v = 0; v < kFusedRegVecs; ++v)
                row0[v] = static_cast<const uint4*>(xin)[min(v * kThreads + (int)threadIdx.x, nvec - 1)];
            if (kSwiglu) {                             // the up half of the row follows the K gate elements
#pragma unroll
                for (int v = 0; v < kFusedRegVecs; ++v)
                    up0[v] = static_cast<const uint4*>(xin)[nvec + min(v * kThreads + (int)threadIdx.x, nvec - 1)];
            }
            if (kNorm && gain) {                       // the gain of the same columns, needed after the reduction
#pragma unroll
                for (int v = 0; v < gain_reg_vecs(kThreads); ++v)
#pragma unroll
                    for (int h = 0; h < (kInBf16 ? 2 : 1); ++h)
                        gain0[v][h] = reinterpret_cast<const float4*>(gain)[(size_t)min(v * kThreads + (int)threadIdx.x, nvec - 1) * (kInBf16 ? 2 : 1) + h];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }

    // the output scales are requested first: loaded where they are used, after the fold, each would add a
    // cache round trip to the tail of a kernel that lives for only a few of them
    float gm[kR] = {};
    float sc_row = 0.0f;
    if (ws == 0) {                                     // the waves that write the output
#pragma unroll
        for (int a = 0; a < kR; ++a) gm[a] = gamma[gstride * rbc[a]];
        if (!kFused && yt != OutType::I32) sc_row = sx[mrow];
    }

    // then the weights: their loads stay in flight while the activations are staged
    Stage st[kD];
#pragma unroll
    for (int d = 0; d < kD; ++d) load(st[d], d);
    __builtin_amdgcn_sched_barrier(0);

    if (kX == kXLds) {
        const int nvec = M * (Kpad >> 4);
        for (int v = threadIdx.x; v < nvec; v += kThreads) {
            const int m = v / (Kpad >> 4), kv = v % (Kpad >> 4);
            uint4 val = make_uint4(0, 0, 0, 0);
            if ((int64_t)kv * 16 + 16 <= K) val = reinterpret_cast<const uint4*>(xq + (int64_t)m * K)[kv];
            xlds[v] = val;
        }
        __syncthreads();
    } else if (kFused) {
        if (kPre == kPreNone && M >= 3 && K <= (int64_t)kWaveTokenVecs * kWave * (kInBf16 ? 8 : 4))
            fused_quantize_wave_per_token<kInBf16, kThreads>(xin, M, K, Kpad, sxl, xlds);
        else
            fused_quantize_to_lds<kInBf16, kPre, kThreads>(xin, row0, up0, row0_in_regs, gain0, M, K, Kpad, gain, eps, red, sxl, xlds);
    }

    int i = 0;
    for (; i + kD < items; i += kD) {
#pragma unroll
        for (int d = 0; d < kD; ++d) {
            // the fences keep the refill of a stage right behind its use, kD steps ahead of need
            mac(st[d], i + d);
            __builtin_amdgcn_sched_barrier(0);
            load(st[d], i + d + kD);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int d = 0; d < kD; ++d) mac(st[d], i + d);

    if (kFused && yt != OutType::I32) sc_row = sxl[mrow];

    if (kS > 1) {
        // fold the K slices; the buffer aliases the x region, so wait until every wave is done with it
        v4i* fold = reinterpret_cast<v4i*>(xlds);
        __syncthreads();
#pragma unroll
        for (int a = 0; a < kR; ++a) fold[((ww * kS + ws) * kR + a) * kWave + lane] = acc[a];
        __syncthreads();
        if (ws != 0) return;
#pragma unroll
        for (int a = 0; a < kR; ++a) {
            v4i s = acc[a];
#pragma unroll
            for (int w = 1; w < kS; ++w) {
                const v4i o = fold[((ww * kS + w) * kR + a) * kWave + lane];
                s.x += o.x; s.y += o.y; s.z += o.z; s.w += o.w;
            }
            acc[a] = s;
        }
    }

    if (kPair) {
        // y_gate and y_up exactly as the plain epilogue would store them in fp32, then the gate
        if (r < M) {
            const float s0 = (gm[0] * sc_row) / kQb, s1 = (gm[kR - 1] * sc_row) / kQb;
            const int64_t n0 = (int64_t)rbw * 16 + 4 * g;
            const int vg[4] = {acc[0].x >> 6, acc[0].y >> 6, acc[0].z >> 6, acc[0].w >> 6};
            const int vu[4] = {acc[kR - 1].x >> 6, acc[kR - 1].y >> 6, acc[kR - 1].z >> 6, acc[kR - 1].w >> 6};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (n0 + e >= N) continue;
                const float h = swiglu_one((float)vg[e] * s0, (float)vu[e] * s1);
                if (yt == OutType::F32) static_cast<float*>(y)[(int64_t)r * N + n0 + e] = h;
                else static_cast<uint16_t*>(y)[(int64_t)r * N + n0 + e] = f32_to_bf16(h);
            }
        }
        return;
    }
    if (r < M) {                                                    // MFMA output column = lane & 15 = token
#pragma unroll
        for (int a = 0; a < kR; ++a) {
            const float scale = (gm[a] * sc_row) / kQb;
            const int64_t n0 = (int64_t)(rbw + a) * 16 + 4 * g;     // rows 4 g .. 4 g + 3 of the row block
            if (n0 < N) store_row4(y, yt, (int64_t)r * N + n0, n0, N, acc[a], scale);
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------------
constexpr size_t kGemvLdsBudget = 65536;

static size_t gemv16_x_lds_bytes(int64_t M, int64_t K) { return (size_t)M * ceil_div(K, 256) * 256; }

// kModes: which activation modes a launch shape is instantiated for (each is a kernel of its own)
constexpr int kModesInt8 = 1;    // kXGlobal, kXLds
constexpr int kModesFused = 2;   // kXFusedBf16, kXFusedF32
constexpr int kModesPre = 4;     // RMSNorm and SwiGLU pre-operations

template <int kR, int kS, int kW, int kD, int kModes>
static hipError_t launch16(int xmode, const void* x, const float* sx, const void* packed, const float* gamma, int gstride,
                     int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream, const float* gain, float eps,
                     LaunchPlan* plan = nullptr) {
    const int Kq = (int)ceil_div(K, kColsPerQuad);
    const int RB = (int)ceil_div(N, kRowsPerBlock);
    int items = (int)ceil_div(ceil_div(K, 256), kS);
    items = (int)ceil_div(items, kD) * kD;
    const size_t header = kGemvLdsHeader * sizeof(uint4);
    const size_t lds_fold = kS > 1 ? (size_t)kW * kS * kR * kWave * 16 : 0;
    const size_t lds_x = gemv16_x_lds_bytes(M, K);
    if (xmode == kXLds && header + lds_x > kGemvLdsBudget) xmode = kXGlobal;
    const size_t lds = header + (xmode != kXGlobal && lds_x > lds_fold ? lds_x : lds_fold);
    dim3 grid((unsigned)ceil_div(RB, kW * kR)), block(kS * kW * kWave);
    const int need = xmode <= kXLds ? kModesInt8 : xmode <= kXFusedF32 ? kModesFused : kModesPre;
    if ((kModes & need) == 0) return hipErrorInvalidDeviceFunction;   // a dispatch rule asked a launch shape for a mode it is not built for
    if (plan) {
        plan->set("decode", {kR, kS, kW, kD, xmode}, grid.x, 1, block.x, lds, 1);
        return hipSuccess;
    }
    const uint4* p = static_cast<const uint4*>(packed);
#define GO(X_) hipLaunchKernelGGL((linear_gemv16_2bit<kR, kS, kW, kD, X_>), grid, block, lds, stream, x, sx, p, gamma, gstride, (int)M, N, \
                                  K, Kq, RB, items, y, yt, gain, eps)
    if constexpr ((kModes & kModesInt8) != 0) {
        if (xmode == kXGlobal) { GO(kXGlobal); return hipGetLastError(); }
        if (xmode == kXLds) { GO(kXLds); return hipGetLastError(); }
    }
    if constexpr ((kModes & kModesFused) != 0) {
        if (xmode == kXFusedBf16) { GO(kXFusedBf16); return hipGetLastError(); }
        if (xmode == kXFusedF32) { GO(kXFusedF32); return hipGetLastError(); }
    }
    if constexpr ((kModes & kModesPre) != 0) {
        if (xmode == kXNormBf16) { GO(kXNormBf16); return hipGetLastError(); }
        if (xmode == kXNormF32) { GO(kXNormF32); return hipGetLastError(); }
        if (xmode == kXSwigluBf16) { GO(kXSwigluBf16); return hipGetLastError(); }
        if (xmode == kXSwigluF32) { GO(kXSwigluF32); return hipGetLastError(); }
    }
#undef GO
    return hipErrorInvalidDeviceFunction;
}

// Fraction of the K steps a shape walks that are real: each of kS waves takes ceil(steps / kS) steps, padded to a
// multiple of the prefetch depth kD with masked steps that still cost their loads and MFMAs.
static double walk_efficiency(int64_t steps, int kS, int kD) {
    const int64_t items = ceil_div(ceil_div(steps, kS), kD) * kD;
    return (double)steps / (double)(kS * items);
}

// Launch shapes from sweeps on MI355X (M = 1, 2 and 4; HIP-graph replay over many distinct weight buffers; twenty
// configurations on the twenty projection shapes of the 3B ... 70B LLaMA family).  What decides:
//   * many row blocks: few waves, each owning four row blocks for all of K with 2-3 steps of loads in flight --
//     the dense step-major front does the rest;
//   * fewer row blocks: K split over the 4-8 waves of a workgroup, one or two row blocks per wave, with a depth
//     such that S * D covers all steps where possible, i.e. the whole matrix is requested within the first memory
//     round trip; at most 256 row blocks: one row block per workgroup, or half the CUs get none;
//   * padding: 20 steps over 4 waves at depth 4 walk 32 (13B-class K = 5120 ran 1.3-1.4x slower than its bytes
//     warrant until the rules looked at it), so shapes are compared by walk_efficiency();
//   * x_q staged in LDS pays only for one token, many row blocks and a short K.
// The fused modes quantize the activations in every workgroup, so they lean towards fewer, wider workgroups; the
// RMSNorm and SwiGLU modes repeat an fp64 reduction or an exponential and a division per element on top (a
// microsecond or two of the CU's time) and go further that way.
#define GEMV16(R_, S_, W_, D_, MODES_, X_) \
    return launch16<R_, S_, W_, D_, MODES_>(X_, x, sx, packed, gamma, gstride, M, N, K, y, yt, stream, gain, eps, plan)

static hipError_t dispatch16_int8(const void* x, const float* sx, const void* packed, const float* gamma, int gstride, int64_t M,
                                  int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream, LaunchPlan* plan) {
    const int64_t RB = ceil_div(N, kRowsPerBlock), steps = ceil_div(K, 256);
    const float* gain = nullptr;
    const float eps = 0.0f;
    const bool pads44 = walk_efficiency(steps, 4, 4) < 0.75;       // four waves at depth 4 would walk over a third more than K
    if (RB >= 2048) {
        // one or two tokens: x_q from LDS, two waves splitting K per row block (30B gate/up 16.1 -> 14.6 us, 70B
        // gate/up 23.0 -> 21.3 us at M = 1 once the weight loads were marked streaming); more tokens: wide waves
        if (M <= 2) GEMV16(1, 2, 2, 4, kModesInt8, kXLds);
        else if (steps >= 32) GEMV16(4, 1, 4, 2, kModesInt8 | kModesFused | kModesPre, kXGlobal);
        else GEMV16(4, 1, 4, 3, kModesInt8, kXGlobal);
    } else if (RB >= 1024) {
        if (steps < 16 && M == 1 && !pads44) GEMV16(1, 4, 1, 4, kModesInt8 | kModesFused | kModesPre, kXLds);
        else if (steps < 16 && M == 1) GEMV16(2, 2, 2, 4, kModesInt8 | kModesPre, kXGlobal);      // e.g. 8 steps: 2 x 4, no padding
        else if (!pads44 && M == 1) GEMV16(1, 2, 2, 4, kModesInt8, kXLds);      // 7B gate/up 6.9 -> 6.6 us, 30B QKV 10.5 -> 9.6 us
        else if (!pads44) GEMV16(2, 4, 1, 4, kModesInt8, kXGlobal);
        else if (M == 1) {
            // a K walk that four waves cannot split evenly: no split, eight single-row-block waves, x_q in LDS
            // (13B gate/up, 20 steps: 9.0 -> 8.2 us)
            if (walk_efficiency(steps, 1, 5) >= walk_efficiency(steps, 1, 4)) GEMV16(1, 1, 8, 5, kModesInt8, kXLds);
            else GEMV16(1, 1, 8, 4, kModesInt8, kXLds);
        } else GEMV16(2, 1, 4, 4, kModesInt8 | kModesFused, kXGlobal);
    } else if (RB <= 256) {
        if (walk_efficiency(steps, 4, 5) > walk_efficiency(steps, 4, 4)) GEMV16(1, 4, 1, 5, kModesInt8 | kModesFused, kXGlobal);
        else GEMV16(1, 4, 1, 4, kModesInt8 | kModesFused | kModesPre, kXGlobal);
    } else if (steps >= 24) {
        GEMV16(2, 4, 1, 4, kModesInt8, kXGlobal);
    } else if (!pads44) {
        if (M > 1 && RB >= 512) GEMV16(2, 2, 2, 4, kModesInt8 | kModesPre, kXGlobal);     // 7B QKV at 2 / 4 / 8 tokens: 5.1 / 5.2 / 5.5 us (four K-split waves: 5.25 / 5.3 / 6.05)
        else GEMV16(1, 4, 1, 4, kModesInt8 | kModesFused | kModesPre, (RB >= 400 && steps < 16) ? kXLds : kXGlobal);
    } else if (RB < 512) {
        if (walk_efficiency(steps, 4, 5) > walk_efficiency(steps, 4, 4)) GEMV16(1, 4, 1, 5, kModesInt8 | kModesFused, kXGlobal);
        else GEMV16(1, 4, 1, 4, kModesInt8 | kModesFused | kModesPre, kXGlobal);
    } else {
        GEMV16(2, 2, 2, 4, kModesInt8 | kModesPre, kXGlobal);
    }
}

// x is quantized in the kernel (xmode: plain, after RMSNorm, after SwiGLU); sx is unused
static hipError_t dispatch16_fused(int xmode, const void* x, const void* packed, const float* gamma, int gstride, int64_t M,
                             int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream, const float* gain, float eps,
                             LaunchPlan* plan) {
    const int64_t RB = ceil_div(N, kRowsPerBlock), steps = ceil_div(K, 256);
    const float* sx = nullptr;
    if (xmode == kXNormBf16 || xmode == kXNormF32) {
        // every workgroup repeats the normalisation (an fp64 reduction and a square root, a microsecond or two of its
        // CU's time), so few, wide workgroups: one wave per row block (or pair of them) and no K split from 769 row
        // blocks on, at most 256 workgroups up to 4096 row blocks
        if (RB >= 2048) GEMV16(2, 1, 8, 3, kModesFused | kModesPre, xmode);
        else if (RB >= 1024) GEMV16(1, 1, 8, 5, kModesFused | kModesPre, xmode);
        else if (RB > 768) GEMV16(1, 1, 4, 5, kModesPre, xmode);
        else if (RB > 512) GEMV16(2, 2, 2, 4, kModesInt8 | kModesPre, xmode);
        else if (RB > 256) GEMV16(1, 2, 2, 4, kModesFused | kModesPre, xmode);
        else GEMV16(1, 4, 1, 4, kModesInt8 | kModesFused | kModesPre, xmode);
    }
    if (xmode >= kXSwigluBf16) {
        // the gate (an exponential and a division per element) is repeated by every workgroup for the whole token
        if (RB >= 2048) GEMV16(4, 1, 4, 2, kModesInt8 | kModesFused | kModesPre, xmode);
        else if (steps >= 64) GEMV16(1, 8, 1, 3, kModesFused | kModesPre, xmode);   // 1024 threads leave this mode too few registers
        else if (steps >= 24) { if (steps <= 40) GEMV16(1, 8, 1, 5, kModesFused | kModesPre, xmode); else GEMV16(1, 8, 1, 3, kModesFused | kModesPre, xmode); }
        else if (RB > 640) GEMV16(1, 1, 4, 5, kModesPre, xmode);
        else if (RB > 320) GEMV16(1, 2, 2, 4, kModesFused | kModesPre, xmode);
        else GEMV16(1, 4, 1, 4, kModesInt8 | kModesFused | kModesPre, xmode);
    }
    // Eight tokens and more: every workgroup quantizes all of them before its first product, so the forms that give a
    // workgroup more row blocks (fewer workgroups repeating that work, eight waves sharing it) win by 10-25 %:
    // 16 tokens on 3200 -> 17280 13.3 -> 10.4 us, on 3200 -> 9600 11.5 -> 8.6 us, on 3200 -> 3200 7.6 -> 6.8 us; 8 tokens
    // on 4096 -> 22016 10.8 -> 9.5 us, on 4096 -> 12288 9.0 -> 7.5 us; 12 tokens on 5120 -> 15360 22.3 -> 18.8 us, on
    // 5120 -> 5120 19.1 -> 15.7 us (at four tokens the forms below are within 3 % of the best).
    if (M >= 8) {
        if (RB >= 1024) GEMV16(4, 4, 2, 2, kModesFused, xmode);
        else if (RB > 384) GEMV16(2, 4, 2, 4, kModesFused, xmode);
        else GEMV16(1, 8, 1, 3, kModesFused | kModesPre, xmode);
    }
    // Many row blocks: eight waves per workgroup, each walking all of K for one or two row blocks of its own -- few
    // workgroups repeat the quantization, no partial sums to fold, and about eight waves per CU with several loads
    // each in flight is the shape in which a plain read loop is fastest on this chip (70B gate/up 22.9 -> 20.8 us,
    // 30B gate/up 15.3 -> 14.4 us, 13B gate/up 8.9 -> 8.0 us, 7B gate/up 7.0 -> 6.8 us, 3B gate/up 6.7 -> 6.45 us).
    if (RB >= 2048) {
        if (steps >= 32) GEMV16(2, 1, 8, 2, kModesFused, xmode);
        else GEMV16(2, 1, 8, 3, kModesFused | kModesPre, xmode);
    } else if (RB >= 1024) {
        if (steps <= 24) {
            if (walk_efficiency(steps, 1, 5) >= walk_efficiency(steps, 1, 4)) GEMV16(1, 1, 8, 5, kModesFused | kModesPre, xmode);
            else GEMV16(1, 1, 8, 4, kModesFused, xmode);
        } else if (RB >= 1536 && walk_efficiency(steps, 2, 4) < 0.9 && walk_efficiency(steps, 1, 4) > walk_efficiency(steps, 2, 4))
            GEMV16(2, 1, 4, 4, kModesInt8 | kModesFused, xmode);
        else GEMV16(1, 2, 2, 4, kModesFused | kModesPre, xmode);
    } else if (steps >= 64) {
        if (steps >= 96) GEMV16(1, 8, 2, 2, kModesFused, xmode); else GEMV16(1, 8, 2, 3, kModesFused, xmode);
    } else if (steps >= 24) {
        if (RB > 256) GEMV16(1, 4, 2, 4, kModesFused, xmode);
        else if (steps <= 40) GEMV16(1, 8, 1, 5, kModesFused | kModesPre, xmode);
        else GEMV16(1, 8, 1, 3, kModesFused | kModesPre, xmode);
    } else if (walk_efficiency(steps, 4, 4) >= 0.8) {
        GEMV16(1, 4, 1, 4, kModesInt8 | kModesFused | kModesPre, xmode);
    } else if (RB < 512) {
        GEMV16(1, 4, 1, 5, kModesInt8 | kModesFused, xmode);
    } else {
        GEMV16(1, 2, 2, 4, kModesFused | kModesPre, xmode);
    }
}
#undef GEMV16

// the product on pre-quantized activations, M <= 16 (the dispatcher of the M <= 64 kernels uses it up to M = 4)
hipError_t launch_linear_gemv16_2bit(const int8_t* xq, const float* sx, const void* packed, const float* gamma, int gstride,
                                     int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream,
                                     LaunchPlan* plan) {
    return dispatch16_int8(xq, sx, packed, gamma, gstride, M, N, K, y, yt, stream, plan);
}

bool gemv_fused_supports(int64_t M, int64_t N, int64_t K, const void* x) {
    (void)N;
    return M >= 1 && M <= 16 && K % 16 == 0 && reinterpret_cast<uintptr_t>(x) % 16 == 0 &&
           kGemvLdsHeader * sizeof(uint4) + gemv16_x_lds_bytes(M, K) <= kGemvLdsBudget;
}

hipError_t launch_linear_fused_2bit(const void* x, bool bf16, const void* packed, const float* gamma, int gstride,
                                    int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream, LaunchPlan* plan) {
    return dispatch16_fused(bf16 ? kXFusedBf16 : kXFusedF32, x, packed, gamma, gstride, M, N, K, y, yt, stream, nullptr, 0.0f, plan);
}

hipError_t launch_rmsnorm_linear_fused_2bit(const void* x, bool bf16, const float* gain, float eps, const void* packed,
                                            const float* gamma, int gstride, int64_t M, int64_t N, int64_t K, void* y,
                                            OutType yt, hipStream_t stream, LaunchPlan* plan) {
    return dispatch16_fused(bf16 ? kXNormBf16 : kXNormF32, x, packed, gamma, gstride, M, N, K, y, yt, stream, gain, eps, plan);
}

// merged gate | up projection with the SwiGLU gate in the epilogue; x goes through the fused quantization
// (xmode: absmax only, or RMSNorm first).  F is a multiple of 16, so the up half starts on a row block.
template <int kS, int kW, int kD>
static void launch16_pair(int xmode, const void* x, const void* packed, const float* gamma, int gstride, int64_t M,
                          int64_t F, int64_t K, void* h, OutType yt, hipStream_t stream, const float* gain, float eps,
                          LaunchPlan* plan) {
    constexpr int kR = 2;
    const int Kq = (int)ceil_div(K, kColsPerQuad);
    const int pair_off = (int)(F / kRowsPerBlock);
    const int RB = 2 * pair_off;
    int items = (int)ceil_div(ceil_div(K, 256), kS);
    items = (int)ceil_div(items, kD) * kD;
    const size_t header = kGemvLdsHeader * sizeof(uint4);
    const size_t lds_fold = kS > 1 ? (size_t)kW * kS * kR * kWave * 16 : 0;
    const size_t lds_x = gemv16_x_lds_bytes(M, K);
    const size_t lds = header + (lds_x > lds_fold ? lds_x : lds_fold);
    dim3 grid((unsigned)ceil_div(pair_off, kW)), block(kS * kW * kWave);
    if (plan) {
        plan->set("decode_pair", {kR, kS, kW, kD, xmode}, grid.x, 1, block.x, lds, 1);
        return;
    }
    const uint4* p = static_cast<const uint4*>(packed);
#define GO(X_) hipLaunchKernelGGL((linear_gemv16_2bit<kR, kS, kW, kD, X_, true>), grid, block, lds, stream, x, (const float*)nullptr, p, gamma, \
                                  gstride, (int)M, F, K, Kq, RB, items, h, yt, gain, eps, pair_off)
    switch (xmode) {
        case kXFusedBf16: GO(kXFusedBf16); break;
        case kXFusedF32: GO(kXFusedF32); break;
        case kXNormBf16: GO(kXNormBf16); break;
        default: GO(kXNormF32); break;
    }
#undef GO
}

hipError_t launch_linear_fused_swiglu_out_2bit(const void* x, bool bf16, bool norm, const float* gain, float eps,
                                               const void* packed, const float* gamma, int gstride, int64_t M, int64_t F,
                                               int64_t K, void* h, OutType yt, hipStream_t stream, LaunchPlan* plan) {
    const int xmode = norm ? (bf16 ? kXNormBf16 : kXNormF32) : (bf16 ? kXFusedBf16 : kXFusedF32);
    // From a sweep of fourteen launch shapes on the gate / up matrices of the 3B ... 70B family: without the
    // normalisation, up to 700 pairs one pair per workgroup with K split over four waves; otherwise one wave per pair
    // and no K split, four pairs per workgroup up to 1024 pairs (at most 256 workgroups), eight beyond.
    const int64_t pairs = F / kRowsPerBlock;
    if (!norm && pairs <= 700) launch16_pair<4, 1, 4>(xmode, x, packed, gamma, gstride, M, F, K, h, yt, stream, gain, eps, plan);
    else if (pairs <= 1024) {
        // depth 5 or 4, whichever pads the K walk less (16 steps at depth 5 walk 20: 7B gate/up with the norm 10.5 -> 9.5 us)
        const int64_t steps = ceil_div(K, 256);
        if (walk_efficiency(steps, 1, 5) >= walk_efficiency(steps, 1, 4))
            launch16_pair<1, 4, 5>(xmode, x, packed, gamma, gstride, M, F, K, h, yt, stream, gain, eps, plan);
        else
            launch16_pair<1, 4, 4>(xmode, x, packed, gamma, gstride, M, F, K, h, yt, stream, gain, eps, plan);
    } else launch16_pair<1, 8, 3>(xmode, x, packed, gamma, gstride, M, F, K, h, yt, stream, gain, eps, plan);
    return plan ? hipSuccess : hipGetLastError();
}

hipError_t launch_swiglu_linear_fused_2bit(const void* gu, bool bf16, const void* packed, const float* gamma, int gstride,
                                           int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream,
                                           LaunchPlan* plan) {
    return dispatch16_fused(bf16 ? kXSwigluBf16 : kXSwigluF32, gu, packed, gamma, gstride, M, N, K, y, yt, stream, nullptr, 0.0f, plan);
}

}  // namespace bitnet

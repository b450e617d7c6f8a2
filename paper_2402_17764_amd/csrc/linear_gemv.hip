// Weight-streaming BitLinear kernels for decode and batched decode (M <= 64) on gfx950.
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

__device__ inline uint32_t quad_word(const uint4& q, int j) { return j == 0 ? q.x : j == 1 ? q.y : j == 2 ? q.z : q.w; }

__device__ inline void store_row4(void* y, OutType yt, int64_t base, int64_t n0, int64_t N, const v4i& s, float scale) {
    const int v[4] = {s.x >> 6, s.y >> 6, s.z >> 6, s.w >> 6};   // drop the decode factor 64 (exact)
    if (yt == OutType::I32) {
        int32_t* yo = static_cast<int32_t*>(y);
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (n0 + e < N) yo[base + e] = v[e];
    } else if (yt == OutType::F32) {
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

// ---------------------------------------------------------------------------------------------------
// M <= 16
// ---------------------------------------------------------------------------------------------------
// Where the activation operand comes from.
enum XMode : int {
    kXGlobal = 0,      // int8 x_q read from global memory with every step
    kXLds = 1,         // int8 x_q copied once per workgroup into LDS
    kXFusedBf16 = 2,   // bf16 x: per-token absmax quantization done in the kernel, x_q lives only in LDS
    kXFusedF32 = 3     // fp32 x, same
};

constexpr int kGemvLdsHeader = 8;       // uint4 slots in front of the x region: reduction scratch + s_x

// In-kernel activation quantization for the fused modes (Section 2 of the paper: per-token absmax,
// Q_b = 127), the same arithmetic as the stand-alone activation kernel: s = max(absmax, 1e-5),
// inv = 127 / s, x_q = clip(rint(x * inv)).  Rows land in LDS zero padded to Kpad columns, s_x[m] in
// sxl[m].  Token 0 is fetched into registers before the weight prefetch is issued (so that waiting for
// it does not wait for the weights) and quantized from there; further tokens take two sweeps.
constexpr int kFusedRegVecs = 4;          // 16-byte vectors of token 0 a thread can hold

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

__device__ inline uint32_t quant_byte(float v, float inv) {
    const float f = rintf(v * inv);                   // one fp32 multiply, ties to even
    return (uint32_t)(int)fminf(kQb, fmaxf(-kQb, f)) & 0xFFu;
}

// one 16-byte vector of x -> its int8 codes, written to the token's LDS row (32-bit words)
template <bool kBf16>
__device__ inline void vec_quantize_store(const uint4& q, float inv, uint32_t* out, int v) {
    const uint32_t u[4] = {q.x, q.y, q.z, q.w};
    if (kBf16) {
        uint32_t o[2] = {0, 0};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t lo = quant_byte(__uint_as_float(u[e] << 16), inv);
            const uint32_t hi = quant_byte(__uint_as_float(u[e] & 0xFFFF0000u), inv);
            o[e >> 1] |= (lo | (hi << 8)) << (16 * (e & 1));
        }
        out[2 * v] = o[0];
        out[2 * v + 1] = o[1];
    } else {
        uint32_t o = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) o |= quant_byte(__uint_as_float(u[e]), inv) << (8 * e);
        out[v] = o;
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

template <bool kBf16, int kThreads>
__device__ inline void fused_quantize_to_lds(const void* __restrict__ xv, const uint4 (&row0)[kFusedRegVecs], bool row0_in_regs,
                                             int M, int64_t K, int Kpad, float* red, float* sxl, uint4* xlds) {
    constexpr int kE = kBf16 ? 8 : 4;                 // elements per 16-byte vector
    const int nvec = (int)(K / kE);
    const int nvec_pad = Kpad / kE;
    for (int m = 0; m < M; ++m) {
        const uint4* row = reinterpret_cast<const uint4*>(static_cast<const char*>(xv) + (int64_t)m * K * (kBf16 ? 2 : 4));
        uint32_t* out = reinterpret_cast<uint32_t*>(xlds) + (size_t)m * (Kpad >> 2);
        const bool regs = m == 0 && row0_in_regs;
        float amax = 0.0f;
        if (regs) {
#pragma unroll
            for (int v = 0; v < kFusedRegVecs; ++v) amax = vec_absmax<kBf16>(row0[v], amax);   // clamped duplicates are harmless
        } else {
            for (int v = threadIdx.x; v < nvec; v += kThreads) amax = vec_absmax<kBf16>(row[v], amax);
        }
        const float sc = block_absmax_to_scale<kThreads>(amax, red);
        const float inv = kQb / sc;                   // one IEEE division per token
        if (threadIdx.x == 0) sxl[m] = sc;
        if (regs) {
#pragma unroll
            for (int v = 0; v < kFusedRegVecs; ++v) {
                const int idx = v * kThreads + (int)threadIdx.x;
                if (idx < nvec) vec_quantize_store<kBf16>(row0[v], inv, out, idx);
            }
        } else {
            for (int v = threadIdx.x; v < nvec; v += kThreads) vec_quantize_store<kBf16>(row[v], inv, out, v);
        }
        for (int v = nvec + threadIdx.x; v < nvec_pad; v += kThreads)                          // zero padding
            vec_quantize_store<kBf16>(make_uint4(0, 0, 0, 0), inv, out, v);
        __syncthreads();                              // red[] is reused by the next token; LDS rows complete
    }
}

// kR    row blocks (16 rows each) per wave
// kS    waves that split K: wave ws takes steps ws, ws + kS, ...
// kW    row slots per workgroup (waves with different row blocks), workgroup = kS * kW waves
// kD    register prefetch depth in steps
// kX    XMode
template <int kR, int kS, int kW, int kD, int kX>
__global__ __launch_bounds__(kS * kW * kWave) void linear_gemv16_2bit(
        const void* __restrict__ xin /* x_q, or x for the fused modes */, const float* __restrict__ sx,
        const uint4* __restrict__ packed, const float* __restrict__ gamma, int M, int64_t N, int64_t K, int Kq, int RB,
        int items /* K steps per wave, rounded up to a multiple of kD */, void* __restrict__ y, OutType yt) {
    extern __shared__ uint4 smem[];
    constexpr int kThreads = kS * kW * kWave;
    constexpr bool kFromLds = kX != kXGlobal;
    constexpr bool kFused = kX == kXFusedBf16 || kX == kXFusedF32;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int r = lane & 15;
    const int g = lane >> 4;
    const int ws = wave % kS;
    const int ww = wave / kS;
    const int steps = (Kq + 3) >> 2;                   // K steps of 256 columns, the last may be partial
    const int tail_quads = 16 * (Kq - 4 * (steps - 1));   // quads in the last step's chunk (64 if whole)
    const int rbw = (blockIdx.x * kW + ww) * kR;
    const int Kpad = steps * 256;
    const int8_t* xq = static_cast<const int8_t*>(xin);

    float* red = reinterpret_cast<float*>(smem);       // [16] reduction scratch (fused modes)
    float* sxl = red + 16;                             // [16] s_x of the fused modes
    uint4* xlds = smem + kGemvLdsHeader;               // x_q rows, Kpad bytes each; later the fold buffer

    const int64_t wstride = (int64_t)RB * 64;          // quads per whole step
    int rbc[kR];
#pragma unroll
    for (int a = 0; a < kR; ++a) rbc[a] = min(rbw + a, RB - 1);   // row blocks past the matrix: clamped, never stored
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
        for (int a = 0; a < kR; ++a) s.w[a] = packed[(int64_t)sl * wstride + (int64_t)rbc[a] * cq + ln];
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
        const uint32_t keep = (step < steps && lane < cq) ? 0xFFFFFFFFu : 0u;
        if (kFromLds) {
#pragma unroll
            for (int j = 0; j < 4; ++j) s.x[j] = xl[sl * 16 + j];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int a = 0; a < kR; ++a)
                acc[a] = __builtin_amdgcn_mfma_i32_16x16x64_i8(decode_word(quad_word(s.w[a], j) & keep), as_v4i(s.x[j]),
                                                               acc[a], 0, 0, 0);
    };

    // fused modes: token 0 goes to registers first (cache hits, back long before the weights)
    uint4 row0[kFusedRegVecs];
    bool row0_in_regs = false;
    if (kFused) {
        const int nvec = (int)(K / (kX == kXFusedBf16 ? 8 : 4));
        row0_in_regs = nvec <= kFusedRegVecs * kThreads;
        if (row0_in_regs) {
#pragma unroll
            for (int v = 0; v < kFusedRegVecs; ++v)
                row0[v] = static_cast<const uint4*>(xin)[min(v * kThreads + (int)threadIdx.x, nvec - 1)];
        }
        __builtin_amdgcn_sched_barrier(0);
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
        fused_quantize_to_lds<kX == kXFusedBf16, kThreads>(xin, row0, row0_in_regs, M, K, Kpad, red, sxl, xlds);
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

    float sc_row = 0.0f;
    if (yt != OutType::I32) sc_row = kFused ? sxl[mrow] : sx[mrow];

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

    if (r < M) {                                                    // MFMA output column = lane & 15 = token
        const float scale = (gamma[0] * sc_row) / kQb;
#pragma unroll
        for (int a = 0; a < kR; ++a) {
            const int64_t n0 = (int64_t)(rbw + a) * 16 + 4 * g;     // rows 4 g .. 4 g + 3 of the row block
            if (n0 < N) store_row4(y, yt, (int64_t)r * N + n0, n0, N, acc[a], scale);
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// 16 < M <= 64: same stream, kMT token tiles per wave, activations read from global memory
// ---------------------------------------------------------------------------------------------------
template <int kR, int kMT>
struct GemvStage {
    uint4 w[kR];          // one quad per row block
    uint4 x[kMT][4];      // 64 activation bytes per token tile
};

template <int kR, int kMT>
__device__ inline void gemv_mac(const GemvStage<kR, kMT>& st, v4i (&acc)[kR][kMT]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int a = 0; a < kR; ++a) {
            const v4i A = decode_word(quad_word(st.w[a], j));
#pragma unroll
            for (int t = 0; t < kMT; ++t)
                acc[a][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A, as_v4i(st.x[t][j]), acc[a][t], 0, 0, 0);
        }
    }
}

// kR row blocks per workgroup (every wave handles all of them), kMT token tiles of 16, kS waves split K
template <int kR, int kMT, int kS>
__global__ __launch_bounds__(kS * kWave) void linear_gemv64_2bit(const int8_t* __restrict__ xq, const float* __restrict__ sx,
                                                                  const uint4* __restrict__ packed,
                                                                  const float* __restrict__ gamma, int M, int64_t N, int64_t K,
                                                                  int Kq, int RB, void* __restrict__ y, OutType yt) {
    __shared__ v4i fold[kS][kR * kMT][kWave];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int r = lane & 15;
    const int g = lane >> 4;
    const int rb0 = blockIdx.x * kR;
    const int full_steps = (int)(K >> 8);            // steps whose 256 columns all exist

    v4i acc[kR][kMT];
#pragma unroll
    for (int a = 0; a < kR; ++a)
#pragma unroll
        for (int t = 0; t < kMT; ++t) acc[a][t] = (v4i){0, 0, 0, 0};

    // per-lane base pointers; row blocks and tokens beyond the matrix are clamped to the last valid one
    const int64_t wstride = (int64_t)RB * 64;
    const uint4* wp[kR];
#pragma unroll
    for (int a = 0; a < kR; ++a) wp[a] = packed + (int64_t)min(rb0 + a, RB - 1) * 64 + lane;
    const uint4* xp[kMT];
#pragma unroll
    for (int t = 0; t < kMT; ++t) {
        const int m = min(16 * t + r, M - 1);
        xp[t] = reinterpret_cast<const uint4*>(xq + (int64_t)m * K + 64 * g);   // + 16 uint4 per step
    }

    auto load = [&](GemvStage<kR, kMT>& st, int step) {
#pragma unroll
        for (int a = 0; a < kR; ++a) st.w[a] = wp[a][(int64_t)step * wstride];
#pragma unroll
        for (int t = 0; t < kMT; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) st.x[t][j] = xp[t][(int64_t)step * 16 + j];
    };

    // software pipeline over this wave's whole steps: wave, wave + kS, ...
    const int mine = full_steps > wave ? (full_steps - wave + kS - 1) / kS : 0;
    if (mine > 0) {
        GemvStage<kR, kMT> s0, s1;
        load(s0, wave);
        int i = 0;
        for (; i + 2 <= mine - 1; i += 2) {
            load(s1, wave + (i + 1) * kS);
            __builtin_amdgcn_sched_barrier(0);
            gemv_mac<kR, kMT>(s0, acc);
            __builtin_amdgcn_sched_barrier(0);
            load(s0, wave + (i + 2) * kS);
            __builtin_amdgcn_sched_barrier(0);
            gemv_mac<kR, kMT>(s1, acc);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (i + 1 <= mine - 1) {
            load(s1, wave + (i + 1) * kS);
            gemv_mac<kR, kMT>(s0, acc);
            gemv_mac<kR, kMT>(s1, acc);
        } else {
            gemv_mac<kR, kMT>(s0, acc);
        }
    }

    // columns past the last whole step (K % 256 != 0): one guarded step, taken by one wave
    if ((K & 255) != 0 && wave == full_steps % kS) {
        const int kq = 4 * full_steps + g;
        const int nq = Kq - 4 * full_steps;
        const int64_t kbase = (int64_t)kq * 64;
        const uint4 zero4 = make_uint4(0, 0, 0, 0);
        GemvStage<kR, kMT> st;
#pragma unroll
        for (int a = 0; a < kR; ++a) {
            st.w[a] = zero4;
            if (kq < Kq) st.w[a] = packed[(int64_t)full_steps * wstride + (int64_t)min(rb0 + a, RB - 1) * 16 * nq + lane];
        }
#pragma unroll
        for (int t = 0; t < kMT; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                st.x[t][j] = zero4;
                if (kbase + 16 * j + 16 <= K) st.x[t][j] = xp[t][(int64_t)full_steps * 16 + j];
            }
        gemv_mac<kR, kMT>(st, acc);
    }

    // fold the K slices of the kS waves
#pragma unroll
    for (int a = 0; a < kR; ++a)
#pragma unroll
        for (int t = 0; t < kMT; ++t) fold[wave][a * kMT + t][lane] = acc[a][t];
    __syncthreads();

    const float gm = gamma[0];
    for (int tile = wave; tile < kR * kMT; tile += kS) {
        v4i s = fold[0][tile][lane];
#pragma unroll
        for (int w = 1; w < kS; ++w) {
            const v4i o = fold[w][tile][lane];
            s.x += o.x; s.y += o.y; s.z += o.z; s.w += o.w;
        }
        const int a = tile / kMT, t = tile % kMT;
        const int m = 16 * t + r;
        const int64_t n0 = (int64_t)(rb0 + a) * 16 + 4 * g;
        if (m >= M || n0 >= N) continue;
        const float scale = yt == OutType::I32 ? 0.0f : (gm * sx[m]) / kQb;
        store_row4(y, yt, (int64_t)m * N + n0, n0, N, s, scale);
    }
}

// ---------------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------------
bool gemv_supports(int64_t M, int64_t N, int64_t K, const void* xq) {
    (void)N;
    return M >= 1 && M <= 64 && K % 16 == 0 && reinterpret_cast<uintptr_t>(xq) % 16 == 0;
}

constexpr size_t kGemvLdsBudget = 65536;

static size_t gemv16_x_lds_bytes(int64_t M, int64_t K) { return (size_t)M * ceil_div(K, 256) * 256; }

template <int kR, int kS, int kW, int kD>
static void launch16(int xmode, const void* x, const float* sx, const void* packed, const float* gamma, int64_t M,
                     int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream) {
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
    const uint4* p = static_cast<const uint4*>(packed);
#define GO(X_) hipLaunchKernelGGL((linear_gemv16_2bit<kR, kS, kW, kD, X_>), grid, block, lds, stream, x, sx, p, gamma, (int)M, N, \
                                  K, Kq, RB, items, y, yt)
    switch (xmode) {
        case kXGlobal: GO(kXGlobal); break;
        case kXLds: GO(kXLds); break;
        case kXFusedBf16: GO(kXFusedBf16); break;
        default: GO(kXFusedF32); break;
    }
#undef GO
}

template <int kR, int kMT, int kS>
static void launch64(const int8_t* xq, const float* sx, const void* packed, const float* gamma, int64_t M,
                     int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream) {
    const int Kq = (int)ceil_div(K, kColsPerQuad);
    const int RB = (int)ceil_div(N, kRowsPerBlock);
    dim3 grid((unsigned)ceil_div(RB, kR));
    hipLaunchKernelGGL((linear_gemv64_2bit<kR, kMT, kS>), grid, dim3(kS * kWave), 0, stream, xq, sx,
                       static_cast<const uint4*>(packed), gamma, (int)M, N, K, Kq, RB, y, yt);
}

// Shape heuristics from sweeps on MI355X (M = 1, HIP-graph replay over many distinct weight buffers):
//   * many row blocks: few waves, each owning four row blocks for all of K with 2-3 steps of loads
//     in flight -- the dense step-major front does the rest;
//   * fewer row blocks: one row block per wave and K split over 4-8 waves, with depth chosen so that
//     S * D covers all steps, i.e. the whole matrix is requested within the first memory round trip;
//   * long K with few row blocks: two row blocks per wave, K split four ways, four steps in flight.
// xmode < 0 (x_q given) lets the shape decide between global and LDS-staged x_q; the fused modes
// pass their own and need the wide workgroups that can hold token 0 in registers.
static void dispatch16(int xmode, const void* x, const float* sx, const void* packed, const float* gamma, int64_t M,
                       int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream) {
    const int64_t RB = ceil_div(N, kRowsPerBlock);
    const int64_t steps = ceil_div(K, 256);
    const bool fused = xmode >= 0;
    const bool fits_lds = kGemvLdsHeader * sizeof(uint4) + gemv16_x_lds_bytes(M, K) <= kGemvLdsBudget;
#define GEMV16(R_, S_, W_, D_, X_) launch16<R_, S_, W_, D_>(fused ? xmode : (X_), x, sx, packed, gamma, M, N, K, y, yt, stream)
    if (M > 4 && !fused) {
        // x traffic grows with M: stage x_q in LDS when it fits, else amortize it over four row blocks
        if (fits_lds && RB < 2048)  GEMV16(1, 4, 1, 4, kXLds);
        else if (RB >= 1024)        GEMV16(4, 1, 4, 2, kXGlobal);
        else                        GEMV16(4, 2, 2, 2, kXGlobal);
    } else if (RB >= 2048) {
        if (fused) GEMV16(4, 1, 4, 2, kXGlobal); else GEMV16(4, 1, 4, 3, kXGlobal);
    } else if (steps >= 64) {
        if (fused) GEMV16(1, 8, 2, 2, kXGlobal); else GEMV16(2, 4, 1, 4, kXGlobal);
    } else if (steps >= 24) {
        if (steps <= 40) GEMV16(1, 8, 1, 5, kXLds); else GEMV16(1, 8, 1, 3, kXLds);
    } else if (RB >= 1024 && steps >= 16 && !fused) {
        GEMV16(2, 4, 1, 4, kXGlobal);
    } else {
        GEMV16(1, 4, 1, 4, (RB >= 400 && steps < 16) ? kXLds : kXGlobal);
    }
#undef GEMV16
}

hipError_t launch_linear_gemv_2bit(const int8_t* xq, const float* sx, const void* packed,
                                   const float* gamma, int64_t M, int64_t N, int64_t K, void* y,
                                   OutType yt, hipStream_t stream) {
    if (M <= 16) {
        dispatch16(-1, xq, sx, packed, gamma, M, N, K, y, yt, stream);
    } else if (M <= 32) {
        launch64<4, 2, 4>(xq, sx, packed, gamma, M, N, K, y, yt, stream);
    } else {
        launch64<2, 4, 4>(xq, sx, packed, gamma, M, N, K, y, yt, stream);
    }
    return hipGetLastError();
}

bool gemv_fused_supports(int64_t M, int64_t N, int64_t K, const void* x) {
    (void)N;
    return M >= 1 && M <= 16 && K % 16 == 0 && reinterpret_cast<uintptr_t>(x) % 16 == 0 &&
           kGemvLdsHeader * sizeof(uint4) + gemv16_x_lds_bytes(M, K) <= kGemvLdsBudget;
}

hipError_t launch_linear_fused_2bit(const void* x, bool bf16, const void* packed, const float* gamma, int64_t M,
                                    int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream) {
    dispatch16(bf16 ? kXFusedBf16 : kXFusedF32, x, nullptr, packed, gamma, M, N, K, y, yt, stream);
    return hipGetLastError();
}

}  // namespace bitnet

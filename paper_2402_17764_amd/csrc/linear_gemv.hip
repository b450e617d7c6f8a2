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
// kR    row blocks (16 rows each) per wave
// kS    waves that split K: wave ws takes steps ws, ws + kS, ...
// kW    row slots per workgroup (waves with different row blocks), workgroup = kS * kW waves
// kD    register prefetch depth in steps
// kXLds activations staged once per workgroup in LDS (needs M * Kpad bytes) instead of global loads
template <int kR, int kS, int kW, int kD, bool kXLds>
__global__ __launch_bounds__(kS * kW * kWave) void linear_gemv16_2bit(
        const int8_t* __restrict__ xq, const float* __restrict__ sx, const uint4* __restrict__ packed,
        const float* __restrict__ gamma, int M, int64_t N, int64_t K, int Kq, int RB,
        int items /* K steps per wave, rounded up to a multiple of kD */, void* __restrict__ y, OutType yt) {
    extern __shared__ uint4 smem[];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int r = lane & 15;
    const int g = lane >> 4;
    const int ws = wave % kS;
    const int ww = wave / kS;
    const int steps = (Kq + 3) >> 2;
    const int rbw = (blockIdx.x * kW + ww) * kR;
    const int Kpad = steps * 256;
    const int last_full = (int)(K >> 8) - 1;         // last step whose 256 columns all exist (-1: none)

    if (kXLds) {
        // rows < M of x_q, zero padded to Kpad columns
        const int nvec = M * (Kpad >> 4);
        for (int v = threadIdx.x; v < nvec; v += kS * kW * kWave) {
            const int m = v / (Kpad >> 4), kv = v % (Kpad >> 4);
            uint4 val = make_uint4(0, 0, 0, 0);
            if ((int64_t)kv * 16 + 16 <= K) val = reinterpret_cast<const uint4*>(xq + (int64_t)m * K)[kv];
            smem[v] = val;
        }
    }

    const uint4* wp[kR];
#pragma unroll
    for (int a = 0; a < kR; ++a) wp[a] = packed + (int64_t)min(rbw + a, RB - 1) * 64 + lane;
    const int64_t wstride = (int64_t)RB * 64;                      // quads per full step
    const int mrow = min(r, M - 1);
    const uint4* xg = reinterpret_cast<const uint4*>(xq + (int64_t)mrow * K + 64 * g);
    const uint4* xl = smem + mrow * (Kpad >> 4) + 4 * g;

    v4i acc[kR];
#pragma unroll
    for (int a = 0; a < kR; ++a) acc[a] = (v4i){0, 0, 0, 0};

    struct Stage { uint4 w[kR]; uint4 x[4]; };
    auto load = [&](Stage& s, int item) {
        const int sl = max(min(ws + item * kS, last_full), 0);     // redirected if past the last full step
#pragma unroll
        for (int a = 0; a < kR; ++a) s.w[a] = wp[a][(int64_t)sl * wstride];
        if (!kXLds) {
#pragma unroll
            for (int j = 0; j < 4; ++j) s.x[j] = xg[(int64_t)sl * 16 + j];
        }
    };
    auto mac = [&](Stage& s, int item) {
        const int step = ws + item * kS;
        const uint32_t keep = step <= last_full ? 0xFFFFFFFFu : 0u;
        if (kXLds) {
            const int sl = max(min(step, last_full), 0);
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

    if (kXLds) __syncthreads();
    if (last_full >= 0) {
        Stage st[kD];
#pragma unroll
        for (int d = 0; d < kD; ++d) load(st[d], d);
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
    }

    // columns past the last whole step (K % 256 != 0): one guarded step, taken by one K-split wave
    if ((K & 255) != 0 && ws == (last_full + 1) % kS) {
        const int step = last_full + 1;
        const int kq = 4 * step + g;
        const int nq = Kq - 4 * step;
        const int64_t kbase = (int64_t)kq * 64;
#pragma unroll
        for (int a = 0; a < kR; ++a) {
            uint4 wq = make_uint4(0, 0, 0, 0);
            const int rb = min(rbw + a, RB - 1);
            if (kq < Kq) wq = packed[(int64_t)step * wstride + (int64_t)rb * 16 * nq + lane];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint4 xv = make_uint4(0, 0, 0, 0);
                if (kbase + 16 * j + 16 <= K) xv = xg[(int64_t)step * 16 + j];
                acc[a] = __builtin_amdgcn_mfma_i32_16x16x64_i8(decode_word(quad_word(wq, j)), as_v4i(xv), acc[a], 0, 0, 0);
            }
        }
    }

    if (kS > 1) {
        // fold the K slices; the LDS region is shared with x, so wait until every wave is done with it
        v4i* fold = reinterpret_cast<v4i*>(smem);
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
        const float scale = yt == OutType::I32 ? 0.0f : (gamma[0] * sx[r]) / kQb;
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

template <int kR, int kS, int kW, int kD>
static void launch16(bool xlds, const int8_t* xq, const float* sx, const void* packed, const float* gamma, int64_t M,
                     int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream) {
    const int Kq = (int)ceil_div(K, kColsPerQuad);
    const int RB = (int)ceil_div(N, kRowsPerBlock);
    const int steps = (Kq + 3) / 4;
    int items = (int)ceil_div(K >> 8, kS);
    items = (int)ceil_div(items, kD) * kD;
    const size_t lds_fold = kS > 1 ? (size_t)kW * kS * kR * kWave * 16 : 0;
    const size_t lds_x = (size_t)M * steps * 256;
    if (lds_x > kGemvLdsBudget) xlds = false;
    const size_t lds = xlds && lds_x > lds_fold ? lds_x : lds_fold;
    dim3 grid((unsigned)ceil_div(RB, kW * kR)), block(kS * kW * kWave);
    const uint4* p = static_cast<const uint4*>(packed);
    if (xlds)
        hipLaunchKernelGGL((linear_gemv16_2bit<kR, kS, kW, kD, true>), grid, block, lds, stream, xq, sx, p, gamma, (int)M, N, K,
                           Kq, RB, items, y, yt);
    else
        hipLaunchKernelGGL((linear_gemv16_2bit<kR, kS, kW, kD, false>), grid, block, lds, stream, xq, sx, p, gamma, (int)M, N, K,
                           Kq, RB, items, y, yt);
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

// Shape heuristics, from sweeps on MI355X: many row blocks -> few deep-prefetching waves, each owning
// four row blocks for all of K; few row blocks -> split K over more waves so that the whole matrix is
// requested within the first memory round trip.
hipError_t launch_linear_gemv_2bit(const int8_t* xq, const float* sx, const void* packed,
                                   const float* gamma, int64_t M, int64_t N, int64_t K, void* y,
                                   OutType yt, hipStream_t stream) {
    const int64_t RB = ceil_div(N, kRowsPerBlock);
    const int64_t steps = ceil_div(K, 256);
#define GEMV16(R_, S_, W_, D_, X_) launch16<R_, S_, W_, D_>(X_, xq, sx, packed, gamma, M, N, K, y, yt, stream)
    if (M <= 16) {
        if (RB >= 2048)                       GEMV16(4, 1, 4, 2, false);
        else if (RB >= 1024 && steps >= 16)   GEMV16(1, 2, 2, 4, true);
        else if (RB >= 1024)                  GEMV16(1, 4, 2, 1, true);
        else if (RB >= 400 && steps >= 64)    GEMV16(2, 4, 1, 4, false);
        else if (RB >= 400)                   GEMV16(1, 4, 1, 4, true);
        else if (steps >= 24)                 GEMV16(1, 16, 1, 1, true);
        else                                  GEMV16(1, 4, 1, 4, false);
    } else if (M <= 32) {
        launch64<4, 2, 4>(xq, sx, packed, gamma, M, N, K, y, yt, stream);
    } else {
        launch64<2, 4, 4>(xq, sx, packed, gamma, M, N, K, y, yt, stream);
    }
#undef GEMV16
    return hipGetLastError();
}

}  // namespace bitnet

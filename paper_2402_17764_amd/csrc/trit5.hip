// The 5-trits-per-byte format (1.6 bits per weight; the paper notes that 2 bits leave room above the
// 1.58-bit information content of a ternary weight, Section 3 of arXiv 2402.17764): packer, unpack
// helper, reference product and a weight-streaming kernel for M <= 16, measured against the 2-bit one.
//
// Layout (bitnet.h): byte p of a 16-byte quad carries digits 0..3 = four consecutive columns 4p..4p+3
// and digit 4 = column 64 + p of the quad's 80 columns.  The streaming kernel keeps a 243-entry table
// in LDS that maps a byte to its five decoded operand bytes (64 * code), so a byte's first four digits
// arrive as one ready MFMA operand register; the sixteen fifth digits of a quad are gathered into the
// four registers of a fifth MFMA.  One step = 320 columns = five v_mfma_i32_16x16x64_i8 per row block.
#include "bitnet_device.hpp"
#include "bitnet_internal.hpp"

namespace bitnet {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kTritCols = 80;            // columns per quad
constexpr int kTritStep = 320;           // columns per step (4 quads)

// byte offset and digit of column k of row n
__host__ __device__ inline void trit5_locate(int64_t n, int64_t k, int64_t RB, int64_t* byte_index, int* digit) {
    const int64_t s = k / kTritStep;
    const int c = (int)(k % kTritStep);
    const int g = c / kTritCols, q = c % kTritCols;
    const int64_t quad = 64 * (RB * s + (n >> 4)) + 16 * g + (n & 15);
    if (q < 64) { *byte_index = quad * 16 + (q >> 2); *digit = q & 3; }
    else        { *byte_index = quad * 16 + (q - 64); *digit = 4; }
}

__device__ inline int trit5_digit(uint32_t byte, int d) {
    const uint32_t p3 = d == 0 ? 1u : d == 1 ? 3u : d == 2 ? 9u : d == 3 ? 27u : 81u;
    return (int)((byte / p3) % 3u) - 1;
}

// ---------------------------------------------------------------------------------------------------
// packer: one wave per chunk of the packed layout (a 16-row block x one step of 320 columns: 20 KB of fp32 in, 1 KiB out)
// ---------------------------------------------------------------------------------------------------
// The wave reads the chunk's 16 x 320 weights as 20 rounds of 64 four-element loads that run along the rows (a thread
// that walked its own 80 columns would touch 64 cache lines per load instruction: 1.3 TB/s), ternarizes them where they
// land and parks the digits (code + 1, one per byte) in a wave-private LDS tile; lane 16 g + r then collects the 80
// digits of row r, quad g and forms its 16 bytes, so that the wave stores the chunk as one 1 KiB run.  The tile's rows
// are 81 words apart: both the row-wise writes and the quad-wise reads spread over the banks.
__device__ inline float trit_w(const float* p) { return *p; }
__device__ inline float trit_w(const uint16_t* p) { return bf16_to_f32(*p); }
__device__ inline void trit_w4(const float* p, float (&w)[4]) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
}
__device__ inline void trit_w4(const uint16_t* p, float (&w)[4]) {
    const uint2 u = *reinterpret_cast<const uint2*>(p);
    w[0] = __uint_as_float(u.x << 16); w[1] = __uint_as_float(u.x & 0xFFFF0000u);
    w[2] = __uint_as_float(u.y << 16); w[3] = __uint_as_float(u.y & 0xFFFF0000u);
}

constexpr int kTritTilePitch = 81;                   // words per tile row: 80 + 1
template <typename T>
__global__ __launch_bounds__(256) void ternarize_pack_trit5(const T* __restrict__ W, int64_t N, int64_t K, int64_t RB,
                                                            int64_t steps, int vec_ok /* rows start on 4-element boundaries */,
                                                            const float* __restrict__ gamma, uint4* __restrict__ packed) {
    __shared__ uint32_t tiles[4][kRowsPerBlock * kTritTilePitch];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int64_t chunk = (int64_t)blockIdx.x * 4 + wave;             // = RB * step + row block: the chunk's place in the packed matrix
    if (chunk >= RB * steps) return;                                   // whole waves leave; no workgroup barrier below
    const int64_t s = chunk / RB, rb = chunk - s * RB;
    const float d = gamma[0] + kEps;                                   // Eq. (1): gamma + eps
    uint32_t* tile = tiles[wave];
#pragma unroll 4
    for (int i = 0; i < 20; ++i) {
        const int f = i * kWave + lane;                                // four-element piece f of the chunk, row-major
        const int row = f / 80, c4 = f - row * 80;
        const int64_t n = rb * kRowsPerBlock + row, k = s * kTritStep + 4 * c4;
        float w[4] = {0.0f, 0.0f, 0.0f, 0.0f};                         // padding quantizes to code 0
        if (n < N) {
            const T* src = W + n * K + k;
            if (vec_ok && k < K) {
                trit_w4(src, w);                                       // K is a multiple of 4 here: k < K covers k + 3
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (k + e < K) w[e] = trit_w(src + e);
            }
        }
        uint32_t t = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float r = fminf(1.0f, fmaxf(-1.0f, rintf(w[e] / d)));   // Eq. (1)-(2)
            t |= (uint32_t)((int)r + 1) << (8 * e);
        }
        tile[row * kTritTilePitch + c4] = t;
    }
    __builtin_amdgcn_wave_barrier();                                   // the tile is the wave's own: its LDS accesses complete in order
    const int g = lane >> 4, r = lane & 15;
    const uint32_t* src = tile + r * kTritTilePitch + 20 * g;
    uint32_t dg[20];
#pragma unroll
    for (int w = 0; w < 20; ++w) dg[w] = src[w];
    uint32_t words[4] = {0, 0, 0, 0};
#pragma unroll
    for (int p = 0; p < 16; ++p) {
        const uint32_t q = dg[p];                                      // digits of columns 4 p .. 4 p + 3
        const uint32_t fifth = (dg[16 + (p >> 2)] >> (8 * (p & 3))) & 0xFFu;   // ... and of column 64 + p
        const uint32_t b = (q & 0xFFu) + 3u * ((q >> 8) & 0xFFu) + 9u * ((q >> 16) & 0xFFu) + 27u * (q >> 24) + 81u * fifth;
        words[p >> 2] |= b << (8 * (p & 3));
    }
    packed[64 * chunk + lane] = make_uint4(words[0], words[1], words[2], words[3]);
}

// ---------------------------------------------------------------------------------------------------
// unpack helper and reference product
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void unpack_trit5(const uint8_t* __restrict__ packed, int64_t N, int64_t K, int64_t RB,
                                                    int8_t* __restrict__ codes) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= N * K) return;
    int64_t bi; int dg;
    trit5_locate(idx / K, idx % K, RB, &bi, &dg);
    codes[idx] = (int8_t)trit5_digit(packed[bi], dg);
}

__global__ __launch_bounds__(256) void linear_reference_trit5(const int8_t* __restrict__ xq, const float* __restrict__ sx,
                                                              const uint8_t* __restrict__ packed,
                                                              const float* __restrict__ gamma, int64_t N, int64_t K,
                                                              int64_t RB, void* __restrict__ y, OutType yt) {
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t m = blockIdx.y;
    if (n >= N) return;
    const int8_t* xr = xq + m * K;
    int32_t acc = 0;
    for (int64_t k = 0; k < K; ++k) {
        int64_t bi; int dg;
        trit5_locate(n, k, RB, &bi, &dg);
        const int code = trit5_digit(packed[bi], dg);
        if (code > 0) acc += xr[k];
        else if (code < 0) acc -= xr[k];
    }
    const int64_t idx = m * N + n;
    if (yt == OutType::I32) static_cast<int32_t*>(y)[idx] = acc;
    else {
        const float v = (float)acc * ((gamma[0] * sx[m]) / kQb);
        if (yt == OutType::F32) static_cast<float*>(y)[idx] = v;
        else static_cast<uint16_t*>(y)[idx] = f32_to_bf16(v);
    }
}

// ---------------------------------------------------------------------------------------------------
// weight-streaming kernel, M <= 16
// ---------------------------------------------------------------------------------------------------
__device__ inline v4i trit_as_v4i(const uint4& u) {
    v4i a;
    a.x = (int)u.x; a.y = (int)u.y; a.z = (int)u.z; a.w = (int)u.w;
    return a;
}

// kR row blocks per wave, kS waves splitting K, kD steps of loads in flight (same scheme as the 2-bit kernel:
// branch-free masked loop, out-of-range steps / rows / tokens redirected and zeroed)
template <int kR, int kS, int kD>
__global__ __launch_bounds__(kS * kWave) void linear_gemv16_trit5(
        const int8_t* __restrict__ xq, const float* __restrict__ sx, const uint4* __restrict__ packed,
        const float* __restrict__ gamma, int M, int64_t N, int64_t K, int RB, int steps, int items,
        void* __restrict__ y, OutType yt) {
    __shared__ uint2 lut[256];                       // byte -> {digits 0..3 as 4 operand bytes, digit 4 as 1 byte}
    __shared__ v4i fold[kS][kR][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int r = lane & 15, g = lane >> 4;
    const int rb0 = blockIdx.x * kR;

    for (int b = threadIdx.x; b < 256; b += kS * kWave) {
        uint32_t lo = 0, hi = 0;
        if (b < 243) {
#pragma unroll
            for (int dgt = 0; dgt < 4; ++dgt) lo |= ((uint32_t)(trit5_digit(b, dgt) * 64) & 0xFFu) << (8 * dgt);
            hi = (uint32_t)(trit5_digit(b, 4) * 64) & 0xFFu;
        }
        lut[b] = make_uint2(lo, hi);
    }

    const int64_t wstride = (int64_t)RB * 64;
    const uint4* wp[kR];
#pragma unroll
    for (int a = 0; a < kR; ++a) wp[a] = packed + (int64_t)min(rb0 + a, RB - 1) * 64 + lane;
    const int8_t* xg = xq + (int64_t)min(r, M - 1) * K;

    v4i acc[kR];
#pragma unroll
    for (int a = 0; a < kR; ++a) acc[a] = (v4i){0, 0, 0, 0};

    struct Stage { uint4 w[kR]; uint4 x[5]; };
    auto load = [&](Stage& s, int item) {
        const int sl = min(wave + item * kS, steps - 1);
#pragma unroll
        for (int a = 0; a < kR; ++a) s.w[a] = load_streaming_b128(wp[a] + (int64_t)sl * wstride);
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            const int64_t col = min((int64_t)sl * kTritStep + kTritCols * g + 16 * j, K - 16);   // past K: zero codes
            s.x[j] = *reinterpret_cast<const uint4*>(xg + col);
        }
    };
    auto mac = [&](Stage& s, int item) {
        const bool live = wave + item * kS < steps;
#pragma unroll
        for (int a = 0; a < kR; ++a) {
            const uint32_t wd[4] = {s.w[a].x, s.w[a].y, s.w[a].z, s.w[a].w};
            v4i op[5];
#pragma unroll
            for (int p = 0; p < 16; ++p) {
                // byte 121 = digits (1,1,1,1,1) = five zero codes: what a step past the end contributes
                const uint32_t byte = live ? ((wd[p >> 2] >> (8 * (p & 3))) & 0xFFu) : 121u;
                const uint2 e = lut[byte];
                op[p >> 2][p & 3] = (int)e.x;
                if ((p & 3) == 0) op[4][p >> 2] = (int)e.y;
                else op[4][p >> 2] |= (int)(e.y << (8 * (p & 3)));
            }
#pragma unroll
            for (int j = 0; j < 5; ++j)
                acc[a] = __builtin_amdgcn_mfma_i32_16x16x64_i8(op[j], trit_as_v4i(s.x[j]), acc[a], 0, 0, 0);
        }
    };

    Stage st[kD];
#pragma unroll
    for (int d = 0; d < kD; ++d) load(st[d], d);
    __syncthreads();                                  // table ready
    int i = 0;
    for (; i + kD < items; i += kD) {
#pragma unroll
        for (int d = 0; d < kD; ++d) {
            mac(st[d], i + d);
            __builtin_amdgcn_sched_barrier(0);
            load(st[d], i + d + kD);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int d = 0; d < kD; ++d) mac(st[d], i + d);

    if (kS > 1) {
#pragma unroll
        for (int a = 0; a < kR; ++a) fold[wave][a][lane] = acc[a];
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int a = 0; a < kR; ++a)
#pragma unroll
            for (int w = 1; w < kS; ++w) {
                const v4i o = fold[w][a][lane];
                acc[a].x += o.x; acc[a].y += o.y; acc[a].z += o.z; acc[a].w += o.w;
            }
    }
    if (r < M) {
        const float scale = yt == OutType::I32 ? 0.0f : (gamma[0] * sx[r]) / kQb;
#pragma unroll
        for (int a = 0; a < kR; ++a) {
            const int64_t n0 = (int64_t)(rb0 + a) * 16 + 4 * g;
            const int v[4] = {acc[a].x >> 6, acc[a].y >> 6, acc[a].z >> 6, acc[a].w >> 6};   // drop the factor 64
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (n0 + e >= N) continue;
                const int64_t idx = (int64_t)r * N + n0 + e;
                if (yt == OutType::I32) static_cast<int32_t*>(y)[idx] = v[e];
                else if (yt == OutType::F32) static_cast<float*>(y)[idx] = (float)v[e] * scale;
                else static_cast<uint16_t*>(y)[idx] = f32_to_bf16((float)v[e] * scale);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------------
hipError_t launch_pack_trit5(const void* W, bool bf16, int64_t N, int64_t K, const float* gamma, void* packed,
                             hipStream_t stream) {
    const int64_t RB = ceil_div(N, kRowsPerBlock);
    const int64_t steps = ceil_div(K, kTritStep);
    dim3 grid((unsigned)ceil_div(RB * steps, 4));
    const int vec_ok = K % 4 == 0 && reinterpret_cast<uintptr_t>(W) % (bf16 ? 8 : 16) == 0;
    if (bf16)
        hipLaunchKernelGGL(ternarize_pack_trit5<uint16_t>, grid, dim3(256), 0, stream, static_cast<const uint16_t*>(W), N, K, RB,
                           steps, vec_ok, gamma, static_cast<uint4*>(packed));
    else
        hipLaunchKernelGGL(ternarize_pack_trit5<float>, grid, dim3(256), 0, stream, static_cast<const float*>(W), N, K, RB,
                           steps, vec_ok, gamma, static_cast<uint4*>(packed));
    return hipGetLastError();
}

hipError_t launch_unpack_trit5(const void* packed, int64_t N, int64_t K, int8_t* codes, hipStream_t stream) {
    hipLaunchKernelGGL(unpack_trit5, dim3((unsigned)ceil_div(N * K, 256)), dim3(256), 0, stream,
                       static_cast<const uint8_t*>(packed), N, K, ceil_div(N, kRowsPerBlock), codes);
    return hipGetLastError();
}

hipError_t launch_linear_reference_trit5(const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                                         int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream) {
    const size_t ysz = yt == OutType::BF16 ? 2 : 4;
    for (int64_t m0 = 0; m0 < M; m0 += 32768) {
        const int64_t mc = (M - m0) < 32768 ? (M - m0) : 32768;
        dim3 grid((unsigned)ceil_div(N, 256), (unsigned)mc);
        hipLaunchKernelGGL(linear_reference_trit5, grid, dim3(256), 0, stream, xq + m0 * K, sx + m0,
                           static_cast<const uint8_t*>(packed), gamma, N, K, ceil_div(N, kRowsPerBlock),
                           static_cast<char*>(y) + m0 * N * ysz, yt);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------
// repacking between the two formats on the device (no weights in full precision needed)
// ---------------------------------------------------------------------------------------------------
// 320 columns are one step of the 5-trit layout (4 quads of 80) and five quads of the 2-bit layout (64 each): one
// thread moves the 320 codes of one row.  Consecutive threads take consecutive rows of a 16-row block, so their
// 16-byte loads and stores form 256-byte runs in both layouts.
//
// 5-trit -> 2-bit.  A 5-trit byte p of quad g holds quad columns 4p .. 4p+3, i.e. step columns 80 g + 4 p + (0 .. 3):
// four columns that the 2-bit layout keeps in one 32-bit word (word (80 g + 4 p) / 16 of the step), in field i = p & 3
// of its four bytes; the table gives those four 2-bit codes already spread to bits 0, 8, 16, 24.  The sixteen fifth
// digits of a quad are step columns 80 g + 64 .. 80 g + 79: exactly one word.
__global__ __launch_bounds__(256) void repack_trit5_to_2bit(const uint4* __restrict__ in, int64_t RB, int64_t steps5,
                                                            int64_t Kq2, uint4* __restrict__ out) {
    __shared__ uint2 lut[256];                       // byte -> {codes 0..3 as 2-bit fields at bits 0, 8, 16, 24; code 4}
    {
        const int b = threadIdx.x;
        uint32_t sp = 0, c4 = 0;
        if (b < 243) {
#pragma unroll
            for (int d = 0; d < 4; ++d) sp |= ((uint32_t)trit5_digit(b, d) & 3u) << (8 * d);
            c4 = (uint32_t)trit5_digit(b, 4) & 3u;
        }
        lut[b] = make_uint2(sp, c4);
    }
    __syncthreads();
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= 16 * RB * steps5) return;
    const int r = (int)(idx & 15);
    const int64_t rb = (idx >> 4) % RB, s5 = (idx >> 4) / RB;
    uint32_t words[20];                              // the row's 320 codes as twenty 2-bit words of 16 columns
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const uint4 q = in[64 * (RB * s5 + rb) + 16 * g + r];
        const uint32_t wd[4] = {q.x, q.y, q.z, q.w};
        uint32_t fifth = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t w = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint2 e = lut[(wd[j] >> (8 * i)) & 0xFFu];               // byte p = 4 j + i
                w |= e.x << (2 * i);
                fifth |= e.y << (8 * i + 2 * j);                                // column 64 + p = 64 + 4 j + i: byte i, field j
            }
            words[5 * g + j] = w;
        }
        words[5 * g + 4] = fifth;
    }
#pragma unroll
    for (int q5 = 0; q5 < 5; ++q5) {
        const int64_t kq = 5 * s5 + q5;
        if (kq < Kq2)
            out[quad_index_2bit(kq, rb, r, Kq2, RB)] = make_uint4(words[4 * q5], words[4 * q5 + 1], words[4 * q5 + 2], words[4 * q5 + 3]);
    }
}

// 2-bit -> 5-trit: the same move backwards; 2-bit quads past the matrix's last one read as zero codes.
__global__ __launch_bounds__(256) void repack_2bit_to_trit5(const uint4* __restrict__ in, int64_t RB, int64_t steps5,
                                                            int64_t Kq2, uint4* __restrict__ out) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= 16 * RB * steps5) return;
    const int r = (int)(idx & 15);
    const int64_t rb = (idx >> 4) % RB, s5 = (idx >> 4) / RB;
    uint32_t words[20];
#pragma unroll
    for (int q5 = 0; q5 < 5; ++q5) {
        const int64_t kq = 5 * s5 + q5;
        uint4 q = make_uint4(0, 0, 0, 0);
        if (kq < Kq2) q = in[quad_index_2bit(kq, rb, r, Kq2, RB)];
        words[4 * q5] = q.x; words[4 * q5 + 1] = q.y; words[4 * q5 + 2] = q.z; words[4 * q5 + 3] = q.w;
    }
    // code + 1 of step column c: word c / 16, bits 8 (c & 3) + 2 ((c & 15) >> 2)
    auto digit = [&](int c) -> uint32_t {
        const uint32_t f = (words[c >> 4] >> (8 * (c & 3) + 2 * ((c & 15) >> 2))) & 3u;   // 0, 1, 3 for codes 0, +1, -1
        return f == 3u ? 0u : f + 1u;
    };
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        uint32_t o[4] = {0, 0, 0, 0};
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const int c = 80 * g + 4 * p;
            const uint32_t b = digit(c) + 3 * digit(c + 1) + 9 * digit(c + 2) + 27 * digit(c + 3) + 81 * digit(80 * g + 64 + p);
            o[p >> 2] |= b << (8 * (p & 3));
        }
        out[64 * (RB * s5 + rb) + 16 * g + r] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

hipError_t launch_repack(const void* in, bool in_trit5, int64_t N, int64_t K, void* out, hipStream_t stream) {
    const int64_t RB = ceil_div(N, kRowsPerBlock), steps5 = ceil_div(K, kTritStep), Kq2 = ceil_div(K, kColsPerQuad);
    dim3 grid((unsigned)ceil_div(16 * RB * steps5, 256));
    if (in_trit5)
        hipLaunchKernelGGL(repack_trit5_to_2bit, grid, dim3(256), 0, stream, static_cast<const uint4*>(in), RB, steps5, Kq2,
                           static_cast<uint4*>(out));
    else
        hipLaunchKernelGGL(repack_2bit_to_trit5, grid, dim3(256), 0, stream, static_cast<const uint4*>(in), RB, steps5, Kq2,
                           static_cast<uint4*>(out));
    return hipGetLastError();
}

bool gemv_trit5_supports(int64_t M, int64_t N, int64_t K, const void* xq) {
    (void)N;
    return M >= 1 && M <= 16 && K % 16 == 0 && reinterpret_cast<uintptr_t>(xq) % 16 == 0;
}

template <int kR, int kS, int kD>
static void launch_trit5(const int8_t* xq, const float* sx, const void* packed, const float* gamma, int64_t M, int64_t N,
                         int64_t K, void* y, OutType yt, hipStream_t stream) {
    const int RB = (int)ceil_div(N, kRowsPerBlock);
    const int steps = (int)ceil_div(K, kTritStep);
    int items = (int)ceil_div(steps, kS);
    items = (int)ceil_div(items, kD) * kD;
    hipLaunchKernelGGL((linear_gemv16_trit5<kR, kS, kD>), dim3((unsigned)ceil_div(RB, kR)), dim3(kS * kWave), 0, stream, xq, sx,
                       static_cast<const uint4*>(packed), gamma, (int)M, N, K, RB, steps, items, y, yt);
}

hipError_t launch_linear_gemv_trit5(const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                                    int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream) {
    const int64_t RB = ceil_div(N, kRowsPerBlock);
    const int64_t steps = ceil_div(K, kTritStep);
    // the share of a wave's padded K walk (a multiple of the prefetch depth) that is real steps
    auto walk = [&](int ks, int kd) { return (double)steps / (double)(ceil_div(ceil_div(steps, (int64_t)ks), (int64_t)kd) * kd * ks); };
    // Measured on MI355X, M = 1, fifteen forms per shape: 3200 -> 3200 4.0 -> 3.5 us and 3200 -> 17280 8.0 -> 6.6 us with
    // depth 3 (ten steps fill three rounds of four waves exactly; thirteen steps would walk 24), 4096 -> 22016 9.4 -> 8.7 us
    // and 28672 -> 8192 17.9 -> 15.5 us with two row blocks per wave.
    if (RB >= 2048)                                   launch_trit5<2, 2, 2>(xq, sx, packed, gamma, M, N, K, y, yt, stream);
    else if (steps >= 64 && RB >= 512)                launch_trit5<2, 8, 2>(xq, sx, packed, gamma, M, N, K, y, yt, stream);
    else if (steps >= 24)                             launch_trit5<1, 8, 2>(xq, sx, packed, gamma, M, N, K, y, yt, stream);
    else if (walk(4, 3) > walk(4, 2))                 launch_trit5<1, 4, 3>(xq, sx, packed, gamma, M, N, K, y, yt, stream);
    else if (RB >= 1024)                              launch_trit5<2, 4, 2>(xq, sx, packed, gamma, M, N, K, y, yt, stream);
    else                                              launch_trit5<1, 4, 2>(xq, sx, packed, gamma, M, N, K, y, yt, stream);
    return hipGetLastError();
}

}  // namespace bitnet

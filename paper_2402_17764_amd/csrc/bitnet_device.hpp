// Device-side helpers shared by the gfx950 kernels of the BitLinear library: wave64 reductions,
// bf16 widening, and the arithmetic of the packed 2-bit tile layout documented in bitnet.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bitnet {

constexpr int kWave = 64;              // CDNA wavefront width
constexpr float kEps = 1e-5f;          // epsilon of Eq. (1) and the floor of the per-token absmax
constexpr float kQb = 127.0f;          // Q_b for 8-bit symmetric activations (Section 2)

constexpr int kRowsPerBlock = 16;      // rows of one packed tile (= MFMA 16x16x64 operand rows)
constexpr int kColsPerQuad = 64;       // columns held by one 16-byte quad of the 2-bit format

__host__ __device__ inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// A 16-byte load with the streaming ("nt") cache policy, for data a launch reads exactly once: the packed weights
// of the M <= 4 decode kernel (3B decode step 0.547 -> 0.493 ms, 70B gate/up 22.5 -> 22.0 us) and W in the packing
// pass of the weight quantizer.  Kernels whose workgroups share weight tiles through the L2 (batched decode with
// token tiles, prefill) measured 1-10 % slower with it and keep ordinary loads.
__device__ inline uint4 load_streaming_b128(const void* p) {
    typedef unsigned v4u __attribute__((ext_vector_type(4)));
    const v4u r = __builtin_nontemporal_load(static_cast<const v4u*>(p));
    return make_uint4(r.x, r.y, r.z, r.w);
}

// bf16 bit pattern -> fp32 (exact).
__device__ inline float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ inline uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// ---- Section 2, the int8 code of one activation ------------------------------------------------------
// x_q = clip(round(x * inv), -127, 127) with inv = fl(127 / s) and round = ties to even.  p = fl(x * inv) is one fp32
// multiply; adding 1.5 * 2^23 to it rounds p to the nearest integer, ties to even, in the addition itself (the sum lies
// in [2^23, 2^24), where floats are the integers; the constant is even, so the tie rule is p's), and leaves that integer,
// two's complement, in the low bits of the result -- one add where rint, a conversion and a clamp were three
// instructions.  The clamp of the definition never binds for finite input: |x| <= s and inv <= (127 / s)(1 + 2^-24) give
// |p| < 127.5.  (Contraction is off for the whole library, so the multiply and the add are never fused.)
constexpr float kRoundMagic = 12582912.0f;       // 1.5 * 2^23
__device__ inline uint32_t quantize_bits(float v, float inv) {
    const float p = v * inv;
    return __float_as_uint(p + kRoundMagic);      // low byte = x_q
}
// four values -> their four codes in one word, lowest address first (two byte permutes and an OR)
__device__ inline uint32_t pack4_quantized(float a, float b, float c, float d, float inv) {
    const uint32_t ab = __builtin_amdgcn_perm(quantize_bits(b, inv), quantize_bits(a, inv), 0x0c0c0400u);   // bytes a, b, 0, 0
    const uint32_t cd = __builtin_amdgcn_perm(quantize_bits(d, inv), quantize_bits(c, inv), 0x04000c0cu);   // bytes 0, 0, c, d
    return ab | cd;
}

// ---- wave64 all-lanes reductions with DPP for the four in-row steps ------------------------------
// quad_perm [1,0,3,2] = 0xB1, quad_perm [2,3,0,1] = 0x4E, row_half_mirror = 0x141, row_mirror = 0x140.
template <int kCtrl>
__device__ inline float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), kCtrl, 0xF, 0xF, true));
}
template <int kCtrl>
__device__ inline uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, kCtrl, 0xF, 0xF, true);
}

// max over the 64 lanes of non-negative finite floats; every lane gets the result.
__device__ inline float wave_max_nonneg(float v) {
    v = fmaxf(v, dpp_f32<0xB1>(v));     // lane ^ 1
    v = fmaxf(v, dpp_f32<0x4E>(v));     // lane ^ 2
    v = fmaxf(v, dpp_f32<0x141>(v));    // other quad of the 8
    v = fmaxf(v, dpp_f32<0x140>(v));    // other half of the 16
    v = fmaxf(v, __shfl_xor(v, 16, kWave));
    v = fmaxf(v, __shfl_xor(v, 32, kWave));
    return v;
}

// OR over each aligned group of four lanes; every lane of the group gets the result.
__device__ inline uint32_t quad_or(uint32_t v) {
    v |= dpp_u32<0xB1>(v);
    v |= dpp_u32<0x4E>(v);
    return v;
}

// ---- double-double accumulation (error-free transformations, Knuth TwoSum) -----------------------
struct dd { double hi, lo; };

__device__ inline void dd_add_double(dd& s, double a) {
    double t = s.hi + a;
    double bb = t - s.hi;
    double err = (s.hi - (t - bb)) + (a - bb);
    s.hi = t;
    s.lo += err;
}
__device__ inline void dd_add_dd(dd& s, const dd& o) {
    double t = s.hi + o.hi;
    double bb = t - s.hi;
    double err = (s.hi - (t - bb)) + (o.hi - bb);
    s.hi = t;
    s.lo += err + o.lo;
}

// one double moved across lanes with a DPP control (both 32-bit halves)
template <int kCtrl>
__device__ inline double dpp_f64(double v) {
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = dpp_u32<kCtrl>((uint32_t)u), hi = dpp_u32<kCtrl>((uint32_t)(u >> 32));
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ inline double readlane_f64(double v, int lane) {
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)u, lane);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(u >> 32), lane);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// Sum over a wave of per-lane double-double partial sums; every lane gets the result.  The sums are exact to
// ~2^-100, far below the rounding of the result to fp64, so the shape of the tree does not show: four DPP steps
// inside each row of 16 lanes, the four rows through scalar reads.
__device__ inline dd wave_sum_dd(dd v) {
    dd_add_dd(v, dd{dpp_f64<0xB1>(v.hi), dpp_f64<0xB1>(v.lo)});       // lane ^ 1
    dd_add_dd(v, dd{dpp_f64<0x4E>(v.hi), dpp_f64<0x4E>(v.lo)});       // lane ^ 2
    dd_add_dd(v, dd{dpp_f64<0x141>(v.hi), dpp_f64<0x141>(v.lo)});     // other quad of the 8
    dd_add_dd(v, dd{dpp_f64<0x140>(v.hi), dpp_f64<0x140>(v.lo)});     // other half of the 16
    dd w{readlane_f64(v.hi, 0), readlane_f64(v.lo, 0)};
    dd_add_dd(w, dd{readlane_f64(v.hi, 16), readlane_f64(v.lo, 16)});
    dd_add_dd(w, dd{readlane_f64(v.hi, 32), readlane_f64(v.lo, 32)});
    dd_add_dd(w, dd{readlane_f64(v.hi, 48), readlane_f64(v.lo, 48)});
    return w;
}

// ... and over the block (the waves in order); every thread gets the result.
template <int kWaves>
__device__ inline double block_sum_dd(dd v, double* sh_hi, double* sh_lo) {
    const dd w = wave_sum_dd(v);
    if (kWaves == 1) return w.hi + w.lo;
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { sh_hi[wave] = w.hi; sh_lo[wave] = w.lo; }
    __syncthreads();
    dd t{sh_hi[0], sh_lo[0]};
#pragma unroll
    for (int q = 1; q < kWaves; ++q) dd_add_dd(t, dd{sh_hi[q], sh_lo[q]});
    return t.hi + t.lo;
}

// ---- SwiGLU gating with fixed arithmetic (shared by the stand-alone producer and the fused decode kernel) ----
// exp(t) in fp32 with every step fixed (no fused multiply-add: the library is compiled with
// contraction off): clamp to [-87, 88], n = round(t log2 e), two-constant reduction by ln 2, degree-6 Horner, scale
// by 2^n.  Relative error below 4e-7; what matters is that the steps, not a library, define the value.
__device__ inline float exp32(float t) {
    t = fminf(fmaxf(t, -87.0f), 88.0f);
    const float n = rintf(t * 1.44269504f);
    float r = t - n * 0.693359375f;
    r = r - n * -2.12194440e-4f;
    float p = 1.0f / 720.0f;
    p = p * r + 1.0f / 120.0f;
    p = p * r + 1.0f / 24.0f;
    p = p * r + 1.0f / 6.0f;
    p = p * r + 0.5f;
    p = p * r + 1.0f;
    p = p * r + 1.0f;
    return ldexpf(p, (int)n);
}

__device__ inline float swiglu_one(float gate, float up) {
    const float e = exp32(-gate);
    const float s = gate / (1.0f + e);                     // IEEE fp32 division
    return s * up;
}

// ---- 2-bit layout ---------------------------------------------------------------------------------
// Eq. (1)-(2) for one weight, given d = gamma + eps: the 2-bit two's-complement code.
__device__ inline uint32_t ternary_code2(float w, float d) {
    float q = w / d;                        // IEEE fp32 division
    float r = rintf(q);                     // ties to even
    r = fminf(1.0f, fmaxf(-1.0f, r));
    return ((uint32_t)(int)r) & 3u;         // -1 -> 0b11, 0 -> 0b00, +1 -> 0b01
}

// Eq. (1)-(2) without a division per weight.  For w > 0, RoundClip(w / d, -1, 1) = 1 exactly when the fp32
// quotient fl(w / d) exceeds 0.5 (a quotient of exactly 0.5 rounds to the even integer 0, anything from 1.5 up is
// clipped to 1), and fl(w / d) is monotone in w; so the code is +1 from a threshold T(d) upward, and by the
// odd symmetry of division and rounding -1 from -T downward.  T is found with the same fp32 division, starting
// at d / 2 (exactly 0.5 after the division) and stepping through neighbouring floats.
__device__ inline float ternary_threshold(float d) {
    float t = 0.5f * d;
#pragma unroll 1
    for (int i = 0; i < 8 && !(t / d > 0.5f); ++i) t = __uint_as_float(__float_as_uint(t) + 1u);
#pragma unroll 1
    for (int i = 0; i < 8 && (__uint_as_float(__float_as_uint(t) - 1u) / d > 0.5f); ++i)
        t = __uint_as_float(__float_as_uint(t) - 1u);
    return t;
}
__device__ inline uint32_t ternary_code2_threshold(float w, float t) {
    return w >= t ? 1u : (w <= -t ? 3u : 0u);           // +1 -> 0b01, -1 -> 0b11, 0 -> 0b00
}

// index of the quad holding row 16*rb + r, columns 64*kq .. 64*kq+63 (Kq quads per row, RB row blocks):
// steps of four quad columns are outermost, row blocks next, then the quad column and the row.
__host__ __device__ inline int64_t quad_index_2bit(int64_t kq, int64_t rb, int r, int64_t Kq, int64_t RB) {
    const int64_t s = kq >> 2, g = kq & 3;
    const int64_t nq = (Kq - 4 * s) < 4 ? (Kq - 4 * s) : 4;
    return 64 * RB * s + 16 * nq * rb + 16 * g + r;
}

// bit position of column c (0..15) inside its 32-bit word
__host__ __device__ inline int code_shift(int c) { return 8 * (c & 3) + 2 * (c >> 2); }

// sign-extend a 2-bit field to int
__device__ inline int code_value(uint32_t bits2) { return ((int)(bits2 << 30)) >> 30; }

}  // namespace bitnet

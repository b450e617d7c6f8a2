// Pieces shared by the weight-streaming BitLinear kernels (decode, M <= 16, and batched decode, M <= 64).
#pragma once
#include "bitnet_device.hpp"
#include "bitnet_internal.hpp"

namespace bitnet {

typedef int v4i __attribute__((ext_vector_type(4)));

// One packed word (16 codes) -> the four int8 operand registers of an MFMA, 64 * code in every byte:
// (w << (6 - 2 i)) & 0xC0C0C0C0 for register i.  The lane's validity is folded into the constant: km is
// 0xC0C0C0C0, or 0 for lanes and steps whose weights must not count.
__device__ inline v4i decode_word_masked(uint32_t w, uint32_t km) {
    v4i a;
    a.x = (int)((w << 6) & km);
    a.y = (int)((w << 4) & km);
    a.z = (int)((w << 2) & km);
    a.w = (int)(w & km);
    return a;
}

__device__ inline v4i as_v4i(const uint4& u) {
    v4i a;
    a.x = (int)u.x; a.y = (int)u.y; a.z = (int)u.z; a.w = (int)u.w;
    return a;
}

__device__ inline uint32_t quad_word(const uint4& q, int j) { return j == 0 ? q.x : j == 1 ? q.y : j == 2 ? q.z : q.w; }

// Pins the order of memory instructions for kernels that count loads in flight: nothing moves across
// it, neither in the optimizer nor in the instruction scheduler.
__device__ inline void issue_fence() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

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

}  // namespace bitnet

// The prefill kernel's K loop built up from an MFMA-only loop, one ingredient at a time, to see what each costs the
// matrix pipe: decode arithmetic, LDS operand reads, the barrier per K step, the weight loads from global memory, the
// LDS-DMA copies of the activations -- the last two either streaming through the L2 as in the product (the sixteen
// workgroups of a weight tile read the same 16 KB per step, the workgroups of a token tile the same 32 KB) or going to
// the same addresses every step (cache hits: the instructions without the traffic).  Registers, LDS and range-checked
// loads only; results are meaningless, rates are what is measured.  Measurement aid (libbitnet_floors.so); no entry
// point of the BitLinear library uses it.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// kValu: decode instructions per slice of eight MFMAs (0 or 16); kLds: ds_read_b128 per slice (0 or 4), one slice ahead;
// kBar: s_waitcnt + barrier per step of 64 MFMAs; kGlob: four 16-byte loads per lane and step, one step ahead; kDma: eight
// 1 KiB LDS-DMA copies per wave and step into the other stage; kHot: the loads and copies hit the same addresses every step
template <int kValu, int kLds, int kBar, int kGlob, int kDma, int kHot>
__global__ __launch_bounds__(256, 2) void ladder_kernel(const v4i* __restrict__ a_src, const v4i* __restrict__ b_src, int nvec, int steps,
                                                        const uint4* __restrict__ gsrc, int gvec, int* __restrict__ out) {
#if defined(__HIP_DEVICE_COMPILE__)
    extern __shared__ uint4 smem[];
    char* lds = reinterpret_cast<char*>(smem);
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    v16i acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
    const int t = (int)(blockIdx.x * 256 + threadIdx.x);
    for (int i = threadIdx.x; i < 4096; i += 256) smem[i] = *reinterpret_cast<const uint4*>(&a_src[(t + i * 7) % nvec]);   // two 32 KB stages
    __syncthreads();
    v4i a[2][4], b[2][2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int i = 0; i < 4; ++i) a[s][i] = a_src[(t * 8 + s * 4 + i) % nvec];
#pragma unroll
        for (int j = 0; j < 2; ++j) b[s][j] = b_src[(t * 4 + s * 2 + j) % nvec];
    }
    uint32_t wq[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) wq[i] = (uint32_t)b_src[(t * 8 + i) % nvec].x | 1u;
    uint4 gq[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) gq[i] = make_uint4(0, 0, 0, 0);
    const int am = lane & 31, kg = lane >> 5;
    const char* srcbase = lds + am * 256;
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4*>(gsrc), 0, gvec * 16, 0x00020000);
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    for (int st = 0; st < steps; ++st) {
        if (kBar) { __builtin_amdgcn_s_waitcnt(0); __syncthreads(); }
        const char* src = srcbase + (st & 1) * 32768;
        const size_t sa = kHot ? 0 : st;
        if (kGlob) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                wq[i] ^= gq[i].x ^ gq[i].z; wq[4 + i] ^= gq[i].y ^ gq[i].w;                          // consume the previous step's quads, request the next
                gq[i] = gsrc[(((size_t)(blockIdx.x >> 4) * steps + sa) * 1024 + i * 256 + threadIdx.x) % (size_t)gvec];
            }
        }
        if (kDma) {
#pragma unroll
            for (int c = 0; c < 8; ++c)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    xrsrc, (__attribute__((address_space(3))) void*)(lds + ((st + 1) & 1) * 32768 + (wave * 8 + c) * 1024), 16,
                    (uint32_t)(((((size_t)(blockIdx.x & 15) * steps + sa) * 32 + wave * 8 + c) * 1024 + lane * 16) % ((size_t)gvec * 16 - 1024)) & ~15u, 0, 0, 0);
        }
        v4i ar[2][4];
        if (kLds) {
#pragma unroll
            for (int fm = 0; fm < 4; ++fm) ar[0][fm] = *reinterpret_cast<const v4i*>(src + fm * 8192 + (((4 * kg) ^ (am & 15)) << 4));
        }
#pragma unroll
        for (int sl = 0; sl < 8; ++sl) {
            const int cur = sl & 1, nxt = cur ^ 1;
            __builtin_amdgcn_sched_barrier(0);
            if (kLds && sl < 7) {
                const int chunk = 8 * ((sl + 1) >> 2) + 4 * kg + ((sl + 1) & 3);
#pragma unroll
                for (int fm = 0; fm < 4; ++fm) ar[nxt][fm] = *reinterpret_cast<const v4i*>(src + fm * 8192 + ((chunk ^ (am & 15)) << 4));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int fm = q >> 1, fn = q & 1;
                const v4i av = kLds ? ar[cur][fm] : a[cur][fm];
                acc[fm][fn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av, b[cur][fn], acc[fm][fn], 0, 0, 0);
                if (kValu) {                                                   // the next slice's B operand: a shift and an AND per register
                    const int reg = q;
                    b[nxt][reg >> 2][reg & 3] = (int)((wq[(sl + reg) & 7] << (2 * (reg & 3))) & 0xC0C0C0C0u);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    const unsigned long long c1 = clock64(), w1 = wall_clock64();
    if (blockIdx.x == 7 && threadIdx.x == 0) { out[1] = (int)(c1 - c0); out[2] = (int)(w1 - w0); }   // shader clock / 100 MHz clock
    int sum = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) sum += acc[i][j][v];
#pragma unroll
    for (int i = 0; i < 8; ++i) sum += (int)wq[i];
    if (sum == 0x7fffffff) out[0] = sum;
#endif
}

template <int V, int L, int Bq, int G, int D, int H>
int ladder_go(const void* a, const void* b, long long bytes, int blocks, int steps, const void* g, long long gbytes, void* out, void* stream) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(ladder_kernel<V, L, Bq, G, D, H>), hipFuncAttributeMaxDynamicSharedMemorySize, 65536) != hipSuccess)
        return -2;
    hipLaunchKernelGGL((ladder_kernel<V, L, Bq, G, D, H>), dim3(blocks), dim3(256), 65536, (hipStream_t)stream, (const v4i*)a, (const v4i*)b,
                       (int)(bytes / 16), steps, (const uint4*)g, (int)(gbytes / 16), (int*)out);
    return (int)hipGetLastError();
}

}  // namespace

// What the L2s deliver into the CUs when nothing else is done: every workgroup (256 threads) reads the whole buffer -- small
// enough to stay in each XCD's L2, a power of two in size -- `reps` times from a place of its own, eight 16-byte loads per
// lane in flight, into registers or, as LDS-DMA copies, into 32 KB of LDS.  The prefill kernel takes 48 KB per 8.4 M
// multiply-adds this way; this is the rate that traffic can reach at most.
template <bool kToLds>
__global__ __launch_bounds__(256, 2) void l2_read_kernel(const uint4* __restrict__ p, int nvec, int reps, uint32_t* __restrict__ out) {
#if defined(__HIP_DEVICE_COMPILE__)
    extern __shared__ uint4 smem[];
    char* lds = reinterpret_cast<char*>(smem);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t mask = (uint32_t)nvec - 1u, rot = (blockIdx.x * 4099u + 17u) & mask;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4*>(p), 0, nvec * 16, 0x00020000);
    uint32_t acc = 0;
    for (int r = 0; r < reps; ++r) {
        for (uint32_t base = 0; base < (uint32_t)nvec; base += 256u * 8u) {
            if (kToLds) {
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)(lds + (wave * 8 + u) * 1024), 16,
                                                             ((base + u * 256u + threadIdx.x + rot) & mask) * 16u, 0, 0, 0);
            } else {
                uint4 q[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) q[u] = p[(base + u * 256u + threadIdx.x + rot) & mask];
#pragma unroll
                for (int u = 0; u < 8; ++u) acc += q[u].x ^ q[u].y ^ q[u].z ^ q[u].w;
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(0);
    if (kToLds) { __syncthreads(); acc = smem[threadIdx.x].x; }
    if (acc == 0x12345678u) out[0] = acc;
#endif
}

// bytes: a power of two from 64 KiB to 64 MiB; to_lds: 0 loads into registers, 1 LDS-DMA copies.  -3: arguments outside that.
extern "C" int l2_read_launch(const void* p, long long bytes, int reps, int blocks, int to_lds, void* out, void* stream) {
    if (!p || !out || bytes < (64ll << 10) || bytes > (64ll << 20) || (bytes & (bytes - 1)) || reps < 1 || blocks < 1) return -3;
    const int nvec = (int)(bytes / 16);
    if (to_lds) hipLaunchKernelGGL(l2_read_kernel<true>, dim3(blocks), dim3(256), 32768, (hipStream_t)stream, (const uint4*)p, nvec, reps, (uint32_t*)out);
    else hipLaunchKernelGGL(l2_read_kernel<false>, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const uint4*)p, nvec, reps, (uint32_t*)out);
    return (int)hipGetLastError();
}

// rung: 0 MFMAs only; 1 + barrier per step; 2 + decode arithmetic; 3 + LDS operand reads; 4 + weight loads (streaming); 5 + LDS-DMA
// copies (streaming) = every ingredient of the product's K loop; 6 as 4 and 7 as 5 with the same addresses every step; 8 barrier +
// weight loads only; 9 barrier + LDS-DMA copies only.  a, b: at least `bytes` of int8 operand data; g: at least gbytes (>= 64 MiB
// and below 2 GiB, one raw buffer) of anything.  out: four ints; out[1] / out[2] is the shader clock in units of 100 MHz.
// Returns -3 for arguments outside that and -1 for an unknown rung, both before anything is launched.
extern "C" int prefill_ladder_launch(int rung, const void* a, const void* b, long long bytes, int blocks, int steps, const void* g,
                                     long long gbytes, void* out, void* stream) {
    if (!a || !b || !g || !out || bytes < 16 || gbytes < (64ll << 20) || gbytes >= (2ll << 30) || steps < 1 || blocks < 1) return -3;
    switch (rung) {
        case 0: return ladder_go<0, 0, 0, 0, 0, 0>(a, b, bytes, blocks, steps, g, gbytes, out, stream);
        case 1: return ladder_go<0, 0, 1, 0, 0, 0>(a, b, bytes, blocks, steps, g, gbytes, out, stream);
        case 2: return ladder_go<16, 0, 1, 0, 0, 0>(a, b, bytes, blocks, steps, g, gbytes, out, stream);
        case 3: return ladder_go<16, 4, 1, 0, 0, 0>(a, b, bytes, blocks, steps, g, gbytes, out, stream);
        case 4: return ladder_go<16, 4, 1, 1, 0, 0>(a, b, bytes, blocks, steps, g, gbytes, out, stream);
        case 5: return ladder_go<16, 4, 1, 1, 1, 0>(a, b, bytes, blocks, steps, g, gbytes, out, stream);
        case 6: return ladder_go<16, 4, 1, 1, 0, 1>(a, b, bytes, blocks, steps, g, gbytes, out, stream);
        case 7: return ladder_go<16, 4, 1, 1, 1, 1>(a, b, bytes, blocks, steps, g, gbytes, out, stream);
        case 8: return ladder_go<0, 0, 1, 1, 0, 0>(a, b, bytes, blocks, steps, g, gbytes, out, stream);
        case 9: return ladder_go<0, 0, 1, 0, 1, 0>(a, b, bytes, blocks, steps, g, gbytes, out, stream);
    }
    return -1;
}

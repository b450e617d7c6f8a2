// A kernel that only reads: the floor under the decode launches (what the memory system gives a launch of a layer's packed
// size when nothing else is done).  Measurement aid, built into a library of its own (libbitnet_read_floor.so); no entry
// point of the BitLinear library uses it.
#include <hip/hip_runtime.h>
#include <stdint.h>
// every thread walks the buffer with a grid stride, kUnroll 16-byte loads in flight; the XOR keeps the loads alive
template <int kUnroll>
__global__ __launch_bounds__(512) void read_only(const uint4* __restrict__ p, int64_t nvec, uint32_t* __restrict__ out) {
    typedef unsigned v4u __attribute__((ext_vector_type(4)));
    const int64_t tid = (int64_t)blockIdx.x * 512 + threadIdx.x, nt = (int64_t)gridDim.x * 512;
    uint32_t acc = 0;
    int64_t i = tid;
    for (; i + (kUnroll - 1) * nt < nvec; i += kUnroll * nt) {
        v4u q[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) q[u] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p + i + u * nt));
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) acc += q[u].x ^ q[u].y ^ q[u].z ^ q[u].w;
    }
    for (; i < nvec; i += nt) { const uint4 q = p[i]; acc += q.x ^ q.y ^ q.z ^ q.w; }
    if (acc == 0x12345678u) out[0] = acc;
}
extern "C" int read_only_launch(const void* p, long long bytes, void* out, int blocks, int unroll, void* stream) {
    const int64_t nvec = bytes / 16;
    hipStream_t s = (hipStream_t)stream;
    if (unroll == 2) hipLaunchKernelGGL(read_only<2>, dim3(blocks), dim3(512), 0, s, (const uint4*)p, nvec, (uint32_t*)out);
    else if (unroll == 4) hipLaunchKernelGGL(read_only<4>, dim3(blocks), dim3(512), 0, s, (const uint4*)p, nvec, (uint32_t*)out);
    else hipLaunchKernelGGL(read_only<8>, dim3(blocks), dim3(512), 0, s, (const uint4*)p, nvec, (uint32_t*)out);
    return (int)hipGetLastError();
}

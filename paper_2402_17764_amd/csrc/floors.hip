// Two kernels that do one thing each, as yardsticks for the product kernels: one only reads a buffer (what the memory
// system gives a launch of a layer's packed size when nothing else is done), one only issues int8 MFMAs from registers
// (what the matrix pipe sustains on operands like the workload's, whose switching activity sets the clock).
// Measurement aids, built into a library of their own (libbitnet_floors.so); no entry point of the BitLinear library
// uses them.
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
// -3: a null pointer, no whole 16-byte vector, no workgroup (checked before anything is launched)
extern "C" int read_only_launch(const void* p, long long bytes, void* out, int blocks, int unroll, void* stream) {
    if (!p || !out || bytes < 16 || blocks < 1) return -3;
    const int64_t nvec = bytes / 16;
    hipStream_t s = (hipStream_t)stream;
    if (unroll == 2) hipLaunchKernelGGL(read_only<2>, dim3(blocks), dim3(512), 0, s, (const uint4*)p, nvec, (uint32_t*)out);
    else if (unroll == 4) hipLaunchKernelGGL(read_only<4>, dim3(blocks), dim3(512), 0, s, (const uint4*)p, nvec, (uint32_t*)out);
    else hipLaunchKernelGGL(read_only<8>, dim3(blocks), dim3(512), 0, s, (const uint4*)p, nvec, (uint32_t*)out);
    return (int)hipGetLastError();
}

// 4 x 2 accumulator fragments of v_mfma_i32_32x32x32_i8 per wave, as in the prefill kernel's 128 x 256 tile, and nothing
// else in the loop.  Each lane takes its eight A and eight B operand registers from the two buffers (16 bytes each, at
// lane-dependent places); the loop alternates between two sets of them so that operands switch as they do in a product.
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256, 2) void mfma_only(const v4i* __restrict__ a_src, const v4i* __restrict__ b_src, int nvec, int iters,
                                                    int* __restrict__ out) {
    v16i acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
    v4i a[2][4], b[2][2];
    const int t = (int)(blockIdx.x * 256 + threadIdx.x);
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int i = 0; i < 4; ++i) a[s][i] = a_src[(t * 8 + s * 4 + i) % nvec];
#pragma unroll
        for (int j = 0; j < 2; ++j) b[s][j] = b_src[(t * 4 + s * 2 + j) % nvec];
    }
    for (int it = 0; it < iters; it += 2) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[s][i], b[s][j], acc[i][j], 0, 0, 0);
    }
    int sum = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) sum += acc[i][j][v];
    if (sum == 0x7fffffff) out[0] = sum;
}
// iters (even) rounds of eight MFMAs per wave: 2 * 32 * 32 * 32 * 8 * iters operations per wave, four waves per workgroup
extern "C" int mfma_only_launch(const void* a_src, const void* b_src, long long bytes, int blocks, int iters, void* out, void* stream) {
    if (!a_src || !b_src || !out || bytes < 16 || blocks < 1 || iters < 1) return -3;
    hipLaunchKernelGGL(mfma_only, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const v4i*)a_src, (const v4i*)b_src, (int)(bytes / 16),
                       iters, (int*)out);
    return (int)hipGetLastError();
}

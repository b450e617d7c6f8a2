// bitnet_quantize_weights_static: bitnet_quantize_weights for callers that cannot allocate (code under HIP-graph
// capture, serving loops, harnesses that forbid hipMalloc) and so cannot provide its workspace.  The block partial
// sums of the |W| reduction (Eq. (3)) go to a static array in device memory instead; everything else -- the kernels,
// their launch shapes, the results -- is bitnet_quantize_weights'.
#include "bitnet.h"

#include "bitnet_internal.hpp"

#include <atomic>
#include <mutex>
#include <stdint.h>

namespace bitnet {

// 2048 (hi, lo) pairs of doubles: what bitnet_quantize_weights_workspace reports for any shape.  Each GPU the library
// runs on holds its own copy until the process ends.
constexpr size_t kStaticScratchBytes = 32768;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
std::mutex g_lock;
void* g_ptr[kMaxDevices] = {};                // device address of `scratch` on each device, once looked up
std::atomic<bool> g_have[kMaxDevices] = {};
}  // namespace

hipError_t static_scratch(void** ptr, size_t* bytes);

// The name `scratch` is only a handle in host code; its device address differs per GPU and comes from the runtime,
// looked up once per device with that device current.
hipError_t static_scratch(void** ptr, size_t* bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_have[dev].load(std::memory_order_acquire)) {
        std::lock_guard<std::mutex> hold(g_lock);
        if (!g_have[dev].load(std::memory_order_relaxed)) {
            void* p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return e;
            if (!p) return hipErrorInvalidSymbol;
            g_ptr[dev] = p;
            g_have[dev].store(true, std::memory_order_release);
        }
    }
    *ptr = g_ptr[dev];
    *bytes = kStaticScratchBytes;
    return hipSuccess;
}

}  // namespace bitnet

extern "C" bitnet_status bitnet_quantize_weights_static(const void* W, bitnet_dtype w_dtype, int64_t N, int64_t K,
                                                        bitnet_format f, void* packed, float* gamma, void* stream) {
    // the argument checks of bitnet_quantize_weights, before any device is touched: with an empty workspace it
    // validates everything else first and launches nothing
    void* const probe = reinterpret_cast<void*>(uintptr_t{256});
    const bitnet_status pre = bitnet_quantize_weights(W, w_dtype, N, K, f, packed, gamma, probe, 0, stream);
    if (pre != BITNET_ERR_WORKSPACE) return pre == BITNET_OK ? BITNET_ERR_WORKSPACE : pre;
    size_t need = 0;
    const bitnet_status q = bitnet_quantize_weights_workspace(N, K, &need);
    if (q != BITNET_OK) return q;
    if (need > bitnet::kStaticScratchBytes) return BITNET_ERR_WORKSPACE;   // partial sums beyond the static array
    void* ptr = nullptr;
    size_t have = 0;
    if (bitnet::static_scratch(&ptr, &have) != hipSuccess) return BITNET_ERR_HIP;
    return bitnet_quantize_weights(W, w_dtype, N, K, f, packed, gamma, ptr, have, stream);
}

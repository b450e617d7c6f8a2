// Host-side launch functions of the kernel translation units; called only by api.hip, which has
// already validated every argument.
#pragma once

#include <hip/hip_runtime.h>
#include <atomic>
#include <initializer_list>
#include <stdint.h>

namespace bitnet {

enum class OutType { F32 = 0, BF16 = 1, I32 = 2 };

// Raises a kernel's dynamic-LDS limit above the 64 KiB default, once per device and kernel (the attribute
// belongs to the function on the current device).  `done` is the caller's per-kernel flag array; the flags are
// atomic, so host threads that meet on a kernel's first use at worst both set the same attribute to the same value.
constexpr int kMaxDevices = 64;
using RaisedFlags = std::atomic<bool>[kMaxDevices];
inline hipError_t raise_dynamic_lds(const void* kernel, int bytes, RaisedFlags& done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (done[dev].load(std::memory_order_acquire)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done[dev].store(true, std::memory_order_release);
    return e;
}

// quant_weights.hip
int quant_weights_num_partials();
// nout: how many consecutive floats receive gamma (one per 16-row block of a segment; 1 for a whole tensor)
hipError_t launch_absmean_gamma(const void* W, bool bf16, int64_t N, int64_t K, float* gamma, void* workspace,
                                hipStream_t stream, int64_t nout = 1);
// rb_off / rb_total: the rows are row blocks rb_off ... of a packed matrix of rb_total row blocks (0: all of it)
hipError_t launch_quantize_weights_2bit(const void* W, bool bf16, int64_t N, int64_t K, void* packed,
                                        float* gamma, void* workspace, hipStream_t stream, int64_t rb_off = 0,
                                        int64_t rb_total = 0, int64_t nout = 1);

// one shard's share of Eq. (3): sum[0 .. 1] = the double-double (hi, lo) pair of sum |W| over these rows
hipError_t launch_abs_sum(const void* W, bool bf16, int64_t N, int64_t K, double* sum, void* workspace, hipStream_t stream);
// how many (hi, lo) pairs the packing pass can fold (one per thread of a workgroup)
int quant_weights_max_sums();
// gamma = fp32((sum of the nsums pairs) / total_count), Eq. (3) over all shards
hipError_t launch_gamma_from_sums(const double* sums, int nsums, int64_t total_count, float* gamma, hipStream_t stream);
// Eq. (1)-(2) + packing of these rows with that gamma (written to *gamma as well)
hipError_t launch_pack_2bit_with_sums(const void* W, bool bf16, int64_t N, int64_t K, const double* sums, int nsums,
                                      int64_t total_count, void* packed, float* gamma, hipStream_t stream);

// quant_acts.hip
hipError_t launch_quantize_acts(const void* x, bool bf16, int64_t M, int64_t K, int8_t* xq, float* sx,
                                hipStream_t stream);

hipError_t launch_rmsnorm_quantize(const void* x, bool bf16, const float* g, float eps, int64_t M, int64_t K,
                                   int8_t* xq, float* sx, hipStream_t stream);
hipError_t launch_swiglu_quantize(const void* gu, bool bf16, int64_t M, int64_t F, int8_t* hq, float* sh,
                                  hipStream_t stream);

// linear_ref.hip
// gstride (all product launchers): 0 = gamma is one float, 1 = gamma[rb] is the scale of 16-row block rb
hipError_t launch_linear_reference_2bit(const int8_t* xq, const float* sx, const void* packed,
                                        const float* gamma, int gstride, int64_t M, int64_t N, int64_t K, void* y,
                                        OutType yt, hipStream_t stream);
hipError_t launch_unpack_2bit(const void* packed, int64_t N, int64_t K, int8_t* codes, hipStream_t stream);

// What a launcher would do.  Every bitnet_linear launcher takes an optional LaunchPlan*: when it is given, the
// launcher fills it in and returns without touching the device or its pointer arguments (bitnet_linear_describe).
struct LaunchPlan {
    const char* kernel = "";          // which kernel family
    int params[6] = {0, 0, 0, 0, 0, 0};  // template parameters of the instantiation, in declaration order
    int nparams = 0;
    unsigned grid_x = 0, grid_y = 1, block = 0;
    size_t lds_bytes = 0;
    int splits = 1;                   // > 1: split-K, a second launch adds the partials
    void set(const char* k, std::initializer_list<int> p, unsigned gx, unsigned gy, unsigned b, size_t lds, int sp) {
        kernel = k; nparams = 0;
        for (int v : p) params[nparams++] = v;
        grid_x = gx; grid_y = gy; block = b; lds_bytes = lds; splits = sp;
    }
};

// linear_gemv.hip
bool gemv_supports(int64_t M, int64_t N, int64_t K, const void* xq);
// workspace (may be null) and force_splits as for launch_linear_gemm_2bit: split-K of the batched-decode kernels
// (4 < M <= 64); never taken by itself at present (skinny_splitk_splits() is 1 for every shape)
int skinny_splitk_splits(int64_t M, int64_t N, int64_t K);
hipError_t launch_linear_gemv_2bit(const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                                   int gstride, int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream,
                                   void* workspace = nullptr, size_t workspace_bytes = 0, int force_splits = 0,
                                   LaunchPlan* plan = nullptr);
// the M <= 16 kernel alone (linear_gemv.hip); launch_linear_gemv_2bit (linear_skinny.hip) routes M <= 4 to it
hipError_t launch_linear_gemv16_2bit(const int8_t* xq, const float* sx, const void* packed, const float* gamma, int gstride,
                                     int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream, LaunchPlan* plan = nullptr);
bool gemv_fused_supports(int64_t M, int64_t N, int64_t K, const void* x);
hipError_t launch_linear_fused_2bit(const void* x, bool bf16, const void* packed, const float* gamma, int gstride,
                                    int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream,
                                    LaunchPlan* plan = nullptr);
// the same with RMSNorm (optional per-column gain, 16-byte aligned) in front of the quantization
hipError_t launch_rmsnorm_linear_fused_2bit(const void* x, bool bf16, const float* gain, float eps, const void* packed,
                                            const float* gamma, int gstride, int64_t M, int64_t N, int64_t K, void* y,
                                            OutType yt, hipStream_t stream, LaunchPlan* plan = nullptr);
// ... and with SwiGLU gating in front: gu is [M][2 K] (gate | up), the product runs over K columns
hipError_t launch_swiglu_linear_fused_2bit(const void* gu, bool bf16, const void* packed, const float* gamma, int gstride,
                                           int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream,
                                           LaunchPlan* plan = nullptr);
// merged gate | up projection ([2 F][K], F a multiple of 16) from x (absmax quantization, RMSNorm first if `norm`),
// h = silu(y_gate) * y_up stored as [M][F] (F32 or BF16)
hipError_t launch_linear_fused_swiglu_out_2bit(const void* x, bool bf16, bool norm, const float* gain, float eps,
                                               const void* packed, const float* gamma, int gstride, int64_t M, int64_t F,
                                               int64_t K, void* h, OutType yt, hipStream_t stream,
                                               LaunchPlan* plan = nullptr);

// linear_gemm.hip
bool gemm_supports(int64_t M, int64_t N, int64_t K, const void* xq);
// workspace (may be null): room for split-K partials; force_splits > 0 picks the number of splits (1, 2, 4, 8) by hand
hipError_t launch_linear_gemm_2bit(const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                                   int gstride, int64_t M, int64_t N, int64_t K, void* y, OutType yt,
                                   hipStream_t stream, void* workspace = nullptr, size_t workspace_bytes = 0,
                                   int force_splits = 0, LaunchPlan* plan = nullptr);
// the same with the tile forced: 32 * fm tokens x 128 * fn weight rows, fm in 2 .. 4, fn in 1 .. 2, kg = 1, or kg = 2 (eight waves in
// two K groups) with (fm, fn) = (3, 1) or (2, 2) and one split, or kg = 3 (eight waves in two row groups: tiles of 128 x 512)
// with (fm, fn) = (4, 2) (hipErrorInvalidValue otherwise); splits > 1 needs a workspace of splitk_workspace_bytes(M, N, splits)
hipError_t launch_linear_gemm_2bit_shape(int fm, int fn, int kg, const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                                         int gstride, int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream,
                                         int splits = 1, void* workspace = nullptr, LaunchPlan* plan = nullptr);
size_t splitk_workspace_bytes(int64_t M, int64_t N, int splits);
// split-K, second launch: y = (sum of `splits` int32 partial accumulators, [M][N] each) * gamma * s_x / 127;
// prefill_assoc: the association of the prefill kernel's per-block-gamma epilogue (gamma * (s_x / 127)) instead of
// the decode kernels' ((gamma * s_x) / 127)
hipError_t launch_splitk_reduce(const int32_t* part, int splits, const float* sx, const float* gamma, int gstride,
                                int prefill_assoc, int64_t M, int64_t N, void* y, OutType yt, hipStream_t stream);

// trit5.hip
hipError_t launch_pack_trit5(const void* W, bool bf16, int64_t N, int64_t K, const float* gamma, void* packed,
                             hipStream_t stream);
hipError_t launch_unpack_trit5(const void* packed, int64_t N, int64_t K, int8_t* codes, hipStream_t stream);
hipError_t launch_linear_reference_trit5(const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                                         int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream);
// the same matrix in the other packing format (in_trit5: 5-trit -> 2-bit, else 2-bit -> 5-trit)
hipError_t launch_repack(const void* in, bool in_trit5, int64_t N, int64_t K, void* out, hipStream_t stream);
bool gemv_trit5_supports(int64_t M, int64_t N, int64_t K, const void* xq);
hipError_t launch_linear_gemv_trit5(const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                                    int64_t M, int64_t N, int64_t K, void* y, OutType yt, hipStream_t stream);

}  // namespace bitnet

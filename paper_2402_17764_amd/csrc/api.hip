// C ABI of the BitLinear library (declared in include/bitnet.h): argument validation on the host,
// then dispatch to the kernel launchers.  Nothing is allocated and no state is kept here.
#include "bitnet.h"

#include "bitnet_device.hpp"
#include "bitnet_internal.hpp"

#include <stdio.h>
#include <string.h>

namespace {

using bitnet::OutType;

constexpr int64_t kMaxElems = (int64_t)1 << 40;
constexpr int64_t kMaxK = 262144;

inline bool aligned(const void* p, size_t a) { return reinterpret_cast<uintptr_t>(p) % a == 0; }

inline bool shape_ok(int64_t M, int64_t N, int64_t K) {
    if (M <= 0 || N <= 0 || K <= 0) return false;
    if (K > kMaxK || M >= ((int64_t)1 << 31) || N >= ((int64_t)1 << 31)) return false;
    if (N > kMaxElems / K || M > kMaxElems / K || M > kMaxElems / N) return false;
    return true;
}

inline bool format_ok(bitnet_format f) { return f == BITNET_PACK_2BIT || f == BITNET_PACK_TRIT5; }

inline size_t dtype_size(bitnet_dtype t) { return t == BITNET_BF16 ? 2 : 4; }

inline bitnet_status from_hip(hipError_t e) { return e == hipSuccess ? BITNET_OK : BITNET_ERR_HIP; }

bool out_type(bitnet_dtype t, OutType* o) {
    switch (t) {
        case BITNET_F32: *o = OutType::F32; return true;
        case BITNET_BF16: *o = OutType::BF16; return true;
        case BITNET_I32: *o = OutType::I32; return true;
        default: break;
    }
    return false;
}

}  // namespace

extern "C" {

int bitnet_version(void) { return 100; }

const char* bitnet_status_string(bitnet_status s) {
    switch (s) {
        case BITNET_OK: return "ok";
        case BITNET_ERR_NULL: return "null pointer";
        case BITNET_ERR_SHAPE: return "bad shape";
        case BITNET_ERR_DTYPE: return "unsupported dtype";
        case BITNET_ERR_FORMAT: return "unsupported packing format";
        case BITNET_ERR_ALIGN: return "misaligned pointer";
        case BITNET_ERR_WORKSPACE: return "workspace too small";
        case BITNET_ERR_HIP: return "HIP launch failed";
        case BITNET_ERR_KERNEL: return "kernel variant cannot run this shape";
        default: break;
    }
    return "unknown status";
}

bitnet_status bitnet_packed_bytes(int64_t N, int64_t K, bitnet_format f, size_t* bytes) {
    if (!bytes) return BITNET_ERR_NULL;
    if (!shape_ok(1, N, K)) return BITNET_ERR_SHAPE;
    const int64_t Np = 16 * bitnet::ceil_div(N, 16);
    if (f == BITNET_PACK_2BIT) {
        *bytes = (size_t)(Np * (64 * bitnet::ceil_div(K, 64)) / 4);
        return BITNET_OK;
    }
    if (f == BITNET_PACK_TRIT5) {
        *bytes = (size_t)(Np * (320 * bitnet::ceil_div(K, 320)) / 5);
        return BITNET_OK;
    }
    return BITNET_ERR_FORMAT;
}

bitnet_status bitnet_quantize_weights_workspace(int64_t N, int64_t K, size_t* bytes) {
    if (!bytes) return BITNET_ERR_NULL;
    if (!shape_ok(1, N, K)) return BITNET_ERR_SHAPE;
    *bytes = (size_t)bitnet::quant_weights_num_partials() * 2 * sizeof(double);
    return BITNET_OK;
}

bitnet_status bitnet_quantize_weights(const void* W, bitnet_dtype w_dtype, int64_t N, int64_t K,
                                      bitnet_format f, void* packed, float* gamma, void* workspace,
                                      size_t workspace_bytes, void* stream) {
    if (!W || !packed || !gamma || !workspace) return BITNET_ERR_NULL;
    if (!shape_ok(1, N, K)) return BITNET_ERR_SHAPE;
    if (w_dtype != BITNET_F32 && w_dtype != BITNET_BF16) return BITNET_ERR_DTYPE;
    if (!format_ok(f)) return BITNET_ERR_FORMAT;
    if (!aligned(W, dtype_size(w_dtype)) || !aligned(packed, 16) || !aligned(gamma, 4) || !aligned(workspace, 16))
        return BITNET_ERR_ALIGN;
    size_t need = 0;
    bitnet_quantize_weights_workspace(N, K, &need);
    if (workspace_bytes < need) return BITNET_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (f == BITNET_PACK_2BIT)
        return from_hip(bitnet::launch_quantize_weights_2bit(W, w_dtype == BITNET_BF16, N, K, packed, gamma, workspace, s));
    hipError_t e = bitnet::launch_absmean_gamma(W, w_dtype == BITNET_BF16, N, K, gamma, workspace, s);
    if (e != hipSuccess) return BITNET_ERR_HIP;
    return from_hip(bitnet::launch_pack_trit5(W, w_dtype == BITNET_BF16, N, K, gamma, packed, s));
}

bitnet_status bitnet_abs_sum(const void* W, bitnet_dtype w_dtype, int64_t N, int64_t K, double* sum, void* workspace,
                             size_t workspace_bytes, void* stream) {
    if (!W || !sum || !workspace) return BITNET_ERR_NULL;
    if (!shape_ok(1, N, K)) return BITNET_ERR_SHAPE;
    if (w_dtype != BITNET_F32 && w_dtype != BITNET_BF16) return BITNET_ERR_DTYPE;
    if (!aligned(W, dtype_size(w_dtype)) || !aligned(sum, 8) || !aligned(workspace, 16)) return BITNET_ERR_ALIGN;
    size_t need = 0;
    bitnet_quantize_weights_workspace(N, K, &need);
    if (workspace_bytes < need) return BITNET_ERR_WORKSPACE;
    return from_hip(bitnet::launch_abs_sum(W, w_dtype == BITNET_BF16, N, K, sum, workspace, static_cast<hipStream_t>(stream)));
}

bitnet_status bitnet_quantize_weights_sharded(const void* W, bitnet_dtype w_dtype, int64_t N, int64_t K, bitnet_format f,
                                              const double* sums, int nsums, int64_t total_rows, void* packed,
                                              float* gamma, void* stream) {
    if (!W || !sums || !packed || !gamma) return BITNET_ERR_NULL;
    if (!shape_ok(1, N, K) || nsums <= 0 || nsums > bitnet::quant_weights_max_sums() || total_rows < N ||
        !shape_ok(1, total_rows, K))
        return BITNET_ERR_SHAPE;
    if (w_dtype != BITNET_F32 && w_dtype != BITNET_BF16) return BITNET_ERR_DTYPE;
    if (!format_ok(f)) return BITNET_ERR_FORMAT;
    if (!aligned(W, dtype_size(w_dtype)) || !aligned(packed, 16) || !aligned(gamma, 4) || !aligned(sums, 8))
        return BITNET_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool bf16 = w_dtype == BITNET_BF16;
    if (f == BITNET_PACK_2BIT)
        return from_hip(bitnet::launch_pack_2bit_with_sums(W, bf16, N, K, sums, nsums, total_rows * K, packed, gamma, s));
    if (bitnet::launch_gamma_from_sums(sums, nsums, total_rows * K, gamma, s) != hipSuccess) return BITNET_ERR_HIP;
    return from_hip(bitnet::launch_pack_trit5(W, bf16, N, K, gamma, packed, s));
}

bitnet_status bitnet_quantize_acts(const void* x, bitnet_dtype x_dtype, int64_t M, int64_t K, int8_t* xq,
                                   float* sx, void* stream) {
    if (!x || !xq || !sx) return BITNET_ERR_NULL;
    if (!shape_ok(M, 1, K)) return BITNET_ERR_SHAPE;
    if (x_dtype != BITNET_F32 && x_dtype != BITNET_BF16) return BITNET_ERR_DTYPE;
    if (!aligned(x, dtype_size(x_dtype)) || !aligned(sx, 4)) return BITNET_ERR_ALIGN;
    return from_hip(bitnet::launch_quantize_acts(x, x_dtype == BITNET_BF16, M, K, xq, sx,
                                                 static_cast<hipStream_t>(stream)));
}

bitnet_status bitnet_rmsnorm_quantize(const void* x, bitnet_dtype x_dtype, const float* g, float eps, int64_t M,
                                      int64_t K, int8_t* xq, float* sx, void* stream) {
    if (!x || !xq || !sx) return BITNET_ERR_NULL;
    if (!shape_ok(M, 1, K) || !(eps >= 0.0f)) return BITNET_ERR_SHAPE;
    if (x_dtype != BITNET_F32 && x_dtype != BITNET_BF16) return BITNET_ERR_DTYPE;
    if (!aligned(x, dtype_size(x_dtype)) || !aligned(sx, 4) || (g && !aligned(g, 4))) return BITNET_ERR_ALIGN;
    return from_hip(bitnet::launch_rmsnorm_quantize(x, x_dtype == BITNET_BF16, g, eps, M, K, xq, sx,
                                                    static_cast<hipStream_t>(stream)));
}

bitnet_status bitnet_swiglu_quantize(const void* gu, bitnet_dtype gu_dtype, int64_t M, int64_t F, int8_t* hq,
                                     float* sh, void* stream) {
    if (!gu || !hq || !sh) return BITNET_ERR_NULL;
    if (F <= 0 || F > kMaxK / 2 || !shape_ok(M, 1, 2 * F)) return BITNET_ERR_SHAPE;
    if (gu_dtype != BITNET_F32 && gu_dtype != BITNET_BF16) return BITNET_ERR_DTYPE;
    if (!aligned(gu, dtype_size(gu_dtype)) || !aligned(sh, 4)) return BITNET_ERR_ALIGN;
    return from_hip(bitnet::launch_swiglu_quantize(gu, gu_dtype == BITNET_BF16, M, F, hq, sh,
                                                   static_cast<hipStream_t>(stream)));
}

static bitnet_status linear_any(const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                                int gstride, int64_t M, int64_t N, int64_t K, bitnet_format f, void* y,
                                bitnet_dtype y_dtype, bitnet_kernel which, void* stream) {
    if (!xq || !sx || !packed || !gamma || !y) return BITNET_ERR_NULL;
    if (!shape_ok(M, N, K)) return BITNET_ERR_SHAPE;
    OutType yt;
    if (!out_type(y_dtype, &yt)) return BITNET_ERR_DTYPE;
    if (!format_ok(f)) return BITNET_ERR_FORMAT;
    if (!aligned(packed, 16) || !aligned(sx, 4) || !aligned(gamma, 4) || !aligned(y, dtype_size(y_dtype)))
        return BITNET_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);

    if (f == BITNET_PACK_TRIT5) {
        if (gstride) return BITNET_ERR_FORMAT;         // per-segment scales exist for the 2-bit format only
        // the 5-trit format has the reference kernel and the weight-streaming kernel for M <= 16; more tokens
        // are walked 16 at a time (the weights are streamed once per group: a storage format, not a prefill one)
        if (which == BITNET_KERNEL_AUTO && M > 16 && bitnet::gemv_trit5_supports(16, N, K, xq)) {
            const size_t ysz = dtype_size(y_dtype);
            for (int64_t m0 = 0; m0 < M; m0 += 16) {
                const int64_t mc = M - m0 < 16 ? M - m0 : 16;
                const hipError_t e = bitnet::launch_linear_gemv_trit5(xq + m0 * K, sx + m0, packed, gamma, mc, N, K,
                                                                      static_cast<char*>(y) + m0 * N * ysz, yt, s);
                if (e != hipSuccess) return BITNET_ERR_HIP;
            }
            return BITNET_OK;
        }
        if (which == BITNET_KERNEL_AUTO)
            which = bitnet::gemv_trit5_supports(M, N, K, xq) ? BITNET_KERNEL_GEMV : BITNET_KERNEL_REFERENCE;
        if (which == BITNET_KERNEL_REFERENCE)
            return from_hip(bitnet::launch_linear_reference_trit5(xq, sx, packed, gamma, M, N, K, y, yt, s));
        if (which == BITNET_KERNEL_GEMV && bitnet::gemv_trit5_supports(M, N, K, xq))
            return from_hip(bitnet::launch_linear_gemv_trit5(xq, sx, packed, gamma, M, N, K, y, yt, s));
        return BITNET_ERR_KERNEL;
    }

    if (which == BITNET_KERNEL_AUTO) {
        if (bitnet::gemv_supports(M, N, K, xq)) which = BITNET_KERNEL_GEMV;
        else if (bitnet::gemm_supports(M, N, K, xq)) which = BITNET_KERNEL_GEMM;
        else which = BITNET_KERNEL_REFERENCE;
    }
    if (((int)which & ~0xFF) == 0x100) {               // prefill kernel, tile forced: 0x100 | two K groups << 7 | fm << 4 | fn
        const int fm = ((int)which >> 4) & 0x7, fn = (int)which & 0x7, wide = ((int)which >> 3) & 1;
        const int kg = wide ? 3 : 1 + (((int)which >> 7) & 1);          // 2: two K groups, 3: two row groups
        if (fm < 2 || fm > 4 || fn < 1 || fn > 2 || !bitnet::gemm_supports(M, N, K, xq)) return BITNET_ERR_KERNEL;
        if (kg == 2 && !((fm == 3 && fn == 1) || (fm == 2 && fn == 2))) return BITNET_ERR_KERNEL;
        if (wide && (fn != 2 || fm != 4 || (((int)which >> 7) & 1))) return BITNET_ERR_KERNEL;
        return from_hip(bitnet::launch_linear_gemm_2bit_shape(fm, fn, kg, xq, sx, packed, gamma, gstride, M, N, K, y, yt, s));
    }
    switch (which) {
        case BITNET_KERNEL_REFERENCE:
            return from_hip(bitnet::launch_linear_reference_2bit(xq, sx, packed, gamma, gstride, M, N, K, y, yt, s));
        case BITNET_KERNEL_GEMV:
            if (!bitnet::gemv_supports(M, N, K, xq)) return BITNET_ERR_KERNEL;
            return from_hip(bitnet::launch_linear_gemv_2bit(xq, sx, packed, gamma, gstride, M, N, K, y, yt, s));
        case BITNET_KERNEL_GEMM:
            if (!bitnet::gemm_supports(M, N, K, xq)) return BITNET_ERR_KERNEL;
            return from_hip(bitnet::launch_linear_gemm_2bit(xq, sx, packed, gamma, gstride, M, N, K, y, yt, s));
        default:
            return BITNET_ERR_KERNEL;
    }
}

bitnet_status bitnet_linear_variant(const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                                    int64_t M, int64_t N, int64_t K, bitnet_format f, void* y,
                                    bitnet_dtype y_dtype, bitnet_kernel which, void* stream) {
    return linear_any(xq, sx, packed, gamma, 0, M, N, K, f, y, y_dtype, which, stream);
}

bitnet_status bitnet_linear(const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                            int64_t M, int64_t N, int64_t K, bitnet_format f, void* y, bitnet_dtype y_dtype,
                            void* stream) {
    return linear_any(xq, sx, packed, gamma, 0, M, N, K, f, y, y_dtype, BITNET_KERNEL_AUTO, stream);
}

bitnet_status bitnet_linear_workspace(int64_t M, int64_t N, int64_t K, size_t* bytes) {
    if (!bytes) return BITNET_ERR_NULL;
    if (!shape_ok(M, N, K)) return BITNET_ERR_SHAPE;
    // prefill kernel: split-K is considered only where even 64 x 128 tiles leave workgroup slots empty (fewer than
    // 512 of them); the batched-decode kernels split only when forced
    const int64_t tiles = ((M + 63) / 64) * ((N + 127) / 128);
    const int skinny_splits = bitnet::skinny_splitk_splits(M, N, K);
    // (the batched-decode kernels serve up to 256 tokens on small layers; x_q is assumed aligned here)
    if (K % 16 != 0) *bytes = 0;                       // the reference kernel runs such shapes
    else if (bitnet::gemv_supports(M, N, K, nullptr)) *bytes = skinny_splits > 1 ? bitnet::splitk_workspace_bytes(M, N, skinny_splits) : 0;
    else *bytes = tiles < 512 ? bitnet::splitk_workspace_bytes(M, N, 8) : 0;
    return BITNET_OK;
}

// bytes of a 2-bit copy of the matrix, rounded up so that what follows it in a workspace stays 256-byte aligned
static size_t repacked_bytes(int64_t N, int64_t K) {
    size_t b = 0;
    bitnet_packed_bytes(N, K, BITNET_PACK_2BIT, &b);
    return (b + 255) / 256 * 256;
}

bitnet_status bitnet_linear_workspace_format(int64_t M, int64_t N, int64_t K, bitnet_format f, size_t* bytes) {
    if (!format_ok(f)) return BITNET_ERR_FORMAT;
    const bitnet_status st = bitnet_linear_workspace(M, N, K, bytes);
    if (st != BITNET_OK || f == BITNET_PACK_2BIT) return st;
    // 5-trit weights and more than 16 tokens: room for the matrix repacked to 2 bits, plus what the 2-bit path may use
    if (M > 16 && K % 16 == 0) *bytes += repacked_bytes(N, K);
    else *bytes = 0;
    return BITNET_OK;
}

bitnet_status bitnet_linear_ws(const int8_t* xq, const float* sx, const void* packed, const float* gamma,
                               int gamma_per_block, int64_t M, int64_t N, int64_t K, bitnet_format f, void* y,
                               bitnet_dtype y_dtype, bitnet_kernel which, void* workspace, size_t workspace_bytes,
                               void* stream) {
    const int gstride = gamma_per_block ? 1 : 0;
    if (f == BITNET_PACK_TRIT5 && which == BITNET_KERNEL_AUTO && !gamma_per_block && workspace && shape_ok(M, N, K) && M > 16 &&
        K % 16 == 0 && workspace_bytes >= repacked_bytes(N, K)) {
        // 5-trit weights at prefill sizes: one pass repacks the matrix to the 2-bit layout at the head of the workspace
        // (0.45 bytes per weight of traffic, against 2 M operations per weight of product), then the 2-bit kernels run
        // on it with the rest of the workspace.  Everything is validated before that first launch.
        if (!xq || !sx || !packed || !gamma || !y) return BITNET_ERR_NULL;
        OutType yt0;
        if (!out_type(y_dtype, &yt0)) return BITNET_ERR_DTYPE;
        if (!aligned(packed, 16) || !aligned(workspace, 16) || !aligned(sx, 4) || !aligned(gamma, 4) || !aligned(y, dtype_size(y_dtype)))
            return BITNET_ERR_ALIGN;
        const size_t head = repacked_bytes(N, K);
        if (bitnet::launch_repack(packed, true, N, K, workspace, static_cast<hipStream_t>(stream)) != hipSuccess) return BITNET_ERR_HIP;
        return bitnet_linear_ws(xq, sx, workspace, gamma, 0, M, N, K, BITNET_PACK_2BIT, y, y_dtype, BITNET_KERNEL_AUTO,
                                workspace_bytes > head ? static_cast<char*>(workspace) + head : nullptr, workspace_bytes - head, stream);
    }
    int force = 0;
    if (((int)which & ~0xFF) == 0x200) {               // split-K forced: 0x200 | splits
        force = (int)which & 0xFF;
        if (force != 2 && force != 4 && force != 8) return BITNET_ERR_KERNEL;
    } else if (which != BITNET_KERNEL_AUTO) {
        return linear_any(xq, sx, packed, gamma, gstride, M, N, K, f, y, y_dtype, which, stream);
    }
    if (!xq || !sx || !packed || !gamma || !y) return BITNET_ERR_NULL;
    if (!shape_ok(M, N, K)) return BITNET_ERR_SHAPE;
    if (workspace && !aligned(workspace, 16)) return BITNET_ERR_ALIGN;
    // a forced split runs on the kernel family the automatic choice would take for this shape: the batched-decode
    // kernels from 5 tokens on where they serve it, the prefill kernel otherwise (the M <= 4 decode kernel has no split form)
    const bool skinny_path = f == BITNET_PACK_2BIT && M > 4 && bitnet::gemv_supports(M, N, K, xq) &&
                             (force || (workspace && bitnet::skinny_splitk_splits(M, N, K) > 1));
    const bool gemm_path = f == BITNET_PACK_2BIT && !skinny_path && (force || !bitnet::gemv_supports(M, N, K, xq)) &&
                           bitnet::gemm_supports(M, N, K, xq);
    if (!gemm_path && !skinny_path) {
        if (force) return BITNET_ERR_KERNEL;
        return linear_any(xq, sx, packed, gamma, gstride, M, N, K, f, y, y_dtype, BITNET_KERNEL_AUTO, stream);
    }
    OutType yt;
    if (!out_type(y_dtype, &yt)) return BITNET_ERR_DTYPE;
    if (!aligned(packed, 16) || !aligned(sx, 4) || !aligned(gamma, 4) || !aligned(y, dtype_size(y_dtype))) return BITNET_ERR_ALIGN;
    if (force && (!workspace || workspace_bytes < bitnet::splitk_workspace_bytes(M, N, force) || force > (K + 255) / 256))
        return BITNET_ERR_WORKSPACE;
    if (skinny_path)
        return from_hip(bitnet::launch_linear_gemv_2bit(xq, sx, packed, gamma, gstride, M, N, K, y, yt, static_cast<hipStream_t>(stream),
                                                        workspace, workspace ? workspace_bytes : 0, force));
    return from_hip(bitnet::launch_linear_gemm_2bit(xq, sx, packed, gamma, gstride, M, N, K, y, yt, static_cast<hipStream_t>(stream),
                                                    workspace, workspace ? workspace_bytes : 0, force));
}

static bitnet_status plan_to_text(const bitnet::LaunchPlan& plan, char* text, size_t text_bytes) {
    char params[96] = "";
    size_t at = 0;
    for (int i = 0; i < plan.nparams && at < sizeof(params) - 16; ++i)
        at += (size_t)snprintf(params + at, sizeof(params) - at, i ? ",%d" : "%d", plan.params[i]);
    const int n = snprintf(text, text_bytes, "kernel=%s params=%s grid=%ux%u block=%u lds=%zu splits=%d", plan.kernel, params,
                           plan.grid_x, plan.grid_y, plan.block, plan.lds_bytes, plan.splits);
    return (n < 0 || (size_t)n >= text_bytes) ? BITNET_ERR_WORKSPACE : BITNET_OK;
}

bitnet_status bitnet_linear_describe(int64_t M, int64_t N, int64_t K, bitnet_format f, size_t workspace_bytes,
                                     char* text, size_t text_bytes) {
    if (!text || text_bytes == 0) return BITNET_ERR_NULL;
    text[0] = 0;
    if (!shape_ok(M, N, K)) return BITNET_ERR_SHAPE;
    if (!format_ok(f)) return BITNET_ERR_FORMAT;
    // the launchers read nothing through their pointers when they are given a plan: stand-ins with the alignment
    // the fast kernels ask for
    const int8_t* xq = reinterpret_cast<const int8_t*>(uintptr_t{256});
    const float* fp = reinterpret_cast<const float*>(uintptr_t{256});
    void* vp = reinterpret_cast<void*>(uintptr_t{256});
    void* ws = workspace_bytes ? vp : nullptr;
    bitnet::LaunchPlan plan;
    if (f == BITNET_PACK_TRIT5 && M > 16 && K % 16 == 0 && workspace_bytes >= repacked_bytes(N, K)) {
        // bitnet_linear_ws repacks to 2 bits at the head of the workspace and runs the 2-bit path on the rest
        const bitnet_status st = bitnet_linear_describe(M, N, K, BITNET_PACK_2BIT, workspace_bytes - repacked_bytes(N, K), text, text_bytes);
        if (st != BITNET_OK) return st;
        const size_t at = strlen(text);
        const int n = snprintf(text + at, text_bytes - at, " repack=trit5_to_2bit");
        return (n < 0 || (size_t)n >= text_bytes - at) ? BITNET_ERR_WORKSPACE : BITNET_OK;
    }
    if (f == BITNET_PACK_TRIT5) {
        plan.kernel = bitnet::gemv_trit5_supports(M < 16 ? M : 16, N, K, xq) ? "trit5_decode" : "trit5_reference";
    } else if (bitnet::gemv_supports(M, N, K, xq)) {
        const hipError_t e = bitnet::launch_linear_gemv_2bit(xq, fp, vp, fp, 0, M, N, K, vp, OutType::BF16, nullptr, ws, workspace_bytes,
                                                            0, &plan);
        if (e != hipSuccess) return BITNET_ERR_HIP;
    } else if (bitnet::gemm_supports(M, N, K, xq)) {
        const hipError_t e = bitnet::launch_linear_gemm_2bit(xq, fp, vp, fp, 0, M, N, K, vp, OutType::BF16, nullptr, ws, workspace_bytes,
                                                            0, &plan);
        if (e != hipSuccess) return BITNET_ERR_HIP;
    } else {
        plan.kernel = "reference";
    }
    return plan_to_text(plan, text, text_bytes);
}

bitnet_status bitnet_entry_describe(bitnet_entry entry, bitnet_dtype x_dtype, int64_t M, int64_t N, int64_t K,
                                    bitnet_format f, size_t workspace_bytes, char* text, size_t text_bytes) {
    if (entry == BITNET_ENTRY_LINEAR) return bitnet_linear_describe(M, N, K, f, workspace_bytes, text, text_bytes);
    if (!text || text_bytes == 0) return BITNET_ERR_NULL;
    text[0] = 0;
    if ((int)entry < 0 || (int)entry > (int)BITNET_ENTRY_FFN_GATE_UP_NORM) return BITNET_ERR_KERNEL;
    const bool pair = entry == BITNET_ENTRY_FFN_GATE_UP || entry == BITNET_ENTRY_FFN_GATE_UP_NORM;
    if (pair && (N <= 0 || N % 16 != 0 || N >= ((int64_t)1 << 29))) return BITNET_ERR_SHAPE;
    const int64_t rows = pair ? 2 * N : N;
    if (!shape_ok(M, rows, K)) return BITNET_ERR_SHAPE;
    if (x_dtype != BITNET_F32 && x_dtype != BITNET_BF16) return BITNET_ERR_DTYPE;
    if (f != BITNET_PACK_2BIT) return BITNET_ERR_FORMAT;
    const float* fp = reinterpret_cast<const float*>(uintptr_t{256});
    void* vp = reinterpret_cast<void*>(uintptr_t{256});
    if (!bitnet::gemv_fused_supports(M, rows, K, vp)) return BITNET_ERR_KERNEL;
    const bool bf16 = x_dtype == BITNET_BF16;
    bitnet::LaunchPlan plan;
    hipError_t e = hipSuccess;
    switch (entry) {
        case BITNET_ENTRY_LINEAR_FUSED:
            e = bitnet::launch_linear_fused_2bit(vp, bf16, vp, fp, 0, M, N, K, vp, OutType::BF16, nullptr, &plan);
            break;
        case BITNET_ENTRY_RMSNORM_LINEAR_FUSED:
            e = bitnet::launch_rmsnorm_linear_fused_2bit(vp, bf16, fp, 0.0f, vp, fp, 0, M, N, K, vp, OutType::BF16, nullptr, &plan);
            break;
        case BITNET_ENTRY_SWIGLU_LINEAR_FUSED:
            e = bitnet::launch_swiglu_linear_fused_2bit(vp, bf16, vp, fp, 0, M, N, K, vp, OutType::BF16, nullptr, &plan);
            break;
        default:
            e = bitnet::launch_linear_fused_swiglu_out_2bit(vp, bf16, entry == BITNET_ENTRY_FFN_GATE_UP_NORM, fp, 0.0f, vp, fp, 0, M,
                                                            N, K, vp, OutType::BF16, nullptr, &plan);
            break;
    }
    if (e != hipSuccess) return BITNET_ERR_HIP;
    return plan_to_text(plan, text, text_bytes);
}

bitnet_status bitnet_linear_segmented(const int8_t* xq, const float* sx, const void* packed, const float* gamma_rb,
                                      int64_t M, int64_t N, int64_t K, bitnet_format f, void* y,
                                      bitnet_dtype y_dtype, bitnet_kernel which, void* stream) {
    return linear_any(xq, sx, packed, gamma_rb, 1, M, N, K, f, y, y_dtype, which, stream);
}

bitnet_status bitnet_quantize_weights_segmented(const void* W, bitnet_dtype w_dtype, int64_t N, int64_t K,
                                                int nseg, const int64_t* seg_rows, bitnet_format f, void* packed,
                                                float* gamma_rb, void* workspace, size_t workspace_bytes,
                                                void* stream) {
    if (!W || !packed || !gamma_rb || !workspace || !seg_rows) return BITNET_ERR_NULL;
    if (!shape_ok(1, N, K) || nseg <= 0) return BITNET_ERR_SHAPE;
    if (w_dtype != BITNET_F32 && w_dtype != BITNET_BF16) return BITNET_ERR_DTYPE;
    if (f != BITNET_PACK_2BIT) return BITNET_ERR_FORMAT;
    if (!aligned(W, dtype_size(w_dtype)) || !aligned(packed, 16) || !aligned(gamma_rb, 4) || !aligned(workspace, 16))
        return BITNET_ERR_ALIGN;
    int64_t total = 0;
    for (int sgm = 0; sgm < nseg; ++sgm) {
        // a segment owns whole 16-row blocks: only the last may end inside one
        if (seg_rows[sgm] <= 0 || (sgm + 1 < nseg && seg_rows[sgm] % 16 != 0)) return BITNET_ERR_SHAPE;
        total += seg_rows[sgm];
    }
    if (total != N) return BITNET_ERR_SHAPE;
    size_t need = 0;
    bitnet_quantize_weights_workspace(N, K, &need);
    if (workspace_bytes < need) return BITNET_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t rb_total = bitnet::ceil_div(N, 16);
    int64_t row0 = 0;
    for (int sgm = 0; sgm < nseg; ++sgm) {
        const int64_t rows = seg_rows[sgm];
        const char* Ws = static_cast<const char*>(W) + row0 * K * (int64_t)dtype_size(w_dtype);
        // the launches of one segment finish with the workspace before the next segment's start (stream order)
        hipError_t e = bitnet::launch_quantize_weights_2bit(Ws, w_dtype == BITNET_BF16, rows, K, packed,
                                                            gamma_rb + row0 / 16, workspace, s, row0 / 16, rb_total,
                                                            bitnet::ceil_div(rows, 16));
        if (e != hipSuccess) return BITNET_ERR_HIP;
        row0 += rows;
    }
    return BITNET_OK;
}

static bitnet_status linear_fused_any(const void* x, bitnet_dtype x_dtype, const void* packed, const float* gamma,
                                      int gstride, int64_t M, int64_t N, int64_t K, bitnet_format f, void* y,
                                      bitnet_dtype y_dtype, void* stream) {
    if (!x || !packed || !gamma || !y) return BITNET_ERR_NULL;
    if (!shape_ok(M, N, K)) return BITNET_ERR_SHAPE;
    if (x_dtype != BITNET_F32 && x_dtype != BITNET_BF16) return BITNET_ERR_DTYPE;
    OutType yt;
    if (!out_type(y_dtype, &yt)) return BITNET_ERR_DTYPE;
    if (!format_ok(f)) return BITNET_ERR_FORMAT;
    if (!aligned(packed, 16) || !aligned(gamma, 4) || !aligned(y, dtype_size(y_dtype))) return BITNET_ERR_ALIGN;
    if (f != BITNET_PACK_2BIT) return BITNET_ERR_FORMAT;
    if (!bitnet::gemv_fused_supports(M, N, K, x)) return BITNET_ERR_KERNEL;
    return from_hip(bitnet::launch_linear_fused_2bit(x, x_dtype == BITNET_BF16, packed, gamma, gstride, M, N, K, y, yt,
                                                     static_cast<hipStream_t>(stream)));
}

bitnet_status bitnet_linear_fused(const void* x, bitnet_dtype x_dtype, const void* packed, const float* gamma,
                                  int64_t M, int64_t N, int64_t K, bitnet_format f, void* y,
                                  bitnet_dtype y_dtype, void* stream) {
    return linear_fused_any(x, x_dtype, packed, gamma, 0, M, N, K, f, y, y_dtype, stream);
}

bitnet_status bitnet_linear_fused_segmented(const void* x, bitnet_dtype x_dtype, const void* packed,
                                            const float* gamma_rb, int64_t M, int64_t N, int64_t K, bitnet_format f,
                                            void* y, bitnet_dtype y_dtype, void* stream) {
    return linear_fused_any(x, x_dtype, packed, gamma_rb, 1, M, N, K, f, y, y_dtype, stream);
}

static bitnet_status rmsnorm_linear_fused_any(const void* x, bitnet_dtype x_dtype, const float* g, float eps,
                                              const void* packed, const float* gamma, int gstride, int64_t M,
                                              int64_t N, int64_t K, bitnet_format f, void* y, bitnet_dtype y_dtype,
                                              void* stream) {
    if (!x || !packed || !gamma || !y) return BITNET_ERR_NULL;
    if (!shape_ok(M, N, K) || !(eps >= 0.0f)) return BITNET_ERR_SHAPE;
    if (x_dtype != BITNET_F32 && x_dtype != BITNET_BF16) return BITNET_ERR_DTYPE;
    OutType yt;
    if (!out_type(y_dtype, &yt)) return BITNET_ERR_DTYPE;
    if (!format_ok(f)) return BITNET_ERR_FORMAT;
    if (!aligned(packed, 16) || !aligned(gamma, 4) || !aligned(y, dtype_size(y_dtype)) || (g && !aligned(g, 16)))
        return BITNET_ERR_ALIGN;
    if (f != BITNET_PACK_2BIT) return BITNET_ERR_FORMAT;
    if (!bitnet::gemv_fused_supports(M, N, K, x)) return BITNET_ERR_KERNEL;
    return from_hip(bitnet::launch_rmsnorm_linear_fused_2bit(x, x_dtype == BITNET_BF16, g, eps, packed, gamma, gstride,
                                                             M, N, K, y, yt, static_cast<hipStream_t>(stream)));
}

bitnet_status bitnet_rmsnorm_linear_fused(const void* x, bitnet_dtype x_dtype, const float* g, float eps,
                                          const void* packed, const float* gamma, int64_t M, int64_t N, int64_t K,
                                          bitnet_format f, void* y, bitnet_dtype y_dtype, void* stream) {
    return rmsnorm_linear_fused_any(x, x_dtype, g, eps, packed, gamma, 0, M, N, K, f, y, y_dtype, stream);
}

bitnet_status bitnet_rmsnorm_linear_fused_segmented(const void* x, bitnet_dtype x_dtype, const float* g, float eps,
                                                    const void* packed, const float* gamma_rb, int64_t M, int64_t N,
                                                    int64_t K, bitnet_format f, void* y, bitnet_dtype y_dtype,
                                                    void* stream) {
    return rmsnorm_linear_fused_any(x, x_dtype, g, eps, packed, gamma_rb, 1, M, N, K, f, y, y_dtype, stream);
}

bitnet_status bitnet_swiglu_linear_fused(const void* gu, bitnet_dtype gu_dtype, const void* packed, const float* gamma,
                                         int64_t M, int64_t N, int64_t F, bitnet_format f, void* y, bitnet_dtype y_dtype,
                                         void* stream) {
    if (!gu || !packed || !gamma || !y) return BITNET_ERR_NULL;
    if (!shape_ok(M, N, F)) return BITNET_ERR_SHAPE;
    if (gu_dtype != BITNET_F32 && gu_dtype != BITNET_BF16) return BITNET_ERR_DTYPE;
    OutType yt;
    if (!out_type(y_dtype, &yt)) return BITNET_ERR_DTYPE;
    if (!format_ok(f)) return BITNET_ERR_FORMAT;
    if (!aligned(packed, 16) || !aligned(gamma, 4) || !aligned(y, dtype_size(y_dtype))) return BITNET_ERR_ALIGN;
    if (f != BITNET_PACK_2BIT) return BITNET_ERR_FORMAT;
    if (!bitnet::gemv_fused_supports(M, N, F, gu)) return BITNET_ERR_KERNEL;
    return from_hip(bitnet::launch_swiglu_linear_fused_2bit(gu, gu_dtype == BITNET_BF16, packed, gamma, 0, M, N, F, y, yt,
                                                            static_cast<hipStream_t>(stream)));
}

bitnet_status bitnet_ffn_gate_up_fused(const void* x, bitnet_dtype x_dtype, int norm, const float* g, float eps,
                                       const void* packed, const float* gamma, int gamma_per_block, int64_t M, int64_t F,
                                       int64_t K, bitnet_format f, void* h, bitnet_dtype h_dtype, void* stream) {
    if (!x || !packed || !gamma || !h) return BITNET_ERR_NULL;
    if (F <= 0 || F % 16 != 0 || F >= ((int64_t)1 << 29) || !shape_ok(M, 2 * F, K) || (norm && !(eps >= 0.0f)))
        return BITNET_ERR_SHAPE;
    if (x_dtype != BITNET_F32 && x_dtype != BITNET_BF16) return BITNET_ERR_DTYPE;
    if (h_dtype != BITNET_F32 && h_dtype != BITNET_BF16) return BITNET_ERR_DTYPE;
    if (!format_ok(f)) return BITNET_ERR_FORMAT;
    if (!aligned(packed, 16) || !aligned(gamma, 4) || !aligned(h, dtype_size(h_dtype)) || (norm && g && !aligned(g, 16)))
        return BITNET_ERR_ALIGN;
    if (f != BITNET_PACK_2BIT) return BITNET_ERR_FORMAT;
    if (!bitnet::gemv_fused_supports(M, 2 * F, K, x)) return BITNET_ERR_KERNEL;
    return from_hip(bitnet::launch_linear_fused_swiglu_out_2bit(
        x, x_dtype == BITNET_BF16, norm != 0, norm ? g : nullptr, eps, packed, gamma, gamma_per_block ? 1 : 0, M, F, K, h,
        h_dtype == BITNET_BF16 ? OutType::BF16 : OutType::F32, static_cast<hipStream_t>(stream)));
}

bitnet_status bitnet_repack_weights(const void* packed_in, bitnet_format f_in, int64_t N, int64_t K, void* packed_out,
                                    bitnet_format f_out, void* stream) {
    if (!packed_in || !packed_out) return BITNET_ERR_NULL;
    if (!shape_ok(1, N, K)) return BITNET_ERR_SHAPE;
    if (!format_ok(f_in) || !format_ok(f_out) || f_in == f_out) return BITNET_ERR_FORMAT;
    if (!aligned(packed_in, 16) || !aligned(packed_out, 16)) return BITNET_ERR_ALIGN;
    return from_hip(bitnet::launch_repack(packed_in, f_in == BITNET_PACK_TRIT5, N, K, packed_out, static_cast<hipStream_t>(stream)));
}

bitnet_status bitnet_unpack_weights(const void* packed, int64_t N, int64_t K, bitnet_format f, int8_t* codes,
                                    void* stream) {
    if (!packed || !codes) return BITNET_ERR_NULL;
    if (!shape_ok(1, N, K)) return BITNET_ERR_SHAPE;
    if (!format_ok(f)) return BITNET_ERR_FORMAT;
    if (!aligned(packed, 16)) return BITNET_ERR_ALIGN;
    if (f == BITNET_PACK_2BIT)
        return from_hip(bitnet::launch_unpack_2bit(packed, N, K, codes, static_cast<hipStream_t>(stream)));
    return from_hip(bitnet::launch_unpack_trit5(packed, N, K, codes, static_cast<hipStream_t>(stream)));
}

}  // extern "C"

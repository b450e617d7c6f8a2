// Absmean ternary weight quantization (Eq. (1)-(3) of arXiv 2402.17764) for gfx950.
//
//   pass 1  abs_sum_partials : grid-stride |W| sum, double-double per thread, fixed-shape tree
//                              inside the block, one (hi, lo) pair per block into the workspace
//   pass 2  finish_gamma     : one block folds the partials in a fixed order, gamma = fp32(S / (N K)); the 2-bit
//                              packing does this at the top of pass 3 instead (one launch and 4.5 us less)
//   pass 3  ternarize_pack   : re-reads W from its end (what pass 1 read last is still in the memory-side
//                              cache), takes the decision of Eq. (1)-(2) in fp32 and writes the packed
//                              layout one 1 KiB (row block, K step) chunk per workgroup pass
//
// The whole path is HBM-bound at 8.25 B per weight (two reads of W, one packed write).  Both reading passes
// are shaped by what a plain read loop reaches on this chip: 8 waves per CU with four 16-byte loads each in
// flight read 6.1-6.2 TB/s, 32 waves per CU 5.1-5.3 TB/s.
#include "bitnet_device.hpp"
#include "bitnet_internal.hpp"

namespace bitnet {

// ---------------------------------------------------------------------------------------------------
// pass 1
// ---------------------------------------------------------------------------------------------------
constexpr int kSumThreads = 512;
constexpr int kSumBlocks = 256;                           // one per CU: 8 waves per CU
constexpr int kSumLoads = 4;                              // 16-byte loads in flight per thread

__device__ inline float widen1(float v) { return v; }
__device__ inline float widen1(uint16_t v) { return bf16_to_f32(v); }

// |.| of the 4 (fp32) or 8 (bf16) elements of one 16-byte vector, each added to one of four accumulators
template <typename T>
__device__ inline void add_abs(const uint4& q, dd (&part)[4]) {
    const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (sizeof(T) == 4) {
            dd_add_double(part[e], (double)fabsf(__uint_as_float(u[e])));
        } else {
            dd_add_double(part[e], (double)fabsf(bf16_to_f32((uint16_t)(u[e] & 0xFFFFu))));
            dd_add_double(part[e], (double)fabsf(bf16_to_f32((uint16_t)(u[e] >> 16))));
        }
    }
}

template <typename T>
__global__ __launch_bounds__(kSumThreads) void abs_sum_partials(const T* __restrict__ W, int64_t count,
                                                                int vec_ok, int64_t stream_vecs,
                                                                double* __restrict__ partials) {
    constexpr int kPer = 16 / (int)sizeof(T);             // elements per 16-byte vector
    dd acc{0.0, 0.0};
    const int64_t tid = (int64_t)blockIdx.x * kSumThreads + threadIdx.x;
    const int64_t nthreads = (int64_t)gridDim.x * kSumThreads;
    int64_t done = 0;
    if (vec_ok) {
        const int64_t nvec = count / kPer;
        const uint4* Wv = reinterpret_cast<const uint4*>(W);
        // the sums are exact, so the split into four accumulators changes nothing but the length of the dependent
        // chains; the next round of loads is requested before this round's values are added
        dd part[4] = {{0.0, 0.0}, {0.0, 0.0}, {0.0, 0.0}, {0.0, 0.0}};
        int64_t i = tid;
        uint4 nxt[kSumLoads];
        bool have = i + (kSumLoads - 1) * nthreads < nvec;
        // The first stream_vecs vectors are read with the streaming policy (a plain read loop reaches 7.1 TB/s that
        // way against 6.4 TB/s); the end of W is read normally so that it stays in the memory-side cache, where the
        // packing pass, which starts from the end, finds it.
        auto request = [&](uint4 (&v)[kSumLoads], int64_t at) {
            if (at + (kSumLoads - 1) * nthreads < stream_vecs) {
#pragma unroll
                for (int u = 0; u < kSumLoads; ++u) v[u] = load_streaming_b128(Wv + at + u * nthreads);
            } else {
#pragma unroll
                for (int u = 0; u < kSumLoads; ++u) v[u] = Wv[at + u * nthreads];
            }
        };
        if (have) request(nxt, i);
        while (have) {
            uint4 cur[kSumLoads];
#pragma unroll
            for (int u = 0; u < kSumLoads; ++u) cur[u] = nxt[u];
            i += kSumLoads * nthreads;
            have = i + (kSumLoads - 1) * nthreads < nvec;
            if (have) request(nxt, i);
#pragma unroll
            for (int u = 0; u < kSumLoads; ++u) add_abs<T>(cur[u], part);
        }
        for (; i < nvec; i += nthreads) add_abs<T>(Wv[i], part);
#pragma unroll
        for (int e = 0; e < 4; ++e) dd_add_dd(acc, part[e]);
        done = nvec * kPer;
    }
    for (int64_t i = done + tid; i < count; i += nthreads) dd_add_double(acc, (double)fabsf(widen1(W[i])));

    // fixed-shape tree over the block: the same pairs are always added in the same order
    __shared__ double sh_hi[kSumThreads];
    __shared__ double sh_lo[kSumThreads];
    sh_hi[threadIdx.x] = acc.hi;
    sh_lo[threadIdx.x] = acc.lo;
    __syncthreads();
    for (int s = kSumThreads / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) {
            dd a{sh_hi[threadIdx.x], sh_lo[threadIdx.x]};
            dd b{sh_hi[threadIdx.x + s], sh_lo[threadIdx.x + s]};
            dd_add_dd(a, b);
            sh_hi[threadIdx.x] = a.hi;
            sh_lo[threadIdx.x] = a.lo;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        partials[2 * blockIdx.x] = sh_hi[0];
        partials[2 * blockIdx.x + 1] = sh_lo[0];
    }
}

// ---------------------------------------------------------------------------------------------------
// pass 2
// ---------------------------------------------------------------------------------------------------
constexpr int kFinishThreads = 256;
// The partial sums of pass 1 added up over one workgroup in a fixed tree: thread t folds partials t, t + 256, ...,
// then the 256 running pairs are halved eight times.  Returned unnormalised to every thread.
__device__ inline dd fold_partials(const double* __restrict__ partials, int nparts, double* sh_hi, double* sh_lo) {
    dd acc{0.0, 0.0};
    for (int i = threadIdx.x; i < nparts; i += kFinishThreads) {
        dd p{partials[2 * i], partials[2 * i + 1]};
        dd_add_dd(acc, p);
    }
    sh_hi[threadIdx.x] = acc.hi;
    sh_lo[threadIdx.x] = acc.lo;
    __syncthreads();
    for (int s = kFinishThreads / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) {
            dd a{sh_hi[threadIdx.x], sh_lo[threadIdx.x]};
            dd b{sh_hi[threadIdx.x + s], sh_lo[threadIdx.x + s]};
            dd_add_dd(a, b);
            sh_hi[threadIdx.x] = a.hi;
            sh_lo[threadIdx.x] = a.lo;
        }
        __syncthreads();
    }
    return dd{sh_hi[0], sh_lo[0]};
}

// gamma[0 .. nout-1] all receive the value (nout > 1: one copy per 16-row block of a segment)
__global__ __launch_bounds__(kFinishThreads) void finish_gamma(const double* __restrict__ partials, int nparts,
                                                            int64_t count, float* __restrict__ gamma, int64_t nout) {
    __shared__ double sh_hi[kFinishThreads];
    __shared__ double sh_lo[kFinishThreads];
    const dd t = fold_partials(partials, nparts, sh_hi, sh_lo);
    const double S = t.hi + t.lo;
    const float g = (float)(S / (double)count);     // Eq. (3); fp64 IEEE division, one rounding to fp32
    for (int64_t i = threadIdx.x; i < nout; i += kFinishThreads) gamma[i] = g;
}

// The sum of pass 1's partials as a normalised double-double pair (hi = fl(hi + lo)): what one shard of a row-sharded
// matrix contributes to Eq. (3).  Same fixed tree as finish_gamma.
__global__ __launch_bounds__(kFinishThreads) void fold_abs_sum(const double* __restrict__ partials, int nparts,
                                                            double* __restrict__ sum) {
    __shared__ double sh_hi[kFinishThreads];
    __shared__ double sh_lo[kFinishThreads];
    const dd t = fold_partials(partials, nparts, sh_hi, sh_lo);
    if (threadIdx.x == 0) {
        const double hi = t.hi + t.lo;
        sum[0] = hi;
        sum[1] = t.lo - (hi - t.hi);                      // exact: |lo| <= |hi|
    }
}

// ---------------------------------------------------------------------------------------------------
// pass 3, 2-bit format
// ---------------------------------------------------------------------------------------------------
// One work item is one 1 KiB chunk of the packed layout: a 16-row block x one K step of 256 columns.  A workgroup
// has four waves; wave w reads rows 4w .. 4w+3 of the item (lane l: columns 4l .. 4l+3 of the step, one 16-byte
// load per row for fp32, marked streaming: this is the last use of W).  The four codes of a lane land in one word at
// bits 8 b + 2 i with i = l & 3; OR-ing the four lanes of a quad completes the word, which every lane of the quad
// then holds.  One ds_bpermute transposes the wave's 4 rows x 16 words so that lane 16 g + 4 t + j holds word j of
// quad column g for row 4w + t: the wave stores four 64-byte runs, no LDS memory and no barrier.  Items are walked
// from the end of W backwards, workgroup b taking items b, b + gridDim.x, ...: neighbouring workgroups read
// neighbouring 1 KiB runs of the same 16 rows, and the next item's rows are requested before this one's are coded.
constexpr int kPackThreads = 256;
constexpr int kPackBlocks = 1024;                          // four per CU
static_assert(kSumBlocks <= kPackThreads, "the packing pass folds one partial sum of pass 1 per thread");

template <typename T> struct PackVec;
template <> struct PackVec<float> {
    __device__ static void load(const float* p, float (&f)[4]) {
        const uint4 q = load_streaming_b128(p);
        f[0] = __uint_as_float(q.x); f[1] = __uint_as_float(q.y); f[2] = __uint_as_float(q.z); f[3] = __uint_as_float(q.w);
    }
};
template <> struct PackVec<uint16_t> {
    __device__ static void load(const uint16_t* p, float (&f)[4]) {
        typedef unsigned v2u __attribute__((ext_vector_type(2)));
        const v2u q = __builtin_nontemporal_load(reinterpret_cast<const v2u*>(p));
        f[0] = __uint_as_float(q.x << 16); f[1] = __uint_as_float(q.x & 0xFFFF0000u);
        f[2] = __uint_as_float(q.y << 16); f[3] = __uint_as_float(q.y & 0xFFFF0000u);
    }
};

// W, N: the rows being packed (a whole matrix, or one segment of it); they become row blocks rb_off ... of a
// packed matrix of RB row blocks in all.
template <typename T, bool kVec>
__global__ __launch_bounds__(kPackThreads) void ternarize_pack_2bit(const T* __restrict__ W, int64_t N, int64_t K,
                                                                    int64_t Kq /* quads per row */, int64_t RB,
                                                                    int64_t rb_off, const double* __restrict__ partials,
                                                                    int nparts, int64_t count, float* __restrict__ gamma_out,
                                                                    int64_t nout, uint32_t* __restrict__ packed) {
    __shared__ double sh_hi[kPackThreads / kWave];
    __shared__ double sh_lo[kPackThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x >> 6;
    const int i = lane & 3;
    const int64_t steps = ceil_div(Kq, 4);
    const int64_t items = ceil_div(N, kRowsPerBlock) * steps;
    // lane 16 g + 4 t + j takes its word from lane 16 g + 4 j + t (which selected row t's word below)
    const int src = ((lane & 48) | ((lane & 3) << 2) | ((lane >> 2) & 3)) << 2;

    auto load = [&](int64_t item, float (&f)[4][4]) {
        item = items - 1 - item;
        const int64_t rb = item / steps, s = item - rb * steps;
        const int64_t k = 256 * s + 4 * lane;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int64_t n = rb * kRowsPerBlock + 4 * w + t;
#pragma unroll
            for (int b = 0; b < 4; ++b) f[t][b] = 0.f;     // padding rows / columns quantize to code 0
            if (n < N) {
                const T* row = W + n * K;
                if (kVec) {
                    if (k < K) PackVec<T>::load(row + k, f[t]);
                } else {
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        if (k + b < K) f[t][b] = widen1(row[k + b]);
                }
            }
        }
    };

    float nxt[4][4];
    int64_t item = blockIdx.x;
    if (item < items) load(item, nxt);

    // Pass 2 folded in: while the first rows are on their way every workgroup adds up the partial sums of pass 1
    // (one per thread; exact sums, so every workgroup gets the same bits) and takes gamma = fp32(S / (N K)), Eq. (3):
    // one fp64 IEEE division, one rounding to fp32.  Workgroup 0 writes it out, once per 16-row block of the segment.
    dd part{0.0, 0.0};
    if ((int)threadIdx.x < nparts) part = dd{partials[2 * threadIdx.x], partials[2 * threadIdx.x + 1]};
    const double S = block_sum_dd<kPackThreads / kWave>(part, sh_hi, sh_lo);
    const float g = (float)(S / (double)count);
    if (blockIdx.x == 0)
        for (int64_t o = threadIdx.x; o < nout; o += kPackThreads) gamma_out[o] = g;
    const float d = g + kEps;                              // gamma + eps, one fp32 add (Eq. (1))
    const float thr = ternary_threshold(d);                // |w| >= thr  <=>  RoundClip(w / d) = +-1

    for (; item < items; item += gridDim.x) {
        float cur[4][4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int b = 0; b < 4; ++b) cur[t][b] = nxt[t][b];
        if (item + gridDim.x < items) load(item + gridDim.x, nxt);
        uint32_t c[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            uint32_t v = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) v |= ternary_code2_threshold(cur[t][b], thr) << (8 * b + 2 * i);
            c[t] = quad_or(v);
        }
        const uint32_t sel = i == 0 ? c[0] : i == 1 ? c[1] : i == 2 ? c[2] : c[3];
        const uint32_t out = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)sel);
        const int64_t it = items - 1 - item;
        const int64_t rb = it / steps, s = it - rb * steps;
        const int64_t nq = (Kq - 4 * s) < 4 ? (Kq - 4 * s) : 4;     // quads of this step (the last may hold fewer)
        const int g = lane >> 4;
        // word index inside the chunk: ((g * 16 + row) * 4 + j) with row = 4 w + t, and lane & 15 = 4 t + j
        if (g < nq) packed[quad_index_2bit(4 * s, rb + rb_off, 0, Kq, RB) * 4 + g * 64 + 16 * w + (lane & 15)] = out;
    }
}

// ---------------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------------
int quant_weights_num_partials() { return 2048; }

// 16-byte vectors of W that pass 1 reads with the streaming policy: all but the last 192 MB (the memory-side cache
// holds 256 MB; what it keeps of W is what pass 3 reads first)
static int64_t abs_sum_stream_vecs(int64_t count, int64_t esz) {
    const int64_t keep = ((int64_t)192 << 20) / 16;
    const int64_t nvec = count * esz / 16;
    return nvec > keep ? nvec - keep : 0;
}

static int abs_sum_blocks(int64_t count) {
    const int64_t want = ceil_div(count, (int64_t)kSumThreads * 16);
    return (int)(want < 1 ? 1 : (want > kSumBlocks ? kSumBlocks : want));
}

static void launch_abs_sum_partials(const void* W, bool bf16, int64_t count, double* partials, int blocks, hipStream_t stream) {
    const int vec_ok = (reinterpret_cast<uintptr_t>(W) % 16) == 0;
    if (bf16)
        hipLaunchKernelGGL(abs_sum_partials<uint16_t>, dim3(blocks), dim3(kSumThreads), 0, stream,
                           static_cast<const uint16_t*>(W), count, vec_ok, abs_sum_stream_vecs(count, 2), partials);
    else
        hipLaunchKernelGGL(abs_sum_partials<float>, dim3(blocks), dim3(kSumThreads), 0, stream,
                           static_cast<const float*>(W), count, vec_ok, abs_sum_stream_vecs(count, 4), partials);
}

// Eq. (3) as passes 1 and 2 (the 5-trit packing reads gamma from memory; the 2-bit packing folds pass 2 into pass 3)
hipError_t launch_absmean_gamma(const void* W, bool bf16, int64_t N, int64_t K, float* gamma, void* workspace,
                                hipStream_t stream, int64_t nout) {
    const int64_t count = N * K;
    double* partials = static_cast<double*>(workspace);
    const int blocks = abs_sum_blocks(count);
    launch_abs_sum_partials(W, bf16, count, partials, blocks, stream);
    hipLaunchKernelGGL(finish_gamma, dim3(1), dim3(kFinishThreads), 0, stream, partials, blocks, count, gamma, nout);
    return hipGetLastError();
}

hipError_t launch_abs_sum(const void* W, bool bf16, int64_t N, int64_t K, double* sum, void* workspace, hipStream_t stream) {
    const int64_t count = N * K;
    double* partials = static_cast<double*>(workspace);
    const int blocks = abs_sum_blocks(count);
    launch_abs_sum_partials(W, bf16, count, partials, blocks, stream);
    hipLaunchKernelGGL(fold_abs_sum, dim3(1), dim3(kFinishThreads), 0, stream, partials, blocks, sum);
    return hipGetLastError();
}

int quant_weights_max_sums() { return kPackThreads; }

hipError_t launch_gamma_from_sums(const double* sums, int nsums, int64_t total_count, float* gamma, hipStream_t stream) {
    hipLaunchKernelGGL(finish_gamma, dim3(1), dim3(kFinishThreads), 0, stream, sums, nsums, total_count, gamma, (int64_t)1);
    return hipGetLastError();
}

hipError_t launch_pack_2bit_with_sums(const void* W, bool bf16, int64_t N, int64_t K, const double* sums, int nsums,
                                      int64_t total_count, void* packed, float* gamma, hipStream_t stream) {
    const size_t esz = bf16 ? 2 : 4;
    const bool vec = (reinterpret_cast<uintptr_t>(W) % (4 * esz)) == 0 && (K % 4 == 0);
    const int64_t Kq = ceil_div(K, kColsPerQuad);
    const int64_t RB = ceil_div(N, kRowsPerBlock);
    const int64_t items = RB * ceil_div(Kq, 4);
    dim3 grid((unsigned)(items < kPackBlocks ? items : kPackBlocks));
    uint32_t* out = static_cast<uint32_t*>(packed);
#define PACK(T_, V_) hipLaunchKernelGGL((ternarize_pack_2bit<T_, V_>), grid, dim3(kPackThreads), 0, stream, w, N, K, Kq, RB, (int64_t)0, \
                                        sums, nsums, total_count, gamma, (int64_t)1, out)
    if (bf16) {
        const uint16_t* w = static_cast<const uint16_t*>(W);
        if (vec) PACK(uint16_t, true); else PACK(uint16_t, false);
    } else {
        const float* w = static_cast<const float*>(W);
        if (vec) PACK(float, true); else PACK(float, false);
    }
#undef PACK
    return hipGetLastError();
}

hipError_t launch_quantize_weights_2bit(const void* W, bool bf16, int64_t N, int64_t K, void* packed,
                                        float* gamma, void* workspace, hipStream_t stream, int64_t rb_off,
                                        int64_t rb_total, int64_t nout) {
    const int64_t count = N * K;
    double* partials = static_cast<double*>(workspace);
    const int blocks = abs_sum_blocks(count);
    const size_t esz = bf16 ? 2 : 4;
    const bool vec = (reinterpret_cast<uintptr_t>(W) % (4 * esz)) == 0 && (K % 4 == 0);
    launch_abs_sum_partials(W, bf16, count, partials, blocks, stream);

    const int64_t Kq = ceil_div(K, kColsPerQuad);
    const int64_t RB = ceil_div(N, kRowsPerBlock);                       // row blocks packed by this call
    const int64_t RBT = rb_total > 0 ? rb_total : RB;                      // ... of the whole packed matrix
    const int64_t items = RB * ceil_div(Kq, 4);
    dim3 grid((unsigned)(items < kPackBlocks ? items : kPackBlocks));
    uint32_t* out = static_cast<uint32_t*>(packed);
#define PACK(T_, V_) hipLaunchKernelGGL((ternarize_pack_2bit<T_, V_>), grid, dim3(kPackThreads), 0, stream, w, N, K, Kq, RBT, rb_off, \
                                        partials, blocks, count, gamma, nout, out)
    if (bf16) {
        const uint16_t* w = static_cast<const uint16_t*>(W);
        if (vec) PACK(uint16_t, true); else PACK(uint16_t, false);
    } else {
        const float* w = static_cast<const float*>(W);
        if (vec) PACK(float, true); else PACK(float, false);
    }
#undef PACK
    return hipGetLastError();
}

}  // namespace bitnet

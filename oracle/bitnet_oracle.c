/*
 * CPU oracle for the BitLinear W1.58A8 product of BitNet b1.58 (arXiv 2402.17764, Section 2).
 * TEST INFRASTRUCTURE ONLY -- see bitnet_oracle.h.  Plain scalar C, no intrinsics, no blocking,
 * no code shared with the GPU library.  Build: gcc -O2 -ffp-contract=off -fopenmp (never
 * -ffast-math: the compensated sum and the fp32 rounding steps rely on IEEE semantics).
 */
#include "bitnet_oracle.h"

#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Eq. (3). */
int oracle_absmean_gamma(const float* W, int64_t N, int64_t K, float* gamma, double* abs_sum) {
    if (!W || !gamma) return 1;
    if (N <= 0 || K <= 0) return 2;
    /* Neumaier's compensated summation: `sum` carries the running fp64 sum, `comp` collects the
       low-order bits each addition drops.  Row-major order, one thread. */
    double sum = 0.0, comp = 0.0;
    const int64_t count = N * K;
    for (int64_t i = 0; i < count; ++i) {
        float w = W[i];
        if (!isfinite(w)) return 3;
        double a = fabs((double)w);
        double t = sum + a;
        if (sum >= a) comp += (sum - t) + a;
        else          comp += (a - t) + sum;
        sum = t;
    }
    double S = sum + comp;
    if (abs_sum) *abs_sum = S;
    *gamma = (float)(S / (double)count);
    return 0;
}

/* Eq. (2): RoundClip(x, a, b) = max(a, min(b, round(x))), round = nearest, ties to even. */
static float round_clip(float x, float a, float b) {
    float r = rintf(x);
    if (r > b) r = b;
    if (r < a) r = a;
    return r;
}

/* Eq. (1). */
int oracle_ternarize(const float* W, int64_t N, int64_t K, float gamma, int8_t* codes) {
    if (!W || !codes) return 1;
    if (N <= 0 || K <= 0) return 2;
    const float denom = gamma + ORACLE_EPS;       /* one fp32 add */
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t i = 0; i < N; ++i) {
        for (int64_t j = 0; j < K; ++j) {
            float w = W[i * K + j];
            if (!isfinite(w)) bad |= 1;
            float q = w / denom;                  /* one fp32 IEEE division */
            codes[i * K + j] = (int8_t)round_clip(q, -1.0f, 1.0f);
        }
    }
    return bad ? 3 : 0;
}

/* Section 2: per-token absmax quantization to [-Q_b, Q_b], Q_b = 127, no zero point. */
int oracle_quantize_acts(const float* x, int64_t M, int64_t K, int8_t* xq, float* sx) {
    if (!x || !xq || !sx) return 1;
    if (M <= 0 || K <= 0) return 2;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        const float* row = x + m * K;
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            if (!isfinite(row[k])) bad |= 1;
            float a = fabsf(row[k]);
            if (a > amax) amax = a;
        }
        float s = amax > 1e-5f ? amax : 1e-5f;
        float inv = (float)ORACLE_QB / s;         /* one fp32 IEEE division per token */
        sx[m] = s;
        for (int64_t k = 0; k < K; ++k) {
            float r = round_clip(row[k] * inv, -(float)ORACLE_QB, (float)ORACLE_QB);
            xq[m * K + k] = (int8_t)r;
        }
    }
    return bad ? 3 : 0;
}

/* acc = x_q . codes^T in integers: a ternary weight adds, subtracts or skips its activation. */
int oracle_ternary_matmul(const int8_t* xq, const int8_t* codes, int64_t M, int64_t N, int64_t K,
                          int32_t* acc) {
    if (!xq || !codes || !acc) return 1;
    if (M <= 0 || N <= 0 || K <= 0) return 2;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            const int8_t* xr = xq + m * K;
            const int8_t* wr = codes + n * K;
            int32_t s = 0;
            for (int64_t k = 0; k < K; ++k) {
                if (wr[k] > 0)      s += xr[k];
                else if (wr[k] < 0) s -= xr[k];
            }
            acc[m * N + n] = s;
        }
    }
    return 0;
}

/* y = acc * gamma * s_x / Q_b, every factor widened to fp64 first. */
int oracle_rescale(const int32_t* acc, float gamma, const float* sx, int64_t M, int64_t N,
                   double* y) {
    if (!acc || !sx || !y) return 1;
    if (M <= 0 || N <= 0) return 2;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
            y[m * N + n] = (double)acc[m * N + n] * (double)gamma * (double)sx[m] / (double)ORACLE_QB;
    return 0;
}

/* Compensated fp64 sum of squares of one row (the squares of fp32 values are exact in fp64). */
static double row_mean_square(const float* x, int64_t K) {
    double sum = 0.0, comp = 0.0;
    for (int64_t k = 0; k < K; ++k) {
        double a = (double)x[k] * (double)x[k];
        double t = sum + a;
        if (sum >= a) comp += (sum - t) + a;
        else          comp += (a - t) + sum;
        sum = t;
    }
    return (sum + comp) / (double)K;
}

/* absmax quantization of one already-computed fp32 row (the per-token step of Section 2). */
static void quantize_row(const float* v, int64_t K, int8_t* q, float* scale) {
    float amax = 0.0f;
    for (int64_t k = 0; k < K; ++k) {
        float a = fabsf(v[k]);
        if (a > amax) amax = a;
    }
    const float s = amax > ORACLE_EPS ? amax : ORACLE_EPS;
    const float inv = (float)ORACLE_QB / s;
    for (int64_t k = 0; k < K; ++k)
        q[k] = (int8_t)round_clip(v[k] * inv, -(float)ORACLE_QB, (float)ORACLE_QB);
    *scale = s;
}

/* RMSNorm, then the activation quantization. */
int oracle_rmsnorm_quantize(const float* x, const float* g, float eps, int64_t M, int64_t K,
                            int8_t* xq, float* sx, float* z) {
    if (!x || !xq || !sx) return 1;
    if (M <= 0 || K <= 0) return 2;
    float* own = z ? NULL : (float*)malloc((size_t)M * (size_t)K * sizeof(float));
    float* zz = z ? z : own;
    if (!zz) return 1;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        const float* row = x + m * K;
        float* zr = zz + m * K;
        for (int64_t k = 0; k < K; ++k)
            if (!isfinite(row[k])) bad = 1;
        const double ms = row_mean_square(row, K);
        const float r = (float)(1.0 / sqrt(ms + (double)eps));
        for (int64_t k = 0; k < K; ++k) {
            float v = row[k] * r;
            if (g) v = v * g[k];
            zr[k] = v;
        }
        quantize_row(zr, K, xq + m * K, sx + m);
    }
    free(own);
    return bad ? 3 : 0;
}

float oracle_exp32(float t) {
    if (t < -87.0f) t = -87.0f;
    if (t > 88.0f) t = 88.0f;
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

/* SwiGLU gating, then the activation quantization. */
int oracle_swiglu_quantize(const float* gu, int64_t M, int64_t F, int8_t* hq, float* sh, float* h) {
    if (!gu || !hq || !sh) return 1;
    if (M <= 0 || F <= 0) return 2;
    float* own = h ? NULL : (float*)malloc((size_t)M * (size_t)F * sizeof(float));
    float* hh = h ? h : own;
    if (!hh) return 1;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        const float* gate = gu + m * 2 * F;
        const float* up = gate + F;
        float* hr = hh + m * F;
        for (int64_t f = 0; f < F; ++f) {
            if (!isfinite(gate[f]) || !isfinite(up[f])) bad = 1;
            const float e = oracle_exp32(-gate[f]);
            const float s = gate[f] / (1.0f + e);
            hr[f] = s * up[f];
        }
        quantize_row(hr, F, hq + m * F, sh + m);
    }
    free(own);
    return bad ? 3 : 0;
}

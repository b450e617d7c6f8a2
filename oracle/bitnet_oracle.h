/*
 * CPU oracle for the BitLinear W1.58A8 product of BitNet b1.58 (arXiv 2402.17764, Section 2).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a plain, slow, scalar statement of what
 * the method computes, written from the paper's equations so that it can be checked against them
 * by eye.  Only tests, the smoke check and the benchmark's cpu_baseline leg may call it; the GPU
 * library neither links nor imports anything from this directory, and nothing here includes a
 * header of the GPU library.
 *
 * All buffers are host memory owned by the caller.  Matrices are row-major:
 *   W, codes : [N][K]   (N output features, K input features, K contiguous)
 *   x, xq    : [M][K]   (M tokens)
 *   acc, y   : [M][N]
 * Every function returns 0 on success, 1 on a NULL pointer, 2 on a non-positive size and
 * 3 on a non-finite input value.
 *
 * Pins (tests that tie each function to something other than itself) are listed beside each
 * declaration; the tests live in tests/test_oracle_*.py.
 */
#ifndef BITNET_ORACLE_H
#define BITNET_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The epsilon of Eq. (1).  The paper prints only the symbol; 1e-5 is this build's reading. */
#define ORACLE_EPS 1e-5f
/* Q_b of Section 2 for 8-bit activations: the symmetric range is [-127, 127]. */
#define ORACLE_QB 127

/*
 * Eq. (3): gamma = (1/(n m)) * sum_ij |W_ij|.
 * The sum runs over the matrix in row-major order in fp64 with Neumaier's compensation, so it is
 * the exact sum to ~1e-32 relative; the single rounding to fp32 happens after the division.
 * abs_sum (optional, may be NULL) receives the fp64 sum.
 * Pins: hand-worked dyadic example (gamma = 0.625); numpy fp64 mean on random matrices; the closed
 * form sigma*sqrt(2/pi) for Gaussian weights; exact power-of-two scaling.
 */
int oracle_absmean_gamma(const float* W, int64_t N, int64_t K, float* gamma, double* abs_sum);

/*
 * Eq. (1)-(2): code_ij = max(-1, min(1, round(W_ij / (gamma + eps)))).
 * gamma + eps is one fp32 addition, W/(gamma+eps) one fp32 IEEE division, round is to nearest with
 * ties to even (the decision is taken in fp32, the precision the GPU kernel decides in).
 * Pins: hand-worked example; the closed form (+1 if q > 0.5, -1 if q < -0.5, else 0) on tie and
 * near-tie values; odd symmetry (negating W negates every code); the Gaussian code mix
 * erf(1/(2 sqrt(pi))) = 31.0 % zeros.
 */
int oracle_ternarize(const float* W, int64_t N, int64_t K, float gamma, int8_t* codes);

/*
 * Section 2, activation quantization: per token m,
 *   s_x[m] = max(max_k |x[m][k]|, 1e-5),  inv = 127 / s_x[m]  (one fp32 division),
 *   x_q[m][k] = clip(round(x[m][k] * inv), -127, 127)          (one fp32 multiply, ties to even).
 * No zero point: the range is symmetric.
 * Pins: hand-worked example; tie cases; |x_q| <= 127 with the absmax element at +-127; power-of-two
 * scaling of a token leaves x_q unchanged; odd symmetry; all-zero token gives zeros.
 */
int oracle_quantize_acts(const float* x, int64_t M, int64_t K, int8_t* xq, float* sx);

/*
 * The BitLinear product (Sections 1-2): acc[m][n] = sum_k x_q[m][k] * code[n][k], in integers.
 * Written as add / subtract / skip, which is all a ternary weight can ask for.
 * Pins: numpy int64 matmul; all-ones codes give row sums; one-hot codes copy x_q; column
 * permutation invariance.
 */
int oracle_ternary_matmul(const int8_t* xq, const int8_t* codes, int64_t M, int64_t N, int64_t K,
                          int32_t* acc);

/*
 * Undo both scales: y[m][n] = acc[m][n] * gamma * s_x[m] / 127, in fp64.
 * Pin: equals the fp64 matrix product of the dequantized operands (x_q s_x/127) (gamma codes)^T.
 */
int oracle_rescale(const int32_t* acc, float gamma, const float* sx, int64_t M, int64_t N,
                   double* y);

/*
 * The block around BitLinear (Section 2, "LLaMA-alike components": RMSNorm and SwiGLU are named,
 * not printed; these are the textbook definitions, with the precision of every step fixed so that
 * the int8 codes they lead to are decided in one stated way).
 *
 * RMSNorm followed by the activation quantization above: per token m,
 *   ms   = (1/K) * sum_k x[m][k]^2          (fp64, compensated: the exact mean of squares)
 *   r    = (float)(1 / sqrt(ms + eps))      (fp64 arithmetic, one rounding to fp32)
 *   z[k] = (x[m][k] * r) * g[k]             (two fp32 multiplies; g == NULL means no gain: one multiply)
 * then s_x, inv and x_q from z exactly as in oracle_quantize_acts.  z (optional, may be NULL)
 * receives the normalised row.
 * Pins: hand-worked dyadic example; the fp64 definition evaluated by numpy (z to 1e-6 relative, codes
 * to one step); unit mean square of z when g is absent; scaling a token by a power of two with eps = 0
 * changes nothing; reduces to oracle_quantize_acts when the token already has unit mean square.
 */
int oracle_rmsnorm_quantize(const float* x, const float* g, float eps, int64_t M, int64_t K,
                            int8_t* xq, float* sx, float* z);

/*
 * The exponential used by the gate below, in fp32 with every step fixed:
 *   t clamped to [-87, 88];  n = round(t * log2(e));  r = (t - n * 0.693359375) - n * (-2.12194440e-4);
 *   p = 1 + r (1 + r (1/2 + r (1/6 + r (1/24 + r (1/120 + r / 720)))))   (Horner, multiply then add);
 *   result = p * 2^n.
 * Pin: libm's exp in fp64 to 4e-7 relative on a dense grid; exp32(0) == 1.
 */
float oracle_exp32(float t);

/*
 * SwiGLU gating followed by the activation quantization: gu is [M][2F], gate = gu[:, :F],
 * up = gu[:, F:];  per element  e = exp32(-gate), s = gate / (1 + e), h = s * up  (fp32 add, IEEE
 * division, fp32 multiply), then s_x, inv and x_q from h as in oracle_quantize_acts.  h (optional)
 * receives the gated row.
 * Pins: silu(gate) * up in fp64 by numpy (1e-6 relative); gate = 0 gives 0; large gate gives
 * gate * up; swapping gate and up halves changes the result (orientation).
 */
int oracle_swiglu_quantize(const float* gu, int64_t M, int64_t F, int8_t* hq, float* sh, float* h);

/* Number of OpenMP threads the row loops will use (the gamma sum is always one thread). */
int oracle_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif

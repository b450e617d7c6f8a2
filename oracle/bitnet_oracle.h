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

/* Number of OpenMP threads the row loops will use (the gamma sum is always one thread). */
int oracle_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif

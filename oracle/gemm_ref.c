/*
 * ECF8 CPU oracle, part 4 -- TEST INFRASTRUCTURE ONLY.
 *
 * Reference for the fused decode + FP8 GEMM case: Y[m][n] = sum_k X[m][k] * W[n][k]
 * with X and W given as raw FP8 E4M3 bytes (OCP "fn": bias 7, no infinities,
 * exponent 15 with mantissa 7 is NaN, exponent 0 is subnormal with step 2^-9).
 * Products of two E4M3 values are exact in binary64 and so is their sum over a
 * few thousand terms to within 2^-53 relative, so Y is the real-number result
 * rounded once.  Also returns A[m][n] = sum_k |X[m][k] * W[n][k]|, the scale the
 * accumulation-order tolerance is stated against.
 * The paper always materialises a layer and hands it to the framework's GEMM
 * (Section 3.3); this reference is that GEMM written out as its definition.
 */
#include <stdint.h>
#include <math.h>

double orc_e4m3_to_double(uint8_t b)
{
    int s = b >> 7, e = (b >> 3) & 15, m = b & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m, -9);
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return s ? -v : v;
}

void orc_gemm_ref(const uint8_t *X, const uint8_t *W, uint64_t M, uint64_t N, uint64_t K,
                  double *Y, double *A)
{
    double lut[256];
    for (int i = 0; i < 256; i++) lut[i] = orc_e4m3_to_double((uint8_t)i);
    for (uint64_t m = 0; m < M; m++)
        for (uint64_t n = 0; n < N; n++) {
            double acc = 0.0, mag = 0.0;
            const uint8_t *x = X + m * K, *w = W + n * K;
            for (uint64_t k = 0; k < K; k++) {
                double p = lut[x[k]] * lut[w[k]];
                acc += p;
                mag += fabs(p);
            }
            Y[m * N + n] = acc;
            A[m * N + n] = mag;
        }
}

/*
 * The same with block scales: W carries one scale per 128 x 128 block
 * (ws[(n/128) * ceil(K/128) + k/128]), X xs_cols scales per row: one (xs[m]) or
 * one per 128 columns (xs[m * xs_cols + k/128]); xs = NULL for ones.  The
 * dequantised product is
 *   Y[m][n] = sum_k (xs[m][k/128] X[m][k]) * (ws[n/128][k/128] W[n][k]).
 * Scales are given as binary32 and taken exactly; A is the same sum over
 * absolute values.
 */
void orc_gemm_ref_scaled(const uint8_t *X, const uint8_t *W, uint64_t M, uint64_t N, uint64_t K,
                         const float *ws, const float *xs, uint64_t xs_cols, double *Y, double *A)
{
    double lut[256];
    const uint64_t kb = (K + 127) / 128;
    for (int i = 0; i < 256; i++) lut[i] = orc_e4m3_to_double((uint8_t)i);
    for (uint64_t m = 0; m < M; m++)
        for (uint64_t n = 0; n < N; n++) {
            double acc = 0.0, mag = 0.0;
            const uint8_t *x = X + m * K, *w = W + n * K;
            for (uint64_t k = 0; k < K; k++) {
                const double sx = !xs ? 1.0 : (double)xs[m * xs_cols + (xs_cols > 1 ? k / 128 : 0)];
                double p = (sx * lut[x[k]]) * ((double)ws[(n / 128) * kb + k / 128] * lut[w[k]]);
                acc += p;
                mag += fabs(p);
            }
            Y[m * N + n] = acc;
            A[m * N + n] = mag;
        }
}

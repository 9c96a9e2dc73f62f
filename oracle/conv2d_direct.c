/* TEST INFRASTRUCTURE ONLY -- CPU checker for the GPU library, not part of it.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may use it.
 *
 * conv2d as the plain definition (the "baseline conv2d" loop nest, step 1 of the
 * paper's Fig. 5; multiply-accumulate form of Fig. 1b; access [n, i + k] of
 * Table 2, i.e. cross-correlation without a kernel flip; 8-bit operands with
 * 32-bit accumulation as in Sec. 5.1):
 *
 *   out[n][k][p][q] = sum_{c,r,s} in0[n][c][p*stride + r - pad][q*stride + s - pad]
 *                                 * wt[k][c][r][s]
 *
 * in0 is `in` inside [0,H)x[0,W) and 0 outside.
 * P = floor((H + 2 pad - R)/stride) + 1, Q likewise from W and S.
 * Operands are signed; each is widened to int32 before the product.
 * No tiling, packing, im2col or reordering: seven loops in definition order.
 */
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

/* Returns 0, or -1 for arguments outside the definition's domain. */
int oracle_conv2d_int8(int N, int C, int H, int W, int K, int R, int S,
                       int stride, int pad,
                       const int8_t *in, const int8_t *wt, int32_t *out)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0 ||
        stride <= 0 || pad < 0 || R > H + 2 * pad || S > W + 2 * pad ||
        !in || !wt || !out)
        return -1;
    const int P = (H + 2 * pad - R) / stride + 1;
    const int Q = (W + 2 * pad - S) / stride + 1;
    const long planes = (long)N * K;

#pragma omp parallel for collapse(2) schedule(static)
    for (long nk = 0; nk < planes; ++nk) {
        for (int p = 0; p < P; ++p) {
            const int n = (int)(nk / K), k = (int)(nk % K);
            for (int q = 0; q < Q; ++q) {
                int32_t acc = 0;
                for (int c = 0; c < C; ++c)
                    for (int r = 0; r < R; ++r)
                        for (int s = 0; s < S; ++s) {
                            const int h = p * stride + r - pad;
                            const int w = q * stride + s - pad;
                            if (h < 0 || h >= H || w < 0 || w >= W) continue;
                            const int32_t x = in[(((size_t)n * C + c) * H + h) * W + w];
                            const int32_t y = wt[(((size_t)k * C + c) * R + r) * S + s];
                            acc += x * y;
                        }
                out[(((size_t)n * K + k) * P + p) * Q + q] = acc;
            }
        }
    }
    return 0;
}

/* Dilated convolution by its definition (Sec. 6.1 adds dilated convolutions to the
 * workloads; the access of Table 2 with the kernel index scaled, [n, i + d*k]):
 *
 *   out[n][k][p][q] = sum_{c,r,s} in0[n][c][p*stride + r*dilation - pad][q*stride + s*dilation - pad]
 *                                 * wt[k][c][r][s]
 *
 * P = floor((H + 2 pad - dilation*(R-1) - 1)/stride) + 1, Q likewise.  dilation = 1 is the
 * function above.  Returns 0, or -1 for arguments outside the definition's domain. */
int oracle_conv2d_int8_dilated(int N, int C, int H, int W, int K, int R, int S,
                               int stride, int pad, int dilation,
                               const int8_t *in, const int8_t *wt, int32_t *out)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0 ||
        stride <= 0 || pad < 0 || dilation <= 0 || !in || !wt || !out)
        return -1;
    const int Re = dilation * (R - 1) + 1, Se = dilation * (S - 1) + 1; /* extent of the spread kernel */
    if (Re > H + 2 * pad || Se > W + 2 * pad) return -1;
    const int P = (H + 2 * pad - Re) / stride + 1;
    const int Q = (W + 2 * pad - Se) / stride + 1;
    const long planes = (long)N * K;

#pragma omp parallel for collapse(2) schedule(static)
    for (long nk = 0; nk < planes; ++nk) {
        for (int p = 0; p < P; ++p) {
            const int n = (int)(nk / K), k = (int)(nk % K);
            for (int q = 0; q < Q; ++q) {
                int32_t acc = 0;
                for (int c = 0; c < C; ++c)
                    for (int r = 0; r < R; ++r)
                        for (int s = 0; s < S; ++s) {
                            const int h = p * stride + r * dilation - pad;
                            const int w = q * stride + s * dilation - pad;
                            if (h < 0 || h >= H || w < 0 || w >= W) continue;
                            const int32_t x = in[(((size_t)n * C + c) * H + h) * W + w];
                            const int32_t y = wt[(((size_t)k * C + c) * R + r) * S + s];
                            acc += x * y;
                        }
                out[(((size_t)n * K + k) * P + p) * Q + q] = acc;
            }
        }
    }
    return 0;
}

/*
 * CPU oracle, fifth part: the convolutional feed-forward network (ConvFFN) that
 * precedes every ConvAttn module in the residual step of the ESC block,
 *
 *     F_{i,j} = F_{i,j-1} + ConvAttn_j(ConvFFN_j(F_{i,j-1}), LK)        (Eq. 3, line 3)
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT: plain definitions as direct
 * loops with double accumulators, sharing no code with the HIP library; only
 * the tests, the smoke check and the benchmark's cpu_baseline leg may use it.
 *
 * Readings taken here.  The paper (Sec. 3, the paragraph below Eq. 3) says only
 * that ConvFFN is the convolutional feed-forward network of the work it cites,
 * with a kernel size of three, and prints no equation for it.  The published
 * description of that network is a feed-forward network of two point-wise
 * layers with a depth-wise convolution branch between them:
 *
 *     U = gelu(W1 . F + b1)                       C   -> C_h channels, per pixel
 *     V = U + gelu(K (*) U + bk)                  depth-wise 3 x 3, zero padding 1
 *     Y = W2 . V + b2                             C_h -> C channels, per pixel
 *
 *   - gelu is the exact erf form, as in the kernel estimator;
 *   - (*) is cross-correlation with zero padding and stride 1, as everywhere
 *     in this oracle;
 *   - the width C_h of the hidden layer is the caller's (the paper does not
 *     print its expansion ratio);
 *   - weights are row-major [out, in], the depth-wise kernel is [C_h, 3, 3];
 *     every bias is optional (NULL = none).
 *
 * Layouts as in esc_oracle.c: tensors contiguous [N,C,H,W]; dtype 0 = float32
 * storage, 1 = bfloat16 bit patterns.  Results and intermediates are unrounded
 * doubles.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

static double ffn_load(const void *base, int dtype, size_t idx)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    uint32_t u = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double ffn_gelu(double v) { return 0.5 * v * (1.0 + erf(v / sqrt(2.0))); }

/*
 * First layer: u[n, m, q] = gelu(b1[m] + sum_c w1[m*C + c] * x[n, c, q]),  m < Ch.
 * u is [N, Ch, H*W] doubles.
 */
void esc_oracle_ffn_expand(const void *x, int dtype, int N, int C, int H, int W, int Ch,
                           const float *w1, const float *b1, double *u)
{
    const size_t P = (size_t)H * W;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < Ch; ++m)
            for (size_t q = 0; q < P; ++q) {
                double s = b1 ? (double)b1[m] : 0.0;
                for (int c = 0; c < C; ++c)
                    s += (double)w1[(size_t)m * C + c] * ffn_load(x, dtype, ((size_t)n * C + c) * P + q);
                u[((size_t)n * Ch + m) * P + q] = ffn_gelu(s);
            }
}

/*
 * The depth-wise branch: v[n, m, y, x] = u[n, m, y, x]
 *      + gelu(bk[m] + sum_{i,j<3} k[m*9 + i*3 + j] * u~[n, m, y+i-1, x+j-1]),
 * u~ = u extended by zeros.  u and v are [N, Ch, H, W] doubles.
 */
void esc_oracle_ffn_dwbranch(const double *u, int N, int Ch, int H, int W, const float *k,
                             const float *bk, double *v)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < Ch; ++m) {
            const double *pu = u + ((size_t)n * Ch + m) * H * W;
            double *pv = v + ((size_t)n * Ch + m) * H * W;
            for (int y = 0; y < H; ++y)
                for (int xx = 0; xx < W; ++xx) {
                    double s = bk ? (double)bk[m] : 0.0;
                    for (int i = 0; i < 3; ++i)
                        for (int j = 0; j < 3; ++j) {
                            const int yy = y + i - 1, xj = xx + j - 1;
                            if (yy < 0 || yy >= H || xj < 0 || xj >= W) continue;
                            s += (double)k[(size_t)m * 9 + i * 3 + j] * pu[(size_t)yy * W + xj];
                        }
                    pv[(size_t)y * W + xx] = pu[(size_t)y * W + xx] + ffn_gelu(s);
                }
        }
}

/*
 * Second layer: y[n, c, q] = b2[c] + sum_m w2[c*Ch + m] * v[n, m, q],  c < C.
 */
void esc_oracle_ffn_project(const double *v, int N, int C, int H, int W, int Ch,
                            const float *w2, const float *b2, double *y)
{
    const size_t P = (size_t)H * W;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (size_t q = 0; q < P; ++q) {
                double s = b2 ? (double)b2[c] : 0.0;
                for (int m = 0; m < Ch; ++m)
                    s += (double)w2[(size_t)c * Ch + m] * v[((size_t)n * Ch + m) * P + q];
                y[((size_t)n * C + c) * P + q] = s;
            }
}

/*
 * ConvFFN as a whole; out is [N, C, H, W] doubles.  Returns 0, or -1 when a
 * buffer could not be allocated or a shape is not positive.
 */
int esc_oracle_convffn_forward(const void *x, int dtype, int N, int C, int H, int W, int Ch,
                               const float *w1, const float *b1, const float *k, const float *bk,
                               const float *w2, const float *b2, double *out)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || Ch < 1) return -1;
    const size_t cnt = (size_t)N * Ch * H * W;
    double *u = (double *)malloc(cnt * sizeof(double));
    double *v = (double *)malloc(cnt * sizeof(double));
    if (!u || !v) {
        free(u);
        free(v);
        return -1;
    }
    esc_oracle_ffn_expand(x, dtype, N, C, H, W, Ch, w1, b1, u);
    esc_oracle_ffn_dwbranch(u, N, Ch, H, W, k, bk, v);
    esc_oracle_ffn_project(v, N, C, H, W, Ch, w2, b2, out);
    free(u);
    free(v);
    return 0;
}

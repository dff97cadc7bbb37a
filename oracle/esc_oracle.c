/*
 * CPU oracle for the ConvAttn forward pass of the ESC paper (Sec. 3,
 * "Convolutional Attention Module", Eq. 4, with the depth-wise large kernel
 * LK^s of the paragraph that introduces Eq. 5).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is the plain definition
 * written as direct loops with double accumulators, one function per line of
 * Eq. 4.  It shares no code with the HIP library and must only be used by the
 * tests, the smoke check and the benchmark's cpu_baseline leg.
 *
 * Readings of the paper taken here (the paper does not spell them out):
 *   - the operator written as a circled asterisk is cross-correlation with
 *     zero padding (Ks-1)/2 on each side, stride 1, so the output keeps HxW;
 *   - GAP runs over the attention slice only (Eq. 4, line 2);
 *   - the kernel estimator is either the paper's two 1x1 convolutions with an
 *     exact (erf) GELU between them (hidden > 0) or the single linear layer of
 *     the benchmark workloads (hidden == 0);
 *   - the 9*Ca estimator outputs are laid out channel-major: o = c*9 + i*3 + j;
 *   - DK and LK are convolved separately and summed (Eq. 4, line 3); the
 *     merged form of Eq. 5 is checked against this in the tests, not used.
 *
 * Layouts: x/out contiguous [N,C,H,W]; lk [Ca,Ks,Ks] with channel stride
 * lk_cstride (0 = one Ks x Ks filter for every channel); dk [N,Ca,3,3].
 * dtype 0 = float32 storage, 1 = bfloat16 storage (uint16 bit patterns).
 * Every function is pinned by tests/test_oracle_*.py (closed forms, FFT,
 * separable kernels, a library grouped convolution).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

/* ---- storage helpers ---------------------------------------------------- */

static double load_elem(const void *base, int dtype, size_t idx)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    uint32_t u = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* float32 -> bfloat16, round to nearest, ties to even; NaN stays NaN. */
uint16_t esc_oracle_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

/* ---- Eq. 4, line 2, first half: global average pooling ------------------- */

/* g[n*Ca + c] = mean over (y,x) of x[n,c,y,x], for c < Ca. */
void esc_oracle_gap(const void *x, int dtype, int N, int C, int H, int W, int Ca, double *g)
{
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < Ca; ++c) {
            size_t base = ((size_t)n * C + c) * H * W;
            double s = 0.0;
            for (int y = 0; y < H; ++y)
                for (int xx = 0; xx < W; ++xx)
                    s += load_elem(x, dtype, base + (size_t)y * W + xx);
            g[(size_t)n * Ca + c] = s / ((double)H * (double)W);
        }
}

/* ---- Eq. 4, line 2, second half: the kernel estimator -------------------- */

static double gelu_exact(double v)
{
    return 0.5 * v * (1.0 + erf(v / sqrt(2.0)));
}

/*
 * hidden == 0: d = w_up[9Ca, Ca] g + b_up.
 * hidden  > 0: d = w_up[9Ca, hidden] gelu(w_down[hidden, Ca] g + b_down) + b_up.
 * dk[n, c, i, j] = d[n, c*9 + i*3 + j].  Bias pointers may be NULL (zero bias).
 */
void esc_oracle_generator(const double *g, int N, int Ca, int hidden,
                          const float *w_down, const float *b_down,
                          const float *w_up, const float *b_up, double *dk)
{
    double t[4096];
    for (int n = 0; n < N; ++n) {
        const double *gn = g + (size_t)n * Ca;
        const double *in = gn;
        int K = Ca;
        if (hidden > 0) {
            for (int m = 0; m < hidden; ++m) {
                double s = b_down ? (double)b_down[m] : 0.0;
                for (int k = 0; k < Ca; ++k)
                    s += (double)w_down[(size_t)m * Ca + k] * gn[k];
                t[m] = gelu_exact(s);
            }
            in = t;
            K = hidden;
        }
        for (int o = 0; o < 9 * Ca; ++o) {
            double s = b_up ? (double)b_up[o] : 0.0;
            for (int k = 0; k < K; ++k)
                s += (double)w_up[(size_t)o * K + k] * in[k];
            dk[(size_t)n * 9 * Ca + o] = s;
        }
    }
}

/* ---- Eq. 4, line 3: one depth-wise "same" cross-correlation -------------- */

/*
 * res[n,c,y,x] (+)= sum_{i,j<K} ker(n,c)[i,j] * xz[n,c, y+i-p, x+j-p],
 * p = (K-1)/2, xz = x extended by zeros.  ker(n,c) = k + n*k_nstride +
 * c*k_cstride (doubles if k_is_double else floats).  accumulate != 0 adds to
 * res instead of overwriting it.
 */
static void depthwise_same(const void *x, int dtype, int N, int C, int H, int W, int Ca,
                           const void *k, int k_is_double, int K,
                           size_t k_nstride, size_t k_cstride,
                           double *res, int accumulate)
{
    const int p = (K - 1) / 2;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < Ca; ++c) {
            size_t xbase = ((size_t)n * C + c) * H * W;
            size_t rbase = ((size_t)n * Ca + c) * H * W;
            size_t kbase = (size_t)n * k_nstride + (size_t)c * k_cstride;
            for (int y = 0; y < H; ++y)
                for (int xx = 0; xx < W; ++xx) {
                    double s = 0.0;
                    for (int i = 0; i < K; ++i) {
                        int yy = y + i - p;
                        if (yy < 0 || yy >= H)
                            continue;
                        for (int j = 0; j < K; ++j) {
                            int xj = xx + j - p;
                            if (xj < 0 || xj >= W)
                                continue;
                            double w = k_is_double
                                           ? ((const double *)k)[kbase + (size_t)i * K + j]
                                           : (double)((const float *)k)[kbase + (size_t)i * K + j];
                            s += w * load_elem(x, dtype, xbase + (size_t)yy * W + xj);
                        }
                    }
                    size_t o = rbase + (size_t)y * W + xx;
                    res[o] = accumulate ? res[o] + s : s;
                }
        }
}

/* F_att (*) LK alone: res[N,Ca,H,W] doubles. */
void esc_oracle_lk_conv(const void *x, int dtype, int N, int C, int H, int W, int Ca,
                        const float *lk, int Ks, long lk_cstride, double *res)
{
    depthwise_same(x, dtype, N, C, H, W, Ca, lk, 0, Ks, 0, (size_t)lk_cstride, res, 0);
}

/* F_att (*) DK alone, DK given per image as doubles [N,Ca,3,3]. */
void esc_oracle_dk_conv(const void *x, int dtype, int N, int C, int H, int W, int Ca,
                        const double *dk, double *res)
{
    depthwise_same(x, dtype, N, C, H, W, Ca, dk, 1, 3, (size_t)9 * Ca, 9, res, 0);
}

/* ---- Eq. 4, lines 1-4 without the fuse convolution ----------------------- */

/*
 * Full forward.  gen_mode: 0 = DK is zero, 1 = DK from the estimator (weights
 * given), 2 = DK taken from dk_in (doubles, [N,Ca,3,3]).
 *   res_att  [N,Ca,H,W] doubles, unrounded F_res                    (required)
 *   dk_out   [N,Ca,3,3] doubles, the DK that was used               (may be NULL)
 *   out      [N,C,H,W] in the storage dtype: F_res rounded once to the
 *            storage type in channels < Ca, bit copies of x elsewhere (may be NULL)
 * Returns 0, or -1 on an argument the definition does not cover.
 */
int esc_oracle_convattn_forward(const void *x, int dtype, int N, int C, int H, int W, int Ca,
                                const float *lk, int Ks, long lk_cstride,
                                int gen_mode, int hidden,
                                const float *w_down, const float *b_down,
                                const float *w_up, const float *b_up,
                                const double *dk_in,
                                double *res_att, double *dk_out, void *out)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || Ca < 0 || Ca > C || Ks < 1 || (Ks % 2) == 0)
        return -1;
    if (hidden > 4096 || 9 * Ca > 4096)
        return -1;
    double dkbuf[4096];
    double gbuf[512];
    if (Ca > 512)
        return -1;
    size_t es = dtype == ORACLE_F32 ? 4 : 2;
    size_t plane = (size_t)H * W;

    /* line 3, large-kernel term: the same LK for every image */
    depthwise_same(x, dtype, N, C, H, W, Ca, lk, 0, Ks, 0, (size_t)lk_cstride, res_att, 0);

    /* line 2 then line 3, dynamic term: one DK per image */
    for (int n = 0; n < N; ++n) {
        const char *xn = (const char *)x + (size_t)n * C * plane * es;
        double *dkn = dkbuf;
        if (gen_mode == 1) {
            esc_oracle_gap(xn, dtype, 1, C, H, W, Ca, gbuf);
            esc_oracle_generator(gbuf, 1, Ca, hidden, w_down, b_down, w_up, b_up, dkbuf);
        } else if (gen_mode == 2) {
            for (int o = 0; o < 9 * Ca; ++o)
                dkbuf[o] = dk_in[(size_t)n * 9 * Ca + o];
        } else {
            for (int o = 0; o < 9 * Ca; ++o)
                dkbuf[o] = 0.0;
        }
        if (dk_out)
            for (int o = 0; o < 9 * Ca; ++o)
                dk_out[(size_t)n * 9 * Ca + o] = dkn[o];
        depthwise_same(xn, dtype, 1, C, H, W, Ca, dkn, 1, 3, 0, 9,
                       res_att + (size_t)n * Ca * plane, 1);
    }

    /* lines 1 and 4: split / concat.  Identity channels are copied bit for bit. */
    if (out) {
        for (int n = 0; n < N; ++n) {
            for (int c = 0; c < Ca; ++c)
                for (size_t q = 0; q < plane; ++q) {
                    double v = res_att[((size_t)n * Ca + c) * plane + q];
                    size_t o = ((size_t)n * C + c) * plane + q;
                    if (dtype == ORACLE_F32)
                        ((float *)out)[o] = (float)v;
                    else
                        ((uint16_t *)out)[o] = esc_oracle_f32_to_bf16((float)v);
                }
            size_t off = ((size_t)n * C + Ca) * plane * es;
            memcpy((char *)out + off, (const char *)x + off, (size_t)(C - Ca) * plane * es);
        }
    }
    return 0;
}

/* Number of OpenMP threads the loops above will use (1 when built without it). */
#ifdef _OPENMP
#include <omp.h>
int esc_oracle_threads(void) { return omp_get_max_threads(); }
void esc_oracle_set_threads(int t) { if (t > 0) omp_set_num_threads(t); }
#else
int esc_oracle_threads(void) { return 1; }
void esc_oracle_set_threads(int t) { (void)t; }
#endif

/*
 * CPU oracle, second part: the point-wise (1x1) steps around the depth-wise
 * convolutions of the ConvAttn module of the ESC paper (Sec. 3):
 *
 *   - Conv_fuse 1x1 on Concat(F_res, F_idt)                    (Eq. 4, line 4)
 *   - the point-wise large-kernel filter LK^c that precedes the depth-wise
 *     LK^s in the decomposed form
 *         F_res = (F_att (*) LK^c) (*) (ZP(DK) + LK^s)                 (Eq. 5)
 *   - the residual connection around the module, F + ConvAttn(..)  (Eq. 3, line 3)
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT: plain definitions as direct
 * loops with double accumulators, sharing no code with the HIP library; only
 * the tests, the smoke check and the benchmark's cpu_baseline leg may use it.
 * It is linked with esc_oracle.c and uses that file's GAP and estimator.
 *
 * Readings of the paper taken here (it does not spell them out):
 *   - a 1x1 convolution is out[co] = b[co] + sum_ci w[co, ci] * in[ci] at every
 *     pixel, weights row-major [out, in]; biases are optional (NULL = none);
 *   - Conv_fuse maps C channels to C channels (the residual add of Eq. 3 needs
 *     equal shapes); LK^c maps the C_a attention channels to C_a channels and
 *     has no bias (it is one factor of a separable filter);
 *   - in Eq. 5 the point-wise filter comes first and BOTH depth-wise kernels,
 *     DK and LK^s, act on its output (the equation applies their sum to
 *     F_att (*) LK^c); DK itself is still estimated from GAP(F_att), the
 *     unfiltered slice, as Eq. 4 line 2 says;
 *   - ZP(DK) + LK^s is evaluated as two separate depth-wise convolutions summed
 *     (zero padding makes them equal; the tests check that equality);
 *   - the residual of Eq. 3 is a tensor of its own (F_{i,j-1}), not the
 *     module's input (ConvFFN's output).
 *
 * Layouts as in esc_oracle.c: tensors contiguous [N,C,H,W]; dtype 0 = float32
 * storage, 1 = bfloat16 bit patterns.  Results are unrounded doubles.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

/* from esc_oracle.c */
void esc_oracle_gap(const void *x, int dtype, int N, int C, int H, int W, int Ca, double *g);
void esc_oracle_generator(const double *g, int N, int Ca, int hidden, const float *w_down,
                          const float *b_down, const float *w_up, const float *b_up, double *dk);

static double load_stored(const void *base, int dtype, size_t idx)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    uint32_t u = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* ---- Eq. 5, first factor: F_att (*) LK^c -------------------------------- */

/*
 * pw[n, co, y, x] = sum_{ci < Ca} lkc[co*Ca + ci] * x[n, ci, y, x]   for co < Ca.
 * x is [N,C,H,W] in the storage dtype (only its first Ca channels are read);
 * pw is [N,Ca,H,W] doubles.
 */
void esc_oracle_pointwise_lkc(const void *x, int dtype, int N, int C, int H, int W, int Ca,
                              const float *lkc, double *pw)
{
    const size_t plane = (size_t)H * W;
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < Ca; ++co)
            for (size_t q = 0; q < plane; ++q) {
                double s = 0.0;
                for (int ci = 0; ci < Ca; ++ci)
                    s += (double)lkc[(size_t)co * Ca + ci] *
                         load_stored(x, dtype, ((size_t)n * C + ci) * plane + q);
                pw[((size_t)n * Ca + co) * plane + q] = s;
            }
}

/* ---- depth-wise "same" cross-correlation of double planes ---------------- */

/*
 * res[n,c,y,x] (+)= sum_{i,j<K} ker(n,c)[i,j] * inz[n,c, y+i-p, x+j-p], p = (K-1)/2,
 * inz = in extended by zeros; in and res are [N,Ca,H,W] doubles;
 * ker(n,c) = k + n*k_nstride + c*k_cstride (doubles if k_is_double, else floats).
 */
static void depthwise_same_f64(const double *in, int N, int Ca, int H, int W, const void *k,
                               int k_is_double, int K, size_t k_nstride, size_t k_cstride,
                               double *res, int accumulate)
{
    const int p = (K - 1) / 2;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < Ca; ++c) {
            const size_t base = ((size_t)n * Ca + c) * H * W;
            const size_t kbase = (size_t)n * k_nstride + (size_t)c * k_cstride;
            for (int y = 0; y < H; ++y)
                for (int xx = 0; xx < W; ++xx) {
                    double s = 0.0;
                    for (int i = 0; i < K; ++i) {
                        const int yy = y + i - p;
                        if (yy < 0 || yy >= H)
                            continue;
                        for (int j = 0; j < K; ++j) {
                            const int xj = xx + j - p;
                            if (xj < 0 || xj >= W)
                                continue;
                            const double w = k_is_double
                                                 ? ((const double *)k)[kbase + (size_t)i * K + j]
                                                 : (double)((const float *)k)[kbase + (size_t)i * K + j];
                            s += w * in[base + (size_t)yy * W + xj];
                        }
                    }
                    const size_t o = base + (size_t)y * W + xx;
                    res[o] = accumulate ? res[o] + s : s;
                }
        }
}

/* ---- Eq. 4, line 4: Conv_fuse 1x1 ---------------------------------------- */

/*
 * out[n, co, q] = b[co] + sum_{ci < C} w[co*C + ci] * cat[n, ci, q]; cat and out
 * are [N,C,H,W] doubles; b may be NULL.
 */
void esc_oracle_fuse_1x1(const double *cat, int N, int C, int H, int W, const float *w,
                         const float *b, double *out)
{
    const size_t plane = (size_t)H * W;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < C; ++co)
            for (size_t q = 0; q < plane; ++q) {
                double s = b ? (double)b[co] : 0.0;
                for (int ci = 0; ci < C; ++ci)
                    s += (double)w[(size_t)co * C + ci] * cat[((size_t)n * C + ci) * plane + q];
                out[((size_t)n * C + co) * plane + q] = s;
            }
}

/* ---- the module with its point-wise steps --------------------------------- */

/*
 * Eq. 4 with line 3 in the form of Eq. 5 when lkc != NULL (and in its own form,
 * with the depth-wise LK, when lkc == NULL), line 4 in full, and the residual
 * of Eq. 3 when residual != NULL:
 *
 *   F_att, F_idt = Split(x)
 *   DK    = Estimator(GAP(F_att))        gen_mode 1; 2: dk_in as given; 0: zero
 *   F_pw  = F_att (*) LK^c               (F_att itself when lkc == NULL)
 *   F_res = F_pw (*) DK + F_pw (*) LK^s
 *   out   = Conv_fuse(Concat(F_res, F_idt)) [+ residual]
 *
 *   res_att [N,Ca,H,W] doubles, F_res (may be NULL)      dk_out [N,Ca,3,3] doubles (may be NULL)
 *   out     [N,C,H,W] doubles (required)                 residual [N,C,H,W] storage dtype or NULL
 * Returns 0, or -1 on an argument the definition does not cover or when memory runs out.
 */
int esc_oracle_convattn_fused_forward(const void *x, int dtype, int N, int C, int H, int W, int Ca,
                                      const float *lkc, const float *lk, int Ks, long lk_cstride,
                                      int gen_mode, int hidden, const float *w_down,
                                      const float *b_down, const float *w_up, const float *b_up,
                                      const double *dk_in, const float *w_fuse, const float *b_fuse,
                                      const void *residual, double *res_att, double *dk_out,
                                      double *out)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || Ca < 0 || Ca > C || Ks < 1 || (Ks % 2) == 0)
        return -1;
    if (Ca > 512 || hidden > 4096 || 9 * Ca > 4096 || w_fuse == NULL || out == NULL)
        return -1;
    const size_t plane = (size_t)H * W;
    double *pw = malloc(sizeof(double) * (size_t)N * (Ca > 0 ? Ca : 1) * plane);
    double *fres = malloc(sizeof(double) * (size_t)N * (Ca > 0 ? Ca : 1) * plane);
    double *cat = malloc(sizeof(double) * (size_t)N * C * plane);
    double *dk = malloc(sizeof(double) * (size_t)N * (Ca > 0 ? Ca : 1) * 9);
    double gbuf[512];
    if (!pw || !fres || !cat || !dk) {
        free(pw); free(fres); free(cat); free(dk);
        return -1;
    }

    /* line 2: DK per image from the unfiltered attention slice */
    for (int n = 0; n < N; ++n) {
        double *dkn = dk + (size_t)n * 9 * Ca;
        if (gen_mode == 1) {
            const size_t es = dtype == ORACLE_F32 ? 4 : 2;
            esc_oracle_gap((const char *)x + (size_t)n * C * plane * es, dtype, 1, C, H, W, Ca, gbuf);
            esc_oracle_generator(gbuf, 1, Ca, hidden, w_down, b_down, w_up, b_up, dkn);
        } else {
            for (int o = 0; o < 9 * Ca; ++o)
                dkn[o] = gen_mode == 2 ? dk_in[(size_t)n * 9 * Ca + o] : 0.0;
        }
    }
    if (dk_out)
        memcpy(dk_out, dk, sizeof(double) * (size_t)N * Ca * 9);

    /* Eq. 5, first factor (or F_att itself) */
    if (lkc) {
        esc_oracle_pointwise_lkc(x, dtype, N, C, H, W, Ca, lkc, pw);
    } else {
        for (int n = 0; n < N; ++n)
            for (int c = 0; c < Ca; ++c)
                for (size_t q = 0; q < plane; ++q)
                    pw[((size_t)n * Ca + c) * plane + q] =
                        load_stored(x, dtype, ((size_t)n * C + c) * plane + q);
    }

    /* line 3 / Eq. 5: the two depth-wise convolutions of F_pw, summed */
    depthwise_same_f64(pw, N, Ca, H, W, lk, 0, Ks, 0, (size_t)lk_cstride, fres, 0);
    depthwise_same_f64(pw, N, Ca, H, W, dk, 1, 3, (size_t)9 * Ca, 9, fres, 1);
    if (res_att)
        memcpy(res_att, fres, sizeof(double) * (size_t)N * Ca * plane);

    /* line 4: concat, then the fuse convolution */
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (size_t q = 0; q < plane; ++q)
                cat[((size_t)n * C + c) * plane + q] =
                    c < Ca ? fres[((size_t)n * Ca + c) * plane + q]
                           : load_stored(x, dtype, ((size_t)n * C + c) * plane + q);
    esc_oracle_fuse_1x1(cat, N, C, H, W, w_fuse, b_fuse, out);

    /* Eq. 3, line 3: the residual connection around the module */
    if (residual)
        for (size_t q = 0; q < (size_t)N * C * plane; ++q)
            out[q] += load_stored(residual, dtype, q);

    free(pw); free(fres); free(cat); free(dk);
    return 0;
}

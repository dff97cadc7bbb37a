/*
 * CPU oracle, third part: the ConvAttn module with the DENSE large kernel of the
 * ESC paper's main variants (Sec. 3: LK in R^{13x13x16x16}, shared by the whole
 * model; Eq. 4 line 3):
 *
 *   F_res = (F_att (*) DK) + (F_att (*) LK)
 *
 * with LK a full C_a -> C_a convolution and DK the depth-wise dynamic kernel,
 * kept as two separate convolutions (the paper: DK "can be merged into LK by
 * padding both spatial and channel dimensions ... we do not").
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT: the plain definition as direct
 * loops with double accumulators, sharing no code with the HIP library; only
 * the tests, the smoke check and the benchmark's cpu_baseline leg may use it.
 * Linked with esc_oracle.c, whose GAP, estimator and DK convolution it uses.
 *
 * Readings (the paper does not spell them out): cross-correlation, zero padding
 * (Ks-1)/2, stride 1, as for the depth-wise form; weight layout
 * lk[co][ci][i][j] row-major (output channel first), no bias.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

void esc_oracle_gap(const void *x, int dtype, int N, int C, int H, int W, int Ca, double *g);
void esc_oracle_generator(const double *g, int N, int Ca, int hidden, const float *w_down,
                          const float *b_down, const float *w_up, const float *b_up, double *dk);
void esc_oracle_dk_conv(const void *x, int dtype, int N, int C, int H, int W, int Ca,
                        const double *dk, double *res);
uint16_t esc_oracle_f32_to_bf16(float f);

static double load_px(const void *base, int dtype, size_t idx)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    uint32_t u = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/*
 * res[n,co,y,x] = sum_{ci<Ca} sum_{i,j<Ks} lk[co][ci][i][j] * xz[n,ci,y+i-p,x+j-p],
 * p = (Ks-1)/2, xz = x extended by zeros; res is [N,Ca,H,W] doubles.
 */
void esc_oracle_dense_lk_conv(const void *x, int dtype, int N, int C, int H, int W, int Ca,
                              const float *lk, int Ks, double *res)
{
    const int p = (Ks - 1) / 2;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < Ca; ++co)
            for (int y = 0; y < H; ++y)
                for (int xx = 0; xx < W; ++xx) {
                    double s = 0.0;
                    for (int ci = 0; ci < Ca; ++ci) {
                        const size_t xbase = ((size_t)n * C + ci) * H * W;
                        const float *k = lk + ((size_t)co * Ca + ci) * Ks * Ks;
                        for (int i = 0; i < Ks; ++i) {
                            const int yy = y + i - p;
                            if (yy < 0 || yy >= H)
                                continue;
                            for (int j = 0; j < Ks; ++j) {
                                const int xj = xx + j - p;
                                if (xj < 0 || xj >= W)
                                    continue;
                                s += (double)k[i * Ks + j] * load_px(x, dtype, xbase + (size_t)yy * W + xj);
                            }
                        }
                    }
                    res[(((size_t)n * Ca + co) * H + y) * W + xx] = s;
                }
}

/*
 * Eq. 4 lines 1-4 (without Conv_fuse) with the dense LK.  gen_mode: 0 = DK zero,
 * 1 = DK from the estimator, 2 = DK from dk_in (doubles).  res_att [N,Ca,H,W]
 * doubles (required); dk_out [N,Ca,3,3] doubles or NULL; out [N,C,H,W] storage
 * dtype or NULL (F_res rounded once, identity channels bit copies).
 * tmp: caller's scratch of N*Ca*H*W doubles.  Returns 0, or -1 on bad arguments.
 */
int esc_oracle_convattn_dense_forward(const void *x, int dtype, int N, int C, int H, int W, int Ca,
                                      const float *lk, int Ks, int gen_mode, int hidden,
                                      const float *w_down, const float *b_down, const float *w_up,
                                      const float *b_up, const double *dk_in, double *tmp,
                                      double *res_att, double *dk_out, void *out)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || Ca < 0 || Ca > C || Ks < 1 || (Ks % 2) == 0)
        return -1;
    if (Ca > 455 || hidden > 4096)
        return -1;
    static double dk[512 * 9 * 64];
    double gbuf[512];
    if ((size_t)N * Ca * 9 > sizeof dk / sizeof dk[0])
        return -1;
    const size_t plane = (size_t)H * W, es = dtype == ORACLE_F32 ? 4 : 2;
    for (int n = 0; n < N; ++n) {
        double *dkn = dk + (size_t)n * 9 * Ca;
        if (gen_mode == 1) {
            esc_oracle_gap((const char *)x + (size_t)n * C * plane * es, dtype, 1, C, H, W, Ca, gbuf);
            esc_oracle_generator(gbuf, 1, Ca, hidden, w_down, b_down, w_up, b_up, dkn);
        } else {
            for (int o = 0; o < 9 * Ca; ++o)
                dkn[o] = gen_mode == 2 ? dk_in[(size_t)n * 9 * Ca + o] : 0.0;
        }
    }
    if (dk_out)
        memcpy(dk_out, dk, sizeof(double) * (size_t)N * Ca * 9);
    /* line 3: the two convolutions, separately, then their sum */
    esc_oracle_dense_lk_conv(x, dtype, N, C, H, W, Ca, lk, Ks, res_att);
    esc_oracle_dk_conv(x, dtype, N, C, H, W, Ca, dk, tmp);
    for (size_t q = 0; q < (size_t)N * Ca * plane; ++q)
        res_att[q] += tmp[q];
    /* lines 1 and 4 */
    if (out) {
        for (int n = 0; n < N; ++n) {
            for (int c = 0; c < Ca; ++c)
                for (size_t q = 0; q < plane; ++q) {
                    const double v = res_att[((size_t)n * Ca + c) * plane + q];
                    const size_t o = ((size_t)n * C + c) * plane + q;
                    if (dtype == ORACLE_F32)
                        ((float *)out)[o] = (float)v;
                    else
                        ((uint16_t *)out)[o] = esc_oracle_f32_to_bf16((float)v);
                }
            const size_t off = ((size_t)n * C + Ca) * plane * es;
            memcpy((char *)out + off, (const char *)x + off, (size_t)(C - Ca) * plane * es);
        }
    }
    return 0;
}

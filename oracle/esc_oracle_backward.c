/*
 * CPU oracle, fourth part: the backward pass of the ConvAttn module of the ESC
 * paper in its depth-wise form (Sec. 3, Eq. 4 lines 1-4 without Conv_fuse; the
 * paper trains LK end to end, so the module needs gradients, but prints no
 * formulae: these are the derivatives of the definition, written out).
 *
 * Forward, per image n and attention channel c (p = (Ks-1)/2, xz = x extended by zeros):
 *   g[n,c]   = mean_{y,x} x[n,c,y,x]
 *   u[n,m]   = b_down[m] + sum_k w_down[m,k] g[n,k]     t = gelu(u)        (hidden > 0)
 *   d[n,o]   = b_up[o] + sum_k w_up[o,k] t[n,k]         (t = g when hidden == 0)
 *   DK[n,c,i,j] = d[n, c*9 + i*3 + j]
 *   out[n,c,y,x] = sum_{i,j<Ks} LK[c,i,j] xz[n,c,y+i-p,x+j-p] + sum_{i,j<3} DK[n,c,i,j] xz[n,c,y+i-1,x+j-1]
 *   out[n,c] = x[n,c]  for c >= Ca
 *
 * Backward, given go = dL/dout:
 *   dLK[c,i,j]    = sum_{n,y,x} go[n,c,y,x] xz[n,c,y+i-p,x+j-p]
 *   dDK[n,c,i,j]  = sum_{y,x}   go[n,c,y,x] xz[n,c,y+i-1,x+j-1]
 *   dd = dDK flattened;  db_up[o] = sum_n dd[n,o];  dw_up[o,k] = sum_n dd[n,o] t[n,k];  dt[n,k] = sum_o w_up[o,k] dd[n,o]
 *   hidden > 0: du = dt * gelu'(u);  db_down = sum_n du;  dw_down[m,k] = sum_n du[n,m] g[n,k];  dg[n,k] = sum_m w_down[m,k] du[n,m]
 *   hidden == 0: dg = dt
 *   dx[n,c,y,x]   = sum_{i,j<Ks} LK[c,i,j] goz[n,c,y-i+p,x-j+p] + sum_{i,j<3} DK[n,c,i,j] goz[n,c,y-i+1,x-j+1] + dg[n,c] / (H W)
 *   dx[n,c] = go[n,c]  for c >= Ca
 * gelu'(v) = 0.5 (1 + erf(v / sqrt 2)) + v exp(-v^2 / 2) / sqrt(2 pi).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT: direct loops, double accumulators,
 * no code shared with the HIP library; only tests, the smoke check and the
 * benchmark's cpu_baseline leg may use it.  Linked with esc_oracle.c.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

void esc_oracle_gap(const void *x, int dtype, int N, int C, int H, int W, int Ca, double *g);

static double ld(const void *base, int dtype, size_t idx)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    uint32_t u = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/*
 * All pointers host memory.  x, go: [N,C,H,W] storage dtype.  lk [Ca,Ks,Ks] floats with
 * channel stride lk_cstride (0 = one filter for all channels: then dlk is [Ks,Ks], summed
 * over the channels too).  Estimator weights as in the forward (gen_mode 1), or gen_mode 2
 * with dk_in (doubles; no estimator gradients), or gen_mode 0 (DK = 0).
 * Outputs (doubles; any may be NULL): dx [N,C,H,W], dlk, ddk [N,Ca,3,3], dw_up, db_up,
 * dw_down, db_down, dg [N,Ca].
 * Returns 0, or -1 on bad arguments or when memory runs out.
 */
int esc_oracle_convattn_backward(const void *x, const void *go, int dtype, int N, int C, int H, int W,
                                 int Ca, const float *lk, int Ks, long lk_cstride, int gen_mode,
                                 int hidden, const float *w_down, const float *b_down,
                                 const float *w_up, const float *b_up, const double *dk_in,
                                 double *dx, double *dlk, double *ddk_out, double *dw_up,
                                 double *db_up, double *dw_down, double *db_down, double *dg_out)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || Ca < 0 || Ca > C || Ks < 1 || (Ks % 2) == 0 || hidden < 0)
        return -1;
    const int p = (Ks - 1) / 2;
    const size_t plane = (size_t)H * W;
    const int K = hidden > 0 ? hidden : Ca;
    double *g = calloc((size_t)N * (Ca + 1), sizeof(double));
    double *u = calloc((size_t)N * (hidden + 1), sizeof(double));
    double *t = calloc((size_t)N * (K + 1), sizeof(double));
    double *dk = calloc((size_t)N * (Ca + 1) * 9, sizeof(double));
    double *ddk = calloc((size_t)N * (Ca + 1) * 9, sizeof(double));
    double *dg = calloc((size_t)N * (Ca + 1), sizeof(double));
    if (!g || !u || !t || !dk || !ddk || !dg) {
        free(g); free(u); free(t); free(dk); free(ddk); free(dg);
        return -1;
    }
    /* forward quantities the derivatives need */
    if (gen_mode == 1) {
        esc_oracle_gap(x, dtype, N, C, H, W, Ca, g);
        for (int n = 0; n < N; ++n) {
            if (hidden > 0)
                for (int m = 0; m < hidden; ++m) {
                    double s = b_down ? (double)b_down[m] : 0.0;
                    for (int k = 0; k < Ca; ++k)
                        s += (double)w_down[(size_t)m * Ca + k] * g[(size_t)n * Ca + k];
                    u[(size_t)n * hidden + m] = s;
                    t[(size_t)n * K + m] = 0.5 * s * (1.0 + erf(s / sqrt(2.0)));
                }
            else
                for (int k = 0; k < Ca; ++k)
                    t[(size_t)n * K + k] = g[(size_t)n * Ca + k];
            for (int o = 0; o < 9 * Ca; ++o) {
                double s = b_up ? (double)b_up[o] : 0.0;
                for (int k = 0; k < K; ++k)
                    s += (double)w_up[(size_t)o * K + k] * t[(size_t)n * K + k];
                dk[(size_t)n * 9 * Ca + o] = s;
            }
        }
    } else if (gen_mode == 2) {
        for (size_t q = 0; q < (size_t)N * Ca * 9; ++q)
            dk[q] = dk_in[q];
    }

    /* gradients of the two kernels: correlations of go with x */
    const size_t dlk_len = lk_cstride != 0 ? (size_t)Ca * Ks * Ks : (size_t)Ks * Ks;
    if (dlk)
        for (size_t q = 0; q < dlk_len; ++q)
            dlk[q] = 0.0;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < Ca; ++c) {
            const size_t base = ((size_t)n * C + c) * plane;
            if (dlk) {
                double *dst = dlk + (lk_cstride != 0 ? (size_t)c * Ks * Ks : 0);
#pragma omp parallel for collapse(2) schedule(static)
                for (int i = 0; i < Ks; ++i)
                    for (int j = 0; j < Ks; ++j) {
                        double s = 0.0;
                        for (int y = 0; y < H; ++y) {
                            const int yy = y + i - p;
                            if (yy < 0 || yy >= H)
                                continue;
                            for (int xx = 0; xx < W; ++xx) {
                                const int xj = xx + j - p;
                                if (xj < 0 || xj >= W)
                                    continue;
                                s += ld(go, dtype, base + (size_t)y * W + xx) * ld(x, dtype, base + (size_t)yy * W + xj);
                            }
                        }
                        dst[i * Ks + j] += s;
                    }
            }
            for (int i = 0; i < 3; ++i)
                for (int j = 0; j < 3; ++j) {
                    double s = 0.0;
                    for (int y = 0; y < H; ++y) {
                        const int yy = y + i - 1;
                        if (yy < 0 || yy >= H)
                            continue;
                        for (int xx = 0; xx < W; ++xx) {
                            const int xj = xx + j - 1;
                            if (xj < 0 || xj >= W)
                                continue;
                            s += ld(go, dtype, base + (size_t)y * W + xx) * ld(x, dtype, base + (size_t)yy * W + xj);
                        }
                    }
                    ddk[((size_t)n * Ca + c) * 9 + i * 3 + j] = s;
                }
        }
    if (ddk_out)
        memcpy(ddk_out, ddk, sizeof(double) * (size_t)N * Ca * 9);

    /* the estimator, backwards */
    if (gen_mode == 1) {
        if (dw_up) for (size_t q = 0; q < (size_t)9 * Ca * K; ++q) dw_up[q] = 0.0;
        if (db_up) for (int o = 0; o < 9 * Ca; ++o) db_up[o] = 0.0;
        if (dw_down) for (size_t q = 0; q < (size_t)hidden * Ca; ++q) dw_down[q] = 0.0;
        if (db_down) for (int m = 0; m < hidden; ++m) db_down[m] = 0.0;
        double *dt = calloc((size_t)K + 1, sizeof(double));
        double *du = calloc((size_t)hidden + 1, sizeof(double));
        if (!dt || !du) {
            free(dt); free(du); free(g); free(u); free(t); free(dk); free(ddk); free(dg);
            return -1;
        }
        for (int n = 0; n < N; ++n) {
            const double *dd = ddk + (size_t)n * 9 * Ca;
            for (int k = 0; k < K; ++k)
                dt[k] = 0.0;
            for (int o = 0; o < 9 * Ca; ++o) {
                if (db_up) db_up[o] += dd[o];
                for (int k = 0; k < K; ++k) {
                    if (dw_up) dw_up[(size_t)o * K + k] += dd[o] * t[(size_t)n * K + k];
                    dt[k] += (double)w_up[(size_t)o * K + k] * dd[o];
                }
            }
            if (hidden > 0) {
                for (int m = 0; m < hidden; ++m) {
                    const double v = u[(size_t)n * hidden + m];
                    const double dgelu = 0.5 * (1.0 + erf(v / sqrt(2.0))) + v * exp(-0.5 * v * v) / sqrt(2.0 * 3.14159265358979323846);
                    du[m] = dt[m] * dgelu;
                    if (db_down) db_down[m] += du[m];
                    for (int k = 0; k < Ca; ++k) {
                        if (dw_down) dw_down[(size_t)m * Ca + k] += du[m] * g[(size_t)n * Ca + k];
                        dg[(size_t)n * Ca + k] += (double)w_down[(size_t)m * Ca + k] * du[m];
                    }
                }
            } else {
                for (int k = 0; k < Ca; ++k)
                    dg[(size_t)n * Ca + k] = dt[k];
            }
        }
        free(dt);
        free(du);
    }
    if (dg_out)
        memcpy(dg_out, dg, sizeof(double) * (size_t)N * Ca);

    /* gradient of the input */
    if (dx) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int n = 0; n < N; ++n)
            for (int c = 0; c < C; ++c) {
                const size_t base = ((size_t)n * C + c) * plane;
                if (c >= Ca) {
                    for (size_t q = 0; q < plane; ++q)
                        dx[base + q] = ld(go, dtype, base + q);
                    continue;
                }
                const float *k = lk + (size_t)c * lk_cstride;
                const double *d = dk + ((size_t)n * Ca + c) * 9;
                const double add = dg[(size_t)n * Ca + c] / ((double)H * (double)W);
                for (int y = 0; y < H; ++y)
                    for (int xx = 0; xx < W; ++xx) {
                        double s = add;
                        for (int i = 0; i < Ks; ++i) {
                            const int yy = y - i + p;
                            if (yy < 0 || yy >= H)
                                continue;
                            for (int j = 0; j < Ks; ++j) {
                                const int xj = xx - j + p;
                                if (xj < 0 || xj >= W)
                                    continue;
                                s += (double)k[i * Ks + j] * ld(go, dtype, base + (size_t)yy * W + xj);
                            }
                        }
                        for (int i = 0; i < 3; ++i) {
                            const int yy = y - i + 1;
                            if (yy < 0 || yy >= H)
                                continue;
                            for (int j = 0; j < 3; ++j) {
                                const int xj = xx - j + 1;
                                if (xj < 0 || xj >= W)
                                    continue;
                                s += d[i * 3 + j] * ld(go, dtype, base + (size_t)yy * W + xj);
                            }
                        }
                        dx[base + (size_t)y * W + xx] = s;
                    }
            }
    }
    free(g); free(u); free(t); free(dk); free(ddk); free(dg);
    return 0;
}

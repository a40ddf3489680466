/*
 * fp64 CPU oracle for the locally connected autoencoder path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the HIP kernels are
 * compared with: plain loops in definition order, double precision, no
 * blocking, no fusion.  Nothing in the product path may call it; it shares no
 * header, helper or constant with the GPU code.
 *
 * What each function follows:
 *   - layer geometry (valid receptive fields of size R, stride S, F filters
 *     per location, untied weights): Sec. 3.1, the paragraph on the network
 *     topology (300/16/4 -> 72x72 locations is exact "valid" arithmetic);
 *   - W x, W^T h, and the cost: Eq. 1 (RICA with offset b and scale alpha);
 *   - local contrast normalisation: named in Sec. 3.1 and not defined there;
 *     the reading taken here is Gaussian-windowed local standardisation with
 *     statistics pooled over channels (parity unpinned by the paper: pinned
 *     only by invariants and library special cases);
 *   - L2 pooling: not part of the paper's network (Sec. 3.1 leaves pooling
 *     out); defined here as the square root of the windowed sum of squares
 *     (parity unpinned by the paper, same remark).
 *
 * Layouts: activations [B][H][W][C] (C fastest); layer output [B][LH][LW][F];
 * weights [LH][LW][K][F] with k = (kh*R + kw)*C + c.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int n_loc(int H, int R, int S) { return (H - R) / S + 1; }

/* y[b,i,j,f] = alpha * sum_k W[i,j,k,f] * patch(b,i,j)[k] + bias[i,j,f]   (Eq. 1: alpha W x) */
void orc_lc_forward(int B, int H, int W, int C, int R, int S, int F,
                    const double *x, const double *w, const double *bias,
                    double alpha, double *y) {
    const int LH = n_loc(H, R, S), LW = n_loc(W, R, S), K = R * R * C;
#pragma omp parallel for collapse(2) schedule(static)
    for (int i = 0; i < LH; ++i)
        for (int j = 0; j < LW; ++j) {
            const double *wl = w + ((size_t)i * LW + j) * K * F;
            for (int b = 0; b < B; ++b)
                for (int f = 0; f < F; ++f) {
                    double acc = 0.0;
                    for (int kh = 0; kh < R; ++kh)
                        for (int kw = 0; kw < R; ++kw)
                            for (int c = 0; c < C; ++c) {
                                const int k = (kh * R + kw) * C + c;
                                const double xv = x[(((size_t)b * H + i * S + kh) * W + j * S + kw) * C + c];
                                acc += wl[(size_t)k * F + f] * xv;
                            }
                    double out = alpha * acc;
                    if (bias) out += bias[((size_t)i * LW + j) * F + f];
                    y[(((size_t)b * LH + i) * LW + j) * F + f] = out;
                }
        }
}

/* dx = 0; dx[b, i*S+kh, j*S+kw, c] += sum_f W[i,j,k,f] * dy[b,i,j,f]   (Eq. 1: W^T h, overlap-add) */
void orc_lc_backward_data(int B, int H, int W, int C, int R, int S, int F,
                          const double *dy, const double *w, double *dx) {
    const int LH = n_loc(H, R, S), LW = n_loc(W, R, S), K = R * R * C;
    (void)K;
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b) {
        double *dxb = dx + (size_t)b * H * W * C;
        memset(dxb, 0, sizeof(double) * (size_t)H * W * C);
        for (int i = 0; i < LH; ++i)
            for (int j = 0; j < LW; ++j) {
                const double *wl = w + ((size_t)i * LW + j) * (size_t)R * R * C * F;
                const double *dyl = dy + (((size_t)b * LH + i) * LW + j) * F;
                for (int kh = 0; kh < R; ++kh)
                    for (int kw = 0; kw < R; ++kw)
                        for (int c = 0; c < C; ++c) {
                            const int k = (kh * R + kw) * C + c;
                            double acc = 0.0;
                            for (int f = 0; f < F; ++f) acc += wl[(size_t)k * F + f] * dyl[f];
                            dxb[((size_t)(i * S + kh) * W + j * S + kw) * C + c] += acc;
                        }
            }
    }
}

/* dW[i,j,k,f] = beta*dW[i,j,k,f] + sum_b patch(b,i,j)[k] * dy[b,i,j,f] */
void orc_lc_backward_weights(int B, int H, int W, int C, int R, int S, int F,
                             const double *x, const double *dy, double beta, double *dw) {
    const int LH = n_loc(H, R, S), LW = n_loc(W, R, S), K = R * R * C;
#pragma omp parallel for collapse(2) schedule(static)
    for (int i = 0; i < LH; ++i)
        for (int j = 0; j < LW; ++j) {
            double *dwl = dw + ((size_t)i * LW + j) * K * F;
            for (int kh = 0; kh < R; ++kh)
                for (int kw = 0; kw < R; ++kw)
                    for (int c = 0; c < C; ++c) {
                        const int k = (kh * R + kw) * C + c;
                        for (int f = 0; f < F; ++f) {
                            double acc = 0.0;
                            for (int b = 0; b < B; ++b)
                                acc += x[(((size_t)b * H + i * S + kh) * W + j * S + kw) * C + c] *
                                       dy[(((size_t)b * LH + i) * LW + j) * F + f];
                            double *o = &dwl[(size_t)k * F + f];
                            *o = (beta != 0.0 ? beta * *o : 0.0) + acc;
                        }
                    }
        }
}

/* y[b,i,j,c] = sqrt(eps + sum_{p,q<ks} x[b,i*st+p,j*st+q,c]^2), no padding */
void orc_l2pool_fwd(int B, int H, int W, int C, int ks, int st, double eps,
                    const double *x, double *y) {
    const int Ho = n_loc(H, ks, st), Wo = n_loc(W, ks, st);
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b)
        for (int i = 0; i < Ho; ++i)
            for (int j = 0; j < Wo; ++j)
                for (int c = 0; c < C; ++c) {
                    double s = 0.0;
                    for (int p = 0; p < ks; ++p)
                        for (int q = 0; q < ks; ++q) {
                            const double v = x[(((size_t)b * H + i * st + p) * W + j * st + q) * C + c];
                            s += v * v;
                        }
                    y[(((size_t)b * Ho + i) * Wo + j) * C + c] = sqrt(eps + s);
                }
}

/* chain rule of the above: every window that contains an input adds x*dy/y */
void orc_l2pool_bwd(int B, int H, int W, int C, int ks, int st,
                    const double *x, const double *y, const double *dy, double *dx) {
    const int Ho = n_loc(H, ks, st), Wo = n_loc(W, ks, st);
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b) {
        double *dxb = dx + (size_t)b * H * W * C;
        memset(dxb, 0, sizeof(double) * (size_t)H * W * C);
        for (int i = 0; i < Ho; ++i)
            for (int j = 0; j < Wo; ++j)
                for (int c = 0; c < C; ++c) {
                    const size_t o = (((size_t)b * Ho + i) * Wo + j) * C + c;
                    const double g = dy[o] / y[o];
                    for (int p = 0; p < ks; ++p)
                        for (int q = 0; q < ks; ++q) {
                            const size_t xi = ((size_t)(i * st + p) * W + j * st + q) * C + c;
                            dxb[xi] += x[(size_t)b * H * W * C + xi] * g;
                        }
                }
    }
}

/* separable Gaussian window g[p] ~ exp(-p^2/(2 sigma^2)), p=-r..r, normalised to sum 1 */
static void gauss_taps(int ks, double sigma, double *g) {
    const int r = (ks - 1) / 2;
    double s = 0.0;
    for (int p = -r; p <= r; ++p) { g[p + r] = exp(-(double)(p * p) / (2.0 * sigma * sigma)); s += g[p + r]; }
    for (int p = 0; p < ks; ++p) g[p] /= s;
}

/*
 * Local contrast normalisation, the reading taken for Sec. 3.1's "LCN":
 *   mu  = window-weighted mean of x over the ks x ks neighbourhood and all C channels,
 *   m2  = the same mean of x^2, var = max(m2 - mu^2, 0), rstd = 1/sqrt(var+eps),
 *   y   = (x - mu) * rstd.
 * At the border the window is truncated and its weights renormalised.
 */
void orc_lcn_fwd(int B, int H, int W, int C, int ks, double sigma, double eps,
                 const double *x, double *y, double *mu, double *rstd) {
    const int r = (ks - 1) / 2;
    double g[64];
    gauss_taps(ks, sigma, g);
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b)
        for (int i = 0; i < H; ++i)
            for (int j = 0; j < W; ++j) {
                double Z = 0.0, s1 = 0.0, s2 = 0.0;
                for (int p = -r; p <= r; ++p)
                    for (int q = -r; q <= r; ++q) {
                        const int ii = i + p, jj = j + q;
                        if (ii < 0 || ii >= H || jj < 0 || jj >= W) continue;
                        const double wt = g[p + r] * g[q + r];
                        Z += wt;
                        const double *xp = x + (((size_t)b * H + ii) * W + jj) * C;
                        for (int c = 0; c < C; ++c) { s1 += wt * xp[c]; s2 += wt * xp[c] * xp[c]; }
                    }
                const double m = s1 / (C * Z), m2 = s2 / (C * Z);
                double var = m2 - m * m;
                if (var < 0.0) var = 0.0;
                const double rs = 1.0 / sqrt(var + eps);
                const size_t pix = ((size_t)b * H + i) * W + j;
                mu[pix] = m;
                rstd[pix] = rs;
                for (int c = 0; c < C; ++c) y[pix * C + c] = (x[pix * C + c] - m) * rs;
            }
}

/*
 * Chain rule of orc_lcn_fwd (the clamp of var is taken as inactive).
 * With t_p = sum_c dy[p,c], s_p = sum_c dy[p,c](x[p,c]-mu_p):
 *   dL/dmu_p = -rstd_p t_p + rstd_p^3 mu_p s_p,   dL/dm2_p = -rstd_p^3 s_p / 2,
 * and mu_p, m2_p depend on x[q,c] through the weight w[q-p]/(C Z_p).
 */
void orc_lcn_bwd(int B, int H, int W, int C, int ks, double sigma,
                 const double *x, const double *mu, const double *rstd,
                 const double *dy, double *dx) {
    const int r = (ks - 1) / 2;
    double g[64];
    gauss_taps(ks, sigma, g);
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b) {
        const size_t img = (size_t)b * H * W;
        for (size_t e = 0; e < (size_t)H * W * C; ++e) dx[img * C + e] = dy[img * C + e] * rstd[img + e / C];
        for (int i = 0; i < H; ++i)
            for (int j = 0; j < W; ++j) {
                const size_t p_ = img + (size_t)i * W + j;
                double Z = 0.0;
                for (int p = -r; p <= r; ++p)
                    for (int q = -r; q <= r; ++q) {
                        const int ii = i + p, jj = j + q;
                        if (ii < 0 || ii >= H || jj < 0 || jj >= W) continue;
                        Z += g[p + r] * g[q + r];
                    }
                double t = 0.0, s = 0.0;
                for (int c = 0; c < C; ++c) {
                    t += dy[p_ * C + c];
                    s += dy[p_ * C + c] * (x[p_ * C + c] - mu[p_]);
                }
                const double rs = rstd[p_], rs3 = rs * rs * rs;
                const double dmu = -rs * t + rs3 * mu[p_] * s;
                const double dm2 = -0.5 * rs3 * s;
                for (int p = -r; p <= r; ++p)
                    for (int q = -r; q <= r; ++q) {
                        const int ii = i + p, jj = j + q;
                        if (ii < 0 || ii >= H || jj < 0 || jj >= W) continue;
                        const double a = g[p + r] * g[q + r] / (C * Z);
                        const size_t q_ = img + (size_t)ii * W + jj;
                        for (int c = 0; c < C; ++c)
                            dx[q_ * C + c] += a * (dmu + dm2 * 2.0 * x[q_ * C + c]);
                    }
            }
    }
}

/*
 * Variants of the local contrast normalisation of Sec. 3.1 (the paper names LCN without defining it, so the
 * common published forms are provided beside orc_lcn_fwd).  flags:
 *   1  statistics per channel (window over space only) instead of pooled over all channels;
 *   2  zero-padded borders: pixels outside the image count as zeros and the window weights are NOT renormalised;
 *   4  two stages: subtractive (v = x - local mean of x), then divisive (v / sqrt(local mean of v^2 + eps)),
 *      where the local mean of v^2 uses every neighbour's own v.
 * Without flag 4 this is the one-stage form of orc_lcn_fwd: var = max(mean(x^2) - mean(x)^2, 0).
 * mu and rstd hold one value per pixel ([B,H,W]) when pooled, one per element ([B,H,W,C]) with flag 1.
 */
static double lcn_window_mean(int H, int W, int C, int ks, const double *g, int zero_pad, int per_channel,
                              const double *f /* one image [H,W,C] */, int i, int j, int c) {
    const int r = (ks - 1) / 2;
    double Z = 0.0, s = 0.0;
    for (int p = -r; p <= r; ++p)
        for (int q = -r; q <= r; ++q) {
            const int ii = i + p, jj = j + q;
            if (ii < 0 || ii >= H || jj < 0 || jj >= W) continue;
            const double wt = g[p + r] * g[q + r];
            Z += wt;
            const double *fp = f + ((size_t)ii * W + jj) * C;
            if (per_channel) s += wt * fp[c];
            else for (int cc = 0; cc < C; ++cc) s += wt * fp[cc];
        }
    if (zero_pad) Z = 1.0;              /* taps sum to one over the full window */
    return s / (per_channel ? Z : Z * C);
}

void orc_lcn_var_fwd(int B, int H, int W, int C, int ks, double sigma, double eps, unsigned flags,
                     const double *x, double *y, double *mu, double *rstd) {
    const int pc = (flags & 1u) != 0, zp = (flags & 2u) != 0, two = (flags & 4u) != 0;
    const int CS = pc ? C : 1;
    const size_t img = (size_t)H * W * C;
    double g[64];
    gauss_taps(ks, sigma, g);
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b) {
        const double *xb = x + b * img;
        double *f = (double *)malloc(img * sizeof(double));   /* x^2 (one stage) or v^2 (two stages) */
        double *mub = mu + (size_t)b * H * W * CS, *rsb = rstd + (size_t)b * H * W * CS;
        for (int i = 0; i < H; ++i)
            for (int j = 0; j < W; ++j)
                for (int c = 0; c < CS; ++c)
                    mub[((size_t)i * W + j) * CS + c] = lcn_window_mean(H, W, C, ks, g, zp, pc, xb, i, j, c);
        for (size_t e = 0; e < img; ++e) {
            const double m = mub[pc ? e : e / C];
            f[e] = two ? (xb[e] - m) * (xb[e] - m) : xb[e] * xb[e];
        }
        for (int i = 0; i < H; ++i)
            for (int j = 0; j < W; ++j)
                for (int c = 0; c < CS; ++c) {
                    const size_t s_ = ((size_t)i * W + j) * CS + c;
                    double var = lcn_window_mean(H, W, C, ks, g, zp, pc, f, i, j, c);
                    if (!two) { var -= mub[s_] * mub[s_]; if (var < 0.0) var = 0.0; }
                    rsb[s_] = 1.0 / sqrt(var + eps);
                }
        for (size_t e = 0; e < img; ++e) {
            const size_t s_ = pc ? e : e / C;
            y[b * img + e] = (xb[e] - mub[s_]) * rsb[s_];
        }
        free(f);
    }
}

/*
 * Chain rule of orc_lcn_var_fwd (the clamp of the one-stage variance is taken as inactive).  Statistic s (a
 * pixel, or a pixel and channel) owns the elements e(s) and draws on element q with weight a_s(q) = window
 * weight / normaliser of s.
 *   one stage:  b_s = sum_{e(s)} dy (x - mu_s);  dmu_s = -rstd_s sum_{e(s)} dy + rstd_s^3 mu_s b_s;
 *               dm2_s = -rstd_s^3 b_s / 2;       dx[q] = dy[q] rstd + sum_s a_s(q) (dmu_s + 2 x[q] dm2_s).
 *   two stages: dvar_s = -rstd_s^3 b_s / 2 with v in place of x - mu;
 *               dv[q] = dy[q] rstd + 2 v[q] sum_s a_s(q) dvar_s;   dx[q] = dv[q] - sum_s a_s(q) sum_{e(s)} dv.
 */
void orc_lcn_var_bwd(int B, int H, int W, int C, int ks, double sigma, unsigned flags,
                     const double *x, const double *mu, const double *rstd, const double *dy, double *dx) {
    const int pc = (flags & 1u) != 0, zp = (flags & 2u) != 0, two = (flags & 4u) != 0;
    const int CS = pc ? C : 1, CR = pc ? 1 : C, r = (ks - 1) / 2;
    const size_t img = (size_t)H * W * C;
    double g[64];
    gauss_taps(ks, sigma, g);
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b) {
        const double *xb = x + b * img, *dyb = dy + b * img;
        const double *mub = mu + (size_t)b * H * W * CS, *rsb = rstd + (size_t)b * H * W * CS;
        double *dxb = dx + b * img;
        double *dv = (double *)malloc(img * sizeof(double));
        for (size_t e = 0; e < img; ++e) dv[e] = dyb[e] * rsb[pc ? e : e / C];
        /* first sweep: every statistic scatters the gradient of its mean (one stage) and of its variance */
        for (int i = 0; i < H; ++i)
            for (int j = 0; j < W; ++j)
                for (int c = 0; c < CS; ++c) {
                    const size_t s_ = ((size_t)i * W + j) * CS + c;
                    double Z = 0.0;
                    for (int p = -r; p <= r; ++p)
                        for (int q = -r; q <= r; ++q) {
                            const int ii = i + p, jj = j + q;
                            if (ii < 0 || ii >= H || jj < 0 || jj >= W) continue;
                            Z += g[p + r] * g[q + r];
                        }
                    if (zp) Z = 1.0;
                    double t = 0.0, bs = 0.0;
                    for (int cc = 0; cc < CR; ++cc) {
                        const size_t e = s_ * CR + cc;
                        t += dyb[e];
                        bs += dyb[e] * (xb[e] - mub[s_]);
                    }
                    const double rs3 = rsb[s_] * rsb[s_] * rsb[s_];
                    const double dvar = -0.5 * rs3 * bs;
                    const double dmu = two ? 0.0 : -rsb[s_] * t + rs3 * mub[s_] * bs;
                    for (int p = -r; p <= r; ++p)
                        for (int q = -r; q <= r; ++q) {
                            const int ii = i + p, jj = j + q;
                            if (ii < 0 || ii >= H || jj < 0 || jj >= W) continue;
                            const double a = g[p + r] * g[q + r] / (Z * CR);
                            for (int cc = 0; cc < CR; ++cc) {
                                const size_t e = (((size_t)ii * W + jj) * CS + c) * CR + cc;
                                const double base = two ? xb[e] - mub[((size_t)ii * W + jj) * CS + c] : xb[e];
                                dv[e] += a * (dmu + 2.0 * base * dvar);
                            }
                        }
                }
        memcpy(dxb, dv, img * sizeof(double));
        if (two) {
            /* second sweep: v = x - mean(x), so each statistic takes the sum of dv over its elements back out */
            for (int i = 0; i < H; ++i)
                for (int j = 0; j < W; ++j)
                    for (int c = 0; c < CS; ++c) {
                        const size_t s_ = ((size_t)i * W + j) * CS + c;
                        double Z = 0.0, t = 0.0;
                        for (int p = -r; p <= r; ++p)
                            for (int q = -r; q <= r; ++q) {
                                const int ii = i + p, jj = j + q;
                                if (ii < 0 || ii >= H || jj < 0 || jj >= W) continue;
                                Z += g[p + r] * g[q + r];
                            }
                        if (zp) Z = 1.0;
                        for (int cc = 0; cc < CR; ++cc) t += dv[s_ * CR + cc];
                        for (int p = -r; p <= r; ++p)
                            for (int q = -r; q <= r; ++q) {
                                const int ii = i + p, jj = j + q;
                                if (ii < 0 || ii >= H || jj < 0 || jj >= W) continue;
                                const double a = g[p + r] * g[q + r] / (Z * CR);
                                for (int cc = 0; cc < CR; ++cc)
                                    dxb[(((size_t)ii * W + jj) * CS + c) * CR + cc] -= a * t;
                            }
                    }
        }
        free(dv);
    }
}

/*
 * RICA cost of Eq. 1 for one stage, divided by the batch size:
 *   h = alpha W x,  xh = W^T h + b,  J = (1/B) [ sum (xh-x)^2 + lambda sum sqrt(h^2 + eps_s) ].
 * h (size B*L*F) and r = xh - x (size B*H*W*C) are returned for the gradient.
 */
double orc_sae_cost(int B, int H, int W, int C, int R, int S, int F,
                    const double *x, const double *w, const double *b, double alpha,
                    double lambda, double eps_s, double *h, double *r) {
    const int LH = n_loc(H, R, S), LW = n_loc(W, R, S);
    const size_t nh = (size_t)B * LH * LW * F, nx = (size_t)B * H * W * C, img = (size_t)H * W * C;
    orc_lc_forward(B, H, W, C, R, S, F, x, w, NULL, alpha, h);
    orc_lc_backward_data(B, H, W, C, R, S, F, h, w, r);
    double rec = 0.0, sp = 0.0;
    for (size_t e = 0; e < nx; ++e) { r[e] += b[e % img] - x[e]; rec += r[e] * r[e]; }
    for (size_t e = 0; e < nh; ++e) sp += sqrt(h[e] * h[e] + eps_s);
    return (rec + lambda * sp) / B;
}

/*
 * Gradient of orc_sae_cost with respect to W (both uses of the tied weights),
 * b and alpha, written from the chain rule of Eq. 1:
 *   u  = dJ/dxh = 2 r / B,                 db = sum_b u,
 *   gh = dJ/dh  = W u + (lambda/B) h / sqrt(h^2+eps_s),
 *   dW = patch(u) h^T  (decoder use)  +  patch(x) (alpha gh)^T  (encoder use),
 *   dalpha = sum (h/alpha) gh  computed as sum a*gh with a = W x.
 * Returns J.  dw has the weight layout, db is [H][W][C].
 */
double orc_sae_grad(int B, int H, int W, int C, int R, int S, int F,
                    const double *x, const double *w, const double *b, double alpha,
                    double lambda, double eps_s,
                    double *dw, double *db, double *dalpha, double *h_out) {
    const int LH = n_loc(H, R, S), LW = n_loc(W, R, S);
    const size_t nh = (size_t)B * LH * LW * F, nx = (size_t)B * H * W * C, img = (size_t)H * W * C;
    double *h = (double *)malloc(sizeof(double) * nh);
    double *a = (double *)malloc(sizeof(double) * nh);
    double *gh = (double *)malloc(sizeof(double) * nh);
    double *u = (double *)malloc(sizeof(double) * nx);
    const double J = orc_sae_cost(B, H, W, C, R, S, F, x, w, b, alpha, lambda, eps_s, h, u);
    for (size_t e = 0; e < nx; ++e) u[e] *= 2.0 / B;
    for (size_t e = 0; e < img; ++e) db[e] = 0.0;
    for (size_t e = 0; e < nx; ++e) db[e % img] += u[e];
    orc_lc_forward(B, H, W, C, R, S, F, u, w, NULL, 1.0, gh);
    for (size_t e = 0; e < nh; ++e) gh[e] += (lambda / B) * h[e] / sqrt(h[e] * h[e] + eps_s);
    orc_lc_forward(B, H, W, C, R, S, F, x, w, NULL, 1.0, a);
    double da = 0.0;
    for (size_t e = 0; e < nh; ++e) da += a[e] * gh[e];
    *dalpha = da;
    orc_lc_backward_weights(B, H, W, C, R, S, F, u, h, 0.0, dw);
    for (size_t e = 0; e < nh; ++e) gh[e] *= alpha;
    orc_lc_backward_weights(B, H, W, C, R, S, F, x, gh, 1.0, dw);
    if (h_out) memcpy(h_out, h, sizeof(double) * nh);
    free(h); free(a); free(gh); free(u);
    return J;
}

/*
 * One plain SGD step on Eq. 1.  flags bit0: after the update rescale every
 * filter W[l,:,f] to unit Euclidean norm (the constraint of Eq. 1); bit1:
 * alpha is learned too.  w, b, alpha are updated in place; h_out receives the
 * features computed with the weights from before the update.
 */
double orc_sae_step(int B, int H, int W, int C, int R, int S, int F,
                    const double *x, double *w, double *b, double *alpha,
                    double lambda, double eps_s, double lr, unsigned flags, double *h_out) {
    const int LH = n_loc(H, R, S), LW = n_loc(W, R, S), K = R * R * C;
    const size_t nw = (size_t)LH * LW * K * F, img = (size_t)H * W * C;
    double *dw = (double *)malloc(sizeof(double) * nw);
    double *db = (double *)malloc(sizeof(double) * img);
    double da = 0.0;
    const double J = orc_sae_grad(B, H, W, C, R, S, F, x, w, b, *alpha, lambda, eps_s, dw, db, &da, h_out);
    for (size_t e = 0; e < nw; ++e) w[e] -= lr * dw[e];
    for (size_t e = 0; e < img; ++e) b[e] -= lr * db[e];
    if (flags & 2u) *alpha -= lr * da;
    if (flags & 1u) {
        for (size_t l = 0; l < (size_t)LH * LW; ++l)
            for (int f = 0; f < F; ++f) {
                double n2 = 0.0;
                for (int k = 0; k < K; ++k) { const double v = w[(l * K + k) * F + f]; n2 += v * v; }
                /* a filter that is all zeros has no direction to normalise: it stays as it is */
                const double inv = n2 > 0.0 ? 1.0 / sqrt(n2) : 0.0;
                for (int k = 0; k < K; ++k) w[(l * K + k) * F + f] *= inv;
            }
    }
    free(dw); free(db);
    return J;
}

/*
 * Single-output evaluations of the three layer primitives, taking the fp32
 * arrays as they are (up-cast element by element).  They let a test check a
 * sample of outputs of a full-size layer without converting or traversing the
 * whole problem.  Each is the definition above restricted to one output.
 */
double orc_lc_forward_at(int B, int H, int W, int C, int R, int S, int F,
                         const float *x, const float *w, const float *bias, double alpha,
                         int b, int i, int j, int f) {
    const int LW = n_loc(W, R, S);
    (void)B;
    const float *wl = w + ((size_t)i * LW + j) * (size_t)R * R * C * F;
    double acc = 0.0;
    for (int kh = 0; kh < R; ++kh)
        for (int kw = 0; kw < R; ++kw)
            for (int c = 0; c < C; ++c) {
                const int k = (kh * R + kw) * C + c;
                acc += (double)wl[(size_t)k * F + f] *
                       (double)x[(((size_t)b * H + i * S + kh) * W + j * S + kw) * C + c];
            }
    double out = alpha * acc;
    if (bias) out += (double)bias[((size_t)i * LW + j) * F + f];
    return out;
}

double orc_lc_backward_data_at(int B, int H, int W, int C, int R, int S, int F,
                               const float *dy, const float *w, int b, int row, int col, int c) {
    const int LH = n_loc(H, R, S), LW = n_loc(W, R, S);
    (void)B;
    double acc = 0.0;
    for (int i = 0; i < LH; ++i)
        for (int j = 0; j < LW; ++j) {
            const int kh = row - i * S, kw = col - j * S;
            if (kh < 0 || kh >= R || kw < 0 || kw >= R) continue;
            const int k = (kh * R + kw) * C + c;
            const float *wl = w + (((size_t)i * LW + j) * (size_t)R * R * C + k) * F;
            const float *dyl = dy + (((size_t)b * LH + i) * LW + j) * F;
            for (int f = 0; f < F; ++f) acc += (double)wl[f] * (double)dyl[f];
        }
    return acc;
}

double orc_lc_backward_weights_at(int B, int H, int W, int C, int R, int S, int F,
                                  const float *x, const float *dy, int i, int j, int k, int f) {
    const int LH = n_loc(H, R, S), LW = n_loc(W, R, S);
    const int c = k % C, kw = (k / C) % R, kh = k / (C * R);
    double acc = 0.0;
    for (int b = 0; b < B; ++b)
        acc += (double)x[(((size_t)b * H + i * S + kh) * W + j * S + kw) * C + c] *
               (double)dy[(((size_t)b * LH + i) * LW + j) * F + f];
    return acc;
}

/*
 * CPU oracle: layer arithmetic of one back-propagation step (paper section 2.1:
 * forward propagation, backward propagation), written as the plain definition of
 * every layer.  TEST INFRASTRUCTURE ONLY: nothing in the product path links, loads
 * or calls this file; it shares no code with the HIP library.
 *
 * The paper inherits its layer mathematics from the framework it extends
 * (section 5, first paragraph) and defines none of it, so each layer here is the
 * textbook definition:
 *   conv      cross-correlation, zero padding, no dilation, no groups, no bias
 *   BN        training mode: per-channel mean and biased variance over batch x space
 *   ReLU      y = x > 0 ? x : 0, gradient 0 at x <= 0
 *   maxpool   -inf padding, first maximal element in (d,h,w) scan order wins ties
 *   FC        y = x W^T + b
 *   loss      softmax cross-entropy, mean over the batch
 *
 * Layout: logical NC(D)HW, filters KC(kd)(kh)(kw), row-major; 2D layers pass D = 1.
 * Storage type REAL is float (liboracle_f32) or double (liboracle_f64, for the
 * finite-difference checks); every sum is accumulated in double either way, so the
 * oracle is the more accurate side of any comparison.  No blocking, no fusion, no
 * reordering beyond "one accumulator per output element, terms added in
 * lexicographic index order".  OpenMP is used over independent outputs only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL float
#endif

typedef int64_t i64;

static i64 out_len(i64 in, i64 k, i64 s, i64 p) { return (in + 2 * p - k) / s + 1; }

/* y[n,k,od,oh,ow] = sum_{c,a,b,e} x[n,c,od*sd-pd+a,oh*sh-ph+b,ow*sw-pw+e] * w[k,c,a,b,e] */
void orc_conv_fwd(const REAL *x, const REAL *w, REAL *y,
                  i64 N, i64 C, i64 D, i64 H, i64 W, i64 K,
                  i64 kd, i64 kh, i64 kw, i64 sd, i64 sh, i64 sw,
                  i64 pd, i64 ph, i64 pw)
{
    const i64 Do = out_len(D, kd, sd, pd), Ho = out_len(H, kh, sh, ph), Wo = out_len(W, kw, sw, pw);
    const i64 osz = Do * Ho * Wo;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (i64 n = 0; n < N; ++n)
        for (i64 k = 0; k < K; ++k) {
            double *acc = (double *)calloc((size_t)osz, sizeof(double));
            for (i64 c = 0; c < C; ++c)
                for (i64 a = 0; a < kd; ++a)
                    for (i64 b = 0; b < kh; ++b)
                        for (i64 e = 0; e < kw; ++e) {
                            const double wv = (double)w[(((k * C + c) * kd + a) * kh + b) * kw + e];
                            for (i64 od = 0; od < Do; ++od) {
                                const i64 id = od * sd - pd + a;
                                if (id < 0 || id >= D) continue;
                                for (i64 oh = 0; oh < Ho; ++oh) {
                                    const i64 ih = oh * sh - ph + b;
                                    if (ih < 0 || ih >= H) continue;
                                    const REAL *xr = x + (((n * C + c) * D + id) * H + ih) * W;
                                    double *ar = acc + (od * Ho + oh) * Wo;
                                    for (i64 ow = 0; ow < Wo; ++ow) {
                                        const i64 iw = ow * sw - pw + e;
                                        if (iw < 0 || iw >= W) continue;
                                        ar[ow] += wv * (double)xr[iw];
                                    }
                                }
                            }
                        }
            REAL *yo = y + (n * K + k) * osz;
            for (i64 i = 0; i < osz; ++i) yo[i] = (REAL)acc[i];
            free(acc);
        }
}

/* dx[n,c,id,ih,iw] = sum over (k,a,b,e,od,oh,ow) with od*sd-pd+a == id etc. of dy * w */
void orc_conv_dgrad(const REAL *dy, const REAL *w, REAL *dx,
                    i64 N, i64 C, i64 D, i64 H, i64 W, i64 K,
                    i64 kd, i64 kh, i64 kw, i64 sd, i64 sh, i64 sw,
                    i64 pd, i64 ph, i64 pw)
{
    const i64 Do = out_len(D, kd, sd, pd), Ho = out_len(H, kh, sh, ph), Wo = out_len(W, kw, sw, pw);
    const i64 isz = D * H * W, osz = Do * Ho * Wo;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (i64 n = 0; n < N; ++n)
        for (i64 c = 0; c < C; ++c) {
            double *acc = (double *)calloc((size_t)isz, sizeof(double));
            for (i64 k = 0; k < K; ++k)
                for (i64 a = 0; a < kd; ++a)
                    for (i64 b = 0; b < kh; ++b)
                        for (i64 e = 0; e < kw; ++e) {
                            const double wv = (double)w[(((k * C + c) * kd + a) * kh + b) * kw + e];
                            const REAL *dyo = dy + (n * K + k) * osz;
                            for (i64 od = 0; od < Do; ++od) {
                                const i64 id = od * sd - pd + a;
                                if (id < 0 || id >= D) continue;
                                for (i64 oh = 0; oh < Ho; ++oh) {
                                    const i64 ih = oh * sh - ph + b;
                                    if (ih < 0 || ih >= H) continue;
                                    double *ar = acc + (id * H + ih) * W;
                                    const REAL *dr = dyo + (od * Ho + oh) * Wo;
                                    for (i64 ow = 0; ow < Wo; ++ow) {
                                        const i64 iw = ow * sw - pw + e;
                                        if (iw < 0 || iw >= W) continue;
                                        ar[iw] += wv * (double)dr[ow];
                                    }
                                }
                            }
                        }
            REAL *dxo = dx + (n * C + c) * isz;
            for (i64 i = 0; i < isz; ++i) dxo[i] = (REAL)acc[i];
            free(acc);
        }
}

/* dw[k,c,a,b,e] = sum_{n,od,oh,ow} dy[n,k,od,oh,ow] * x[n,c,od*sd-pd+a,oh*sh-ph+b,ow*sw-pw+e] */
void orc_conv_wgrad(const REAL *dy, const REAL *x, REAL *dw,
                    i64 N, i64 C, i64 D, i64 H, i64 W, i64 K,
                    i64 kd, i64 kh, i64 kw, i64 sd, i64 sh, i64 sw,
                    i64 pd, i64 ph, i64 pw)
{
    const i64 Do = out_len(D, kd, sd, pd), Ho = out_len(H, kh, sh, ph), Wo = out_len(W, kw, sw, pw);
    const i64 osz = Do * Ho * Wo;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (i64 k = 0; k < K; ++k)
        for (i64 c = 0; c < C; ++c)
            for (i64 a = 0; a < kd; ++a)
                for (i64 b = 0; b < kh; ++b)
                    for (i64 e = 0; e < kw; ++e) {
                        double acc = 0.0;
                        for (i64 n = 0; n < N; ++n) {
                            const REAL *dyo = dy + (n * K + k) * osz;
                            for (i64 od = 0; od < Do; ++od) {
                                const i64 id = od * sd - pd + a;
                                if (id < 0 || id >= D) continue;
                                for (i64 oh = 0; oh < Ho; ++oh) {
                                    const i64 ih = oh * sh - ph + b;
                                    if (ih < 0 || ih >= H) continue;
                                    const REAL *xr = x + (((n * C + c) * D + id) * H + ih) * W;
                                    const REAL *dr = dyo + (od * Ho + oh) * Wo;
                                    for (i64 ow = 0; ow < Wo; ++ow) {
                                        const i64 iw = ow * sw - pw + e;
                                        if (iw < 0 || iw >= W) continue;
                                        acc += (double)dr[ow] * (double)xr[iw];
                                    }
                                }
                            }
                        }
                        dw[(((k * C + c) * kd + a) * kh + b) * kw + e] = (REAL)acc;
                    }
}

/* Training-mode batch normalisation over x[N,C,S] (S = product of spatial sizes).
 * mean_c = (1/m) sum x, var_c = (1/m) sum (x-mean)^2 (biased), m = N*S,
 * istd_c = 1/sqrt(var_c+eps), y = gamma*(x-mean)*istd + beta. */
void orc_bn_fwd(const REAL *x, const REAL *gamma, const REAL *beta, REAL *y,
                REAL *mean, REAL *istd, i64 N, i64 C, i64 S, double eps)
{
    const double m = (double)(N * S);
#pragma omp parallel for schedule(dynamic)
    for (i64 c = 0; c < C; ++c) {
        double s = 0.0;
        for (i64 n = 0; n < N; ++n) {
            const REAL *xr = x + (n * C + c) * S;
            for (i64 i = 0; i < S; ++i) s += (double)xr[i];
        }
        const double mu = s / m;
        double v = 0.0;
        for (i64 n = 0; n < N; ++n) {
            const REAL *xr = x + (n * C + c) * S;
            for (i64 i = 0; i < S; ++i) { const double d = (double)xr[i] - mu; v += d * d; }
        }
        const double is = 1.0 / sqrt(v / m + eps);
        mean[c] = (REAL)mu;
        istd[c] = (REAL)is;
        const double g = (double)gamma[c], b = (double)beta[c];
        for (i64 n = 0; n < N; ++n) {
            const REAL *xr = x + (n * C + c) * S;
            REAL *yr = y + (n * C + c) * S;
            for (i64 i = 0; i < S; ++i) yr[i] = (REAL)(g * ((double)xr[i] - mu) * is + b);
        }
    }
}

/* Backward through the batch statistics, with xh = (x-mean)*istd:
 * dbeta = sum dy, dgamma = sum dy*xh, dx = gamma*istd*(dy - dbeta/m - xh*dgamma/m). */
void orc_bn_bwd(const REAL *x, const REAL *dy, const REAL *gamma,
                const REAL *mean, const REAL *istd,
                REAL *dx, REAL *dgamma, REAL *dbeta, i64 N, i64 C, i64 S)
{
    const double m = (double)(N * S);
#pragma omp parallel for schedule(dynamic)
    for (i64 c = 0; c < C; ++c) {
        const double mu = (double)mean[c], is = (double)istd[c], g = (double)gamma[c];
        double db = 0.0, dg = 0.0;
        for (i64 n = 0; n < N; ++n) {
            const REAL *xr = x + (n * C + c) * S;
            const REAL *dr = dy + (n * C + c) * S;
            for (i64 i = 0; i < S; ++i) {
                db += (double)dr[i];
                dg += (double)dr[i] * (((double)xr[i] - mu) * is);
            }
        }
        dbeta[c] = (REAL)db;
        dgamma[c] = (REAL)dg;
        for (i64 n = 0; n < N; ++n) {
            const REAL *xr = x + (n * C + c) * S;
            const REAL *dr = dy + (n * C + c) * S;
            REAL *dxr = dx + (n * C + c) * S;
            for (i64 i = 0; i < S; ++i) {
                const double xh = ((double)xr[i] - mu) * is;
                dxr[i] = (REAL)(g * is * ((double)dr[i] - db / m - xh * dg / m));
            }
        }
    }
}

void orc_relu_fwd(const REAL *x, REAL *y, i64 n)
{
#pragma omp parallel for
    for (i64 i = 0; i < n; ++i) y[i] = x[i] > (REAL)0 ? x[i] : (REAL)0;
}

/* dx = dy where the forward OUTPUT is positive, else 0 */
void orc_relu_bwd(const REAL *y, const REAL *dy, REAL *dx, i64 n)
{
#pragma omp parallel for
    for (i64 i = 0; i < n; ++i) dx[i] = y[i] > (REAL)0 ? dy[i] : (REAL)0;
}

/* index (within one [D,H,W] slab) of the first maximal in-bounds element of a window */
static i64 window_argmax(const REAL *xs, i64 D, i64 H, i64 W, i64 od, i64 oh, i64 ow,
                         i64 kd, i64 kh, i64 kw, i64 sd, i64 sh, i64 sw,
                         i64 pd, i64 ph, i64 pw)
{
    i64 best = -1;
    REAL bv = 0;
    for (i64 a = 0; a < kd; ++a) {
        const i64 id = od * sd - pd + a;
        if (id < 0 || id >= D) continue;
        for (i64 b = 0; b < kh; ++b) {
            const i64 ih = oh * sh - ph + b;
            if (ih < 0 || ih >= H) continue;
            for (i64 e = 0; e < kw; ++e) {
                const i64 iw = ow * sw - pw + e;
                if (iw < 0 || iw >= W) continue;
                const i64 idx = (id * H + ih) * W + iw;
                if (best < 0 || xs[idx] > bv) { best = idx; bv = xs[idx]; }
            }
        }
    }
    return best;
}

void orc_maxpool_fwd(const REAL *x, REAL *y, i64 NC, i64 D, i64 H, i64 W,
                     i64 kd, i64 kh, i64 kw, i64 sd, i64 sh, i64 sw,
                     i64 pd, i64 ph, i64 pw)
{
    const i64 Do = out_len(D, kd, sd, pd), Ho = out_len(H, kh, sh, ph), Wo = out_len(W, kw, sw, pw);
#pragma omp parallel for schedule(dynamic)
    for (i64 nc = 0; nc < NC; ++nc) {
        const REAL *xs = x + nc * D * H * W;
        REAL *ys = y + nc * Do * Ho * Wo;
        for (i64 od = 0; od < Do; ++od)
            for (i64 oh = 0; oh < Ho; ++oh)
                for (i64 ow = 0; ow < Wo; ++ow) {
                    const i64 am = window_argmax(xs, D, H, W, od, oh, ow, kd, kh, kw, sd, sh, sw, pd, ph, pw);
                    ys[(od * Ho + oh) * Wo + ow] = am >= 0 ? xs[am] : (REAL)(-INFINITY);
                }
    }
}

/* dx = 0, then every output position, in scan order, adds its dy to its argmax */
void orc_maxpool_bwd(const REAL *x, const REAL *dy, REAL *dx, i64 NC, i64 D, i64 H, i64 W,
                     i64 kd, i64 kh, i64 kw, i64 sd, i64 sh, i64 sw,
                     i64 pd, i64 ph, i64 pw)
{
    const i64 Do = out_len(D, kd, sd, pd), Ho = out_len(H, kh, sh, ph), Wo = out_len(W, kw, sw, pw);
#pragma omp parallel for schedule(dynamic)
    for (i64 nc = 0; nc < NC; ++nc) {
        const REAL *xs = x + nc * D * H * W;
        const REAL *ds = dy + nc * Do * Ho * Wo;
        REAL *dxs = dx + nc * D * H * W;
        for (i64 i = 0; i < D * H * W; ++i) dxs[i] = (REAL)0;
        for (i64 od = 0; od < Do; ++od)
            for (i64 oh = 0; oh < Ho; ++oh)
                for (i64 ow = 0; ow < Wo; ++ow) {
                    const i64 am = window_argmax(xs, D, H, W, od, oh, ow, kd, kh, kw, sd, sh, sw, pd, ph, pw);
                    if (am >= 0) dxs[am] += ds[(od * Ho + oh) * Wo + ow];
                }
    }
}

/* y[nc] = mean over the S spatial positions; dx = dy/S spread evenly */
void orc_gavgpool_fwd(const REAL *x, REAL *y, i64 NC, i64 S)
{
#pragma omp parallel for
    for (i64 nc = 0; nc < NC; ++nc) {
        double s = 0.0;
        for (i64 i = 0; i < S; ++i) s += (double)x[nc * S + i];
        y[nc] = (REAL)(s / (double)S);
    }
}

void orc_gavgpool_bwd(const REAL *dy, REAL *dx, i64 NC, i64 S)
{
#pragma omp parallel for
    for (i64 nc = 0; nc < NC; ++nc)
        for (i64 i = 0; i < S; ++i) dx[nc * S + i] = (REAL)((double)dy[nc] / (double)S);
}

/* y[n,o] = sum_i x[n,i] w[o,i] + b[o] */
void orc_fc_fwd(const REAL *x, const REAL *w, const REAL *b, REAL *y, i64 N, i64 I, i64 O)
{
#pragma omp parallel for collapse(2)
    for (i64 n = 0; n < N; ++n)
        for (i64 o = 0; o < O; ++o) {
            double s = 0.0;
            for (i64 i = 0; i < I; ++i) s += (double)x[n * I + i] * (double)w[o * I + i];
            y[n * O + o] = (REAL)(s + (double)b[o]);
        }
}

/* dx[n,i] = sum_o dy[n,o] w[o,i]; dw[o,i] = sum_n dy[n,o] x[n,i]; db[o] = sum_n dy[n,o] */
void orc_fc_bwd(const REAL *x, const REAL *w, const REAL *dy,
                REAL *dx, REAL *dw, REAL *db, i64 N, i64 I, i64 O)
{
#pragma omp parallel for collapse(2)
    for (i64 n = 0; n < N; ++n)
        for (i64 i = 0; i < I; ++i) {
            double s = 0.0;
            for (i64 o = 0; o < O; ++o) s += (double)dy[n * O + o] * (double)w[o * I + i];
            dx[n * I + i] = (REAL)s;
        }
#pragma omp parallel for collapse(2)
    for (i64 o = 0; o < O; ++o)
        for (i64 i = 0; i < I; ++i) {
            double s = 0.0;
            for (i64 n = 0; n < N; ++n) s += (double)dy[n * O + o] * (double)x[n * I + i];
            dw[o * I + i] = (REAL)s;
        }
    for (i64 o = 0; o < O; ++o) {
        double s = 0.0;
        for (i64 n = 0; n < N; ++n) s += (double)dy[n * O + o];
        db[o] = (REAL)s;
    }
}

/* L = -(1/N) sum_n log softmax(z_n)[t_n];  dz = (softmax(z) - onehot(t)) / N.  Returns L.
 * With mx the row maximum, -log softmax(z)[t] = (mx - z_t) + log(sum_j exp(z_j - mx)).  One term of that sum is
 * exp(0) = 1 (the first maximal element's), so the sum is 1 + rest and its logarithm log1p(rest): written this way
 * the definition keeps full precision for a sample whose labelled class leads by a wide margin (rest ~ 1e-15 would
 * otherwise be rounded into the 1).  Likewise softmax(z)[t] - 1 = -(sum of the other classes' terms) / (whole sum). */
double orc_softmax_ce(const REAL *z, const int32_t *t, REAL *dz, i64 N, i64 K)
{
    double loss = 0.0;
    for (i64 n = 0; n < N; ++n) {
        const REAL *zr = z + n * K;
        i64 am = 0;
        for (i64 j = 1; j < K; ++j) if ((double)zr[j] > (double)zr[am]) am = j;
        const double mx = (double)zr[am];
        double rest = 0.0;                       /* every term but the first maximal element's */
        for (i64 j = 0; j < K; ++j) if (j != am) rest += exp((double)zr[j] - mx);
        loss += (mx - (double)zr[t[n]]) + log1p(rest);
        if (dz) {
            double others = 0.0;                 /* every term but the labelled class's */
            for (i64 j = 0; j < K; ++j) if (j != t[n]) others += exp((double)zr[j] - mx);
            const double all = others + exp((double)zr[t[n]] - mx);
            for (i64 j = 0; j < K; ++j) {
                const double g = j == t[n] ? -others / all : exp((double)zr[j] - mx) / all;
                dz[n * K + j] = (REAL)(g / (double)N);
            }
        }
    }
    return loss / (double)N;
}

int orc_real_bytes(void) { return (int)sizeof(REAL); }

/* CPU oracle for the encode side of Rapid-INR (see fit_oracle.h).  TEST INFRASTRUCTURE ONLY. */
#include "fit_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

int64_t fit_n_params(const int32_t *widths, int32_t L) {
    int64_t n = 0;
    for (int32_t l = 0; l < L; ++l) n += (int64_t)widths[l + 1] * widths[l] + widths[l + 1];
    return n;
}

static double kept(const double *params, const uint8_t *keep, int64_t i) {
    return (keep == NULL || keep[i]) ? params[i] : 0.0;
}

/* pixel-centre coordinate j of n on [lo, hi] */
static double centre(int32_t j, int32_t n, double lo, double hi) {
    return lo + (hi - lo) * (2.0 * j + 1.0) / (2.0 * n);
}

/* Forward pass of one pixel.  h[l] (l = 0..L-1) are the layer inputs, z[l] the pre-activations. */
static void forward_pixel(const int32_t *widths, int32_t L, double w0, const double *params, const uint8_t *keep,
                          double x, double y, double **h, double **z) {
    h[0][0] = x;
    h[0][1] = y;
    int64_t off = 0;
    for (int32_t l = 0; l < L; ++l) {
        const int32_t nin = widths[l], nout = widths[l + 1];
        const int64_t boff = off + (int64_t)nout * nin;
        for (int32_t o = 0; o < nout; ++o) {
            double s = kept(params, keep, boff + o);
            for (int32_t i = 0; i < nin; ++i) s += kept(params, keep, off + (int64_t)o * nin + i) * h[l][i];
            z[l][o] = s;
            if (l < L - 1) h[l + 1][o] = sin(w0 * s);
        }
        off = boff + nout;
    }
}

static double **alloc_rows(const int32_t *widths, int32_t L, int shift) {
    double **r = (double **)malloc(sizeof(double *) * (size_t)L);
    for (int32_t l = 0; l < L; ++l) r[l] = (double *)malloc(sizeof(double) * (size_t)widths[l + shift]);
    return r;
}
static void free_rows(double **r, int32_t L) {
    for (int32_t l = 0; l < L; ++l) free(r[l]);
    free(r);
}

void fit_forward(const int32_t *widths, int32_t L, double w0, double lo, double hi, int32_t H, int32_t W,
                 const double *params, const uint8_t *keep, double *out) {
    double **h = alloc_rows(widths, L, 0), **z = alloc_rows(widths, L, 1);
    for (int32_t r = 0; r < H; ++r)
        for (int32_t c = 0; c < W; ++c) {
            forward_pixel(widths, L, w0, params, keep, centre(c, W, lo, hi), centre(r, H, lo, hi), h, z);
            for (int32_t k = 0; k < widths[L]; ++k) out[((int64_t)k * H + r) * W + c] = z[L - 1][k];
        }
    free_rows(h, L);
    free_rows(z, L);
}

void fit_loss_grad(const int32_t *widths, int32_t L, double w0, double lo, double hi, int32_t H, int32_t W,
                   const double *params, const uint8_t *keep, const double *target, double loss_scale,
                   double *loss, double *grad) {
    const int64_t np = fit_n_params(widths, L);
    double **h = alloc_rows(widths, L, 0), **z = alloc_rows(widths, L, 1), **d = alloc_rows(widths, L, 1);
    if (grad) memset(grad, 0, sizeof(double) * (size_t)np);
    double total = 0.0;
    for (int32_t r = 0; r < H; ++r)
        for (int32_t c = 0; c < W; ++c) {
            forward_pixel(widths, L, w0, params, keep, centre(c, W, lo, hi), centre(r, H, lo, hi), h, z);
            for (int32_t k = 0; k < widths[L]; ++k) {
                const double e = z[L - 1][k] - target[((int64_t)k * H + r) * W + c];
                total += e * e;
                d[L - 1][k] = 2.0 * loss_scale * e;          /* d loss / d z_{L-1} */
            }
            if (!grad) continue;
            /* offsets of the layers, walked backwards */
            int64_t off = np;
            for (int32_t l = L - 1; l >= 0; --l) {
                const int32_t nin = widths[l], nout = widths[l + 1];
                off -= (int64_t)nout * nin + nout;
                const int64_t boff = off + (int64_t)nout * nin;
                for (int32_t o = 0; o < nout; ++o) {
                    if (keep == NULL || keep[boff + o]) grad[boff + o] += d[l][o];
                    for (int32_t i = 0; i < nin; ++i) {
                        const int64_t at = off + (int64_t)o * nin + i;
                        if (keep == NULL || keep[at]) grad[at] += d[l][o] * h[l][i];
                    }
                }
                if (l == 0) break;
                /* d loss / d z_{l-1} = (W_l^T d_l) * w0 cos(w0 z_{l-1}) */
                for (int32_t i = 0; i < nin; ++i) {
                    double s = 0.0;
                    for (int32_t o = 0; o < nout; ++o) s += kept(params, keep, off + (int64_t)o * nin + i) * d[l][o];
                    d[l - 1][i] = s * w0 * cos(w0 * z[l - 1][i]);
                }
            }
        }
    *loss = loss_scale * total;
    free_rows(h, L);
    free_rows(z, L);
    free_rows(d, L);
}

void fit_adam_step(double *params, double *m, double *v, const double *grad, const uint8_t *keep, int64_t n,
                   int32_t t, double lr, double b1, double b2, double eps) {
    const double c1 = 1.0 - pow(b1, (double)t), c2 = 1.0 - pow(b2, (double)t);
    for (int64_t i = 0; i < n; ++i) {
        if (keep && !keep[i]) {
            params[i] = 0.0;
            continue;
        }
        m[i] = b1 * m[i] + (1.0 - b1) * grad[i];
        v[i] = b2 * v[i] + (1.0 - b2) * grad[i] * grad[i];
        params[i] -= lr * (m[i] / c1) / (sqrt(v[i] / c2) + eps);
    }
}

double fit_cosine_lr(double lr0, int32_t t, int32_t T) {
    return 0.5 * lr0 * (1.0 + cos(acos(-1.0) * (double)t / (double)T));
}

double fit_psnr(const double *a, const double *b, int64_t n) {
    double s = 0.0;
    for (int64_t i = 0; i < n; ++i) s += (a[i] - b[i]) * (a[i] - b[i]);
    return 10.0 * log10((double)n / s);
}

double fit_prune_ratio(int32_t schedule, double psnr) {
    if (schedule == 0) {                       /* Eq. 2 */
        if (psnr < 30.0) return 0.0;
        if (psnr <= 35.0) return 0.05 * psnr - 1.5;
        return 0.25;
    }
    /* Eq. 3 and Eq. 4 print the same pieces */
    if (psnr < 35.0) return 0.2;
    if (psnr <= 40.0) return 0.04 * psnr - 1.2;
    return 0.4;
}

void fit_l1_mask(const double *w, int64_t n, double ratio, const uint8_t *keep_in, uint8_t *keep_out) {
    int64_t n_prune = (int64_t)rint(ratio * (double)n);
    if (n_prune < 0) n_prune = 0;
    if (n_prune > n) n_prune = n;
    for (int64_t i = 0; i < n; ++i) keep_out[i] = 1;
    /* selection by repeated minimum: O(n * n_prune), plainly the definition */
    for (int64_t k = 0; k < n_prune; ++k) {
        int64_t best = -1;
        double bm = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            if (!keep_out[i]) continue;
            const double mag = (keep_in && !keep_in[i]) ? 0.0 : fabs(w[i]);
            if (best < 0 || mag < bm) {
                best = i;
                bm = mag;
            }
        }
        keep_out[best] = 0;
    }
    if (keep_in)
        for (int64_t i = 0; i < n; ++i)
            if (!keep_in[i]) keep_out[i] = 0;      /* a pruned weight never comes back */
}

void fit_quantize(const double *w, const uint8_t *keep, int64_t n, int32_t bits, double *scale, int32_t *zp,
                  uint16_t *codes) {
    const double qmax = (double)((1 << bits) - 1);
    double mn = 0.0, mx = 0.0;                    /* the range always contains 0 */
    for (int64_t i = 0; i < n; ++i) {
        if (keep && !keep[i]) continue;
        if (w[i] < mn) mn = w[i];
        if (w[i] > mx) mx = w[i];
    }
    double s = (mx - mn) / qmax;
    s = (double)(float)s;                         /* the store keeps the scale as fp32 */
    if (!(s > 0.0)) s = 1.0;
    double z = rint(-mn / s);
    if (z < 0.0) z = 0.0;
    if (z > qmax) z = qmax;
    *scale = s;
    *zp = (int32_t)z;
    for (int64_t i = 0; i < n; ++i) {
        double q = z;
        if (!keep || keep[i]) {
            q = rint(w[i] / s) + z;
            if (q < 0.0) q = 0.0;
            if (q > qmax) q = qmax;
        }
        codes[i] = (uint16_t)q;
    }
}

/* See inr_oracle.h.  Plain scalar loops, fp64, no blocking or fusion. */
#include "inr_oracle.h"
#include <math.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Effective weight (Sec. IV-A mask, Sec. IV-B codes): zero where pruned, the
 * stored float for an fp32 layer, else scale * (code - zp).  The affine product
 * is formed in double (exact: 24-bit by <=17-bit significands) and then rounded
 * once to fp32, i.e. the correctly rounded single-precision product. */
void orc_dequant(const orc_layer *l, double *w_out)
{
    const int64_t cnt = (int64_t)l->n_in * l->n_out;
    for (int64_t k = 0; k < cnt; ++k) {
        double w;
        if (l->keep && !l->keep[k]) {
            w = 0.0;
        } else if (l->bits == 0) {
            w = (double)l->w_f32[k];
        } else {
            int32_t d = (int32_t)l->codes[k] - l->zp;
            w = (double)l->scale * (double)d;
            w = (double)(float)w;
        }
        w_out[k] = w;
    }
}

/* One image: every pixel's centre coordinate through the MLP (Sec. III-A/B). */
static void decode_one(const orc_model *m, int32_t H, int32_t W, double w0, double lo,
                       double hi, int clamp, const double *aff, const double *norm, double *out, uint8_t *out8)
{
    const int L = m->n_layers;
    int maxw = 2;
    int64_t total = 0;
    for (int l = 0; l < L; ++l) {
        if (m->layers[l].n_out > maxw) maxw = m->layers[l].n_out;
        if (m->layers[l].n_in > maxw) maxw = m->layers[l].n_in;
        total += (int64_t)m->layers[l].n_in * m->layers[l].n_out;
    }
    double *wts = (double *)malloc(sizeof(double) * (size_t)total);
    double *h_prev = (double *)malloc(sizeof(double) * (size_t)maxw);
    double *h_next = (double *)malloc(sizeof(double) * (size_t)maxw);
    {
        int64_t off = 0;
        for (int l = 0; l < L; ++l) {
            orc_dequant(&m->layers[l], wts + off);
            off += (int64_t)m->layers[l].n_in * m->layers[l].n_out;
        }
    }
    const int64_t plane = (int64_t)H * W;
    for (int32_t i = 0; i < H; ++i) {
        for (int32_t j = 0; j < W; ++j) {
            /* pixel centres of a [lo, hi] x [lo, hi] grid; component 0 is horizontal */
            const double x = lo + (hi - lo) * (2.0 * j + 1.0) / (2.0 * W);
            const double y = lo + (hi - lo) * (2.0 * i + 1.0) / (2.0 * H);
            if (aff) {   /* augmentation: affine map of the sampling grid */
                h_prev[0] = aff[0] * x + aff[1] * y + aff[2];
                h_prev[1] = aff[3] * x + aff[4] * y + aff[5];
            } else {
                h_prev[0] = x;
                h_prev[1] = y;
            }
            int64_t off = 0;
            for (int l = 0; l < L; ++l) {
                const orc_layer *ly = &m->layers[l];
                for (int o = 0; o < ly->n_out; ++o) {
                    double acc = 0.0;
                    for (int q = 0; q < ly->n_in; ++q)
                        acc += wts[off + (int64_t)o * ly->n_in + q] * h_prev[q];
                    acc += (double)ly->bias[o];
                    h_next[o] = (l < L - 1) ? sin(w0 * acc) : acc;
                }
                off += (int64_t)ly->n_in * ly->n_out;
                double *t = h_prev; h_prev = h_next; h_next = t;
            }
            for (int c = 0; c < 3; ++c) {
                double v = h_prev[c];
                if (clamp) v = fmin(fmax(v, 0.0), 1.0);
                if (out8) out8[c * plane + (int64_t)i * W + j] = (uint8_t)nearbyint(255.0 * v);
                if (norm) v = v * norm[c] + norm[3 + c];
                out[c * plane + (int64_t)i * W + j] = v;
            }
        }
    }
    free(wts); free(h_prev); free(h_next);
}

static int decode_all(const orc_model *models, int64_t n_models, const int64_t *ids, int64_t n,
                      int32_t H, int32_t W, double w0, double lo, double hi, int clamp,
                      const double *affine, const double *norm, double *out_f64, uint8_t *out_u8, int n_threads)
{
    if (!models || !ids || !out_f64 || n < 0 || H <= 0 || W <= 0) return -1;
    if (!clamp && out_u8) return -1;
    for (int64_t s = 0; s < n; ++s) {
        if (ids[s] < 0 || ids[s] >= n_models) return -1;
        const orc_model *m = &models[ids[s]];
        if (m->n_layers < 1 || m->layers[0].n_in != 2 || m->layers[m->n_layers - 1].n_out != 3) return -1;
        for (int l = 1; l < m->n_layers; ++l)
            if (m->layers[l].n_in != m->layers[l - 1].n_out) return -1;
    }
    const int64_t img = 3 * (int64_t)H * W;
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
    for (int64_t s = 0; s < n; ++s)
        decode_one(&models[ids[s]], H, W, w0, lo, hi, clamp, affine ? affine + 6 * s : (const double *)0, norm,
                   out_f64 + s * img, out_u8 ? out_u8 + s * img : (uint8_t *)0);
    return 0;
}

int orc_decode(const orc_model *models, int64_t n_models, const int64_t *ids, int64_t n,
               int32_t H, int32_t W, double w0, double lo, double hi, int clamp,
               double *out_f64, uint8_t *out_u8, int n_threads)
{
    return decode_all(models, n_models, ids, n, H, W, w0, lo, hi, clamp, (const double *)0, (const double *)0,
                      out_f64, out_u8, n_threads);
}

int orc_decode_aug(const orc_model *models, int64_t n_models, const int64_t *ids, int64_t n,
                   int32_t H, int32_t W, double w0, double lo, double hi, int clamp,
                   const double *affine, const double *norm, double *out_f64, int n_threads)
{
    return decode_all(models, n_models, ids, n, H, W, w0, lo, hi, clamp, affine, norm, out_f64, (uint8_t *)0, n_threads);
}

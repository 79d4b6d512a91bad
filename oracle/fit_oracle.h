/* CPU oracle for the encode side of Rapid-INR.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain fp64 statements of: fitting one sine-activated MLP to one image by minimising
 * the squared error over its pixels (Sec. II-A, Eq. 1) with Adam and cosine learning-rate
 * decay (Sec. VI-A); the pruning-ratio schedules of dynamic pruning (Sec. IV-A, Eq. 2-4);
 * L1-magnitude unstructured masks (Sec. IV-A); and the per-layer affine quantiser of hidden
 * layers (Sec. IV-B).  Nothing here is shared with the GPU library.  Only tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it.
 *
 * Parameter vector of a model with L linear layers of widths d_0 = 2, d_1, ..., d_L = 3:
 * for l = 0..L-1 the matrix W_l as [d_{l+1}][d_l] row-major, then the bias b_l [d_{l+1}].
 * The network is h_0 = (x, y), z_l = W_l h_l + b_l, h_{l+1} = sin(w0 z_l) for l < L-1,
 * output f = z_{L-1} (no clamp while fitting).  Coordinates are pixel centres on [lo, hi]^2,
 * component 0 horizontal, the same grid the decode oracle uses.
 *
 * Pins (tests marked "not gpu"): the gradient against central finite differences of the
 * loss; the loss against the decode oracle's output; Adam's first step in closed form; the
 * cosine schedule's end points and mid point; Eq. 2-4 at the values their printed pieces fix
 * and their continuity at the break points; mask counts, order and nesting; quantiser error
 * <= scale/2, exact zero, and range end points.
 */
#ifndef FIT_ORACLE_H
#define FIT_ORACLE_H
#include <stdint.h>

/* Number of parameters of the model. */
int64_t fit_n_params(const int32_t *widths, int32_t L);

/* loss = loss_scale * sum over pixels and channels of (f - target)^2 (Eq. 1; loss_scale = 1 is
 * the printed sum, 1/(3 H W) the mean).  target is [3][H][W].  keep (NULL = all kept) has one
 * byte per parameter; a parameter with keep == 0 is treated as 0 whatever params holds, and its
 * gradient is 0.  grad may be NULL. */
void fit_loss_grad(const int32_t *widths, int32_t L, double w0, double lo, double hi, int32_t H, int32_t W,
                   const double *params, const uint8_t *keep, const double *target, double loss_scale,
                   double *loss, double *grad);

/* The model's output image [3][H][W] (unclamped). */
void fit_forward(const int32_t *widths, int32_t L, double w0, double lo, double hi, int32_t H, int32_t W,
                 const double *params, const uint8_t *keep, double *out);

/* One Adam update, t = 1 for the first:  m = b1 m + (1-b1) g,  v = b2 v + (1-b2) g^2,
 * p -= lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps); pruned parameters stay 0. */
void fit_adam_step(double *params, double *m, double *v, const double *grad, const uint8_t *keep, int64_t n,
                   int32_t t, double lr, double b1, double b2, double eps);

/* Cosine decay to zero over T steps: the rate used for step index t = 0..T-1. */
double fit_cosine_lr(double lr0, int32_t t, int32_t T);

/* Peak signal-to-noise ratio in dB for values on a 0..1 scale: 10 log10(1 / mse). */
double fit_psnr(const double *a, const double *b, int64_t n);

/* Dynamic pruning ratio (Sec. IV-A): schedule 0 = Eq. 2 (small images), 1 = Eq. 3, 2 = Eq. 4. */
double fit_prune_ratio(int32_t schedule, double psnr);

/* L1-magnitude mask over one weight matrix: the round(ratio * n) entries of smallest |w| get
 * keep = 0 (ties: lower index first); entries already pruned in keep_in (NULL = none) count as
 * magnitude 0 and therefore go first, so ratio is the fraction of ALL n entries that end up pruned. */
void fit_l1_mask(const double *w, int64_t n, double ratio, const uint8_t *keep_in, uint8_t *keep_out);

/* Per-layer unsigned affine quantiser to `bits` bits over the kept entries, range extended to
 * contain 0:  scale = (max - min) / (2^bits - 1), zp = rint(-min / scale),
 * code = clamp(rint(w / scale) + zp, 0, 2^bits - 1); all-zero input gives scale 1, zp 0.
 * Pruned entries get code zp. */
void fit_quantize(const double *w, const uint8_t *keep, int64_t n, int32_t bits, double *scale, int32_t *zp,
                  uint16_t *codes);

#endif

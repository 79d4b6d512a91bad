/* rinr_fit — the encode side of an INR-compressed image dataset (MI355X / gfx950).
 *
 * Turns images into the per-image sine MLPs that rinr.h decodes: fit one MLP per image by
 * minimising the squared error over its pixels (paper Sec. II-A, Eq. 1) with Adam and cosine
 * learning-rate decay (Sec. VI-A), prune by weight magnitude with a ratio chosen from the
 * reconstruction's PSNR (Sec. IV-A, Eq. 2-4), re-fit under the mask, and quantise the hidden
 * layers with a per-layer affine map (Sec. IV-B).  The results (fp32 weights, keep masks,
 * codes, scale, zero point) are what rinr_pack takes.
 *
 * Same conventions as rinr.h: plain C ABI, 0 or a negative RINR_E_* code, "host"/"device" says
 * which memory a pointer must point to, the caller owns every buffer it passes.  The library
 * owns the rinr_fit handle and the device state inside it.  Random numbers are never drawn here:
 * initial weights come from the caller.
 *
 * Parameter vector of one model with L linear layers of widths d_0 = 2, d_1, ..., d_L = 3:
 * for l = 0..L-1 the matrix W_l as [d_{l+1}][d_l] row-major, then the bias b_l [d_{l+1}].
 * The network is h_0 = (x, y), z_l = W_l h_l + b_l, h_{l+1} = sin(w0 z_l) for l < L-1, output
 * z_{L-1} (no clamp while fitting); (x, y) is the pixel-centre grid of rinr.h on
 * [coord_lo, coord_hi]^2, component 0 horizontal.
 */
#ifndef RINR_FIT_H
#define RINR_FIT_H

#include "rinr.h"

#ifdef __cplusplus
extern "C" {
#endif

enum { RINR_FIT_MAX_LAYERS = 12 };   /* most linear layers of a model that can be fitted */

/* ---- host-side helpers ---------------------------------------------------------------- */

/* Dynamic pruning ratio as a function of the reconstruction's PSNR in dB (Sec. IV-A).
 * schedule 0 = Eq. 2 (small images: 0 below 30 dB, 0.05 PSNR - 1.5 up to 35 dB, then 0.25);
 * schedule 1 = Eq. 3 and 2 = Eq. 4 (0.2 below 35 dB, 0.04 PSNR - 1.2 up to 40 dB, then 0.4).
 * Any other schedule returns a NaN. */
double rinr_prune_ratio(int32_t schedule, double psnr);

/* L1-magnitude unstructured mask over one weight matrix (Sec. IV-A): keep_out[k] = 0 for the
 * rint(ratio * n) entries of smallest |w| (ties: lower index first), 1 otherwise.  Entries
 * already pruned in keep_in (host, uint8[n], NULL = none) count as magnitude 0, go first and stay
 * pruned, so `ratio` is the fraction of all n entries pruned afterwards.  w: host float[n];
 * keep_out: host uint8[n].  RINR_E_NULL / RINR_E_ARG (n < 0, ratio outside [0, 1] or NaN). */
int rinr_l1_mask(const float *w, int64_t n, double ratio, const uint8_t *keep_in, uint8_t *keep_out);

/* Per-layer unsigned affine quantiser (Sec. IV-B) over the kept entries of one matrix, range
 * extended to contain 0:  scale = fp32((max - min) / (2^bits - 1)), zp = rint(-min / scale),
 * code = clamp(rint(w / scale) + zp, 0, 2^bits - 1), arithmetic in double; pruned entries get
 * code zp; an all-zero matrix gives scale 1, zp 0.  bits 2..8 or 16.  keep: host uint8[n] or NULL.
 * Outputs (host): *scale, *zp, codes uint16[n]; w = scale * (code - zp) is what rinr.h decodes.
 * RINR_E_NULL / RINR_E_ARG (n < 0, bad bits, a non-finite kept weight). */
int rinr_quantize_layer(const float *w, const uint8_t *keep, int64_t n, int32_t bits, float *scale, int32_t *zp,
                        uint16_t *codes);

/* ---- fitting on the GPU (Eq. 1) --------------------------------------------------------- */

typedef struct {
    int32_t n_layers;                           /* linear layers L, 2..RINR_FIT_MAX_LAYERS       */
    int32_t widths[RINR_FIT_MAX_LAYERS + 1];    /* d_0..d_L: d_0 == 2, d_L == 3, others 1..64    */
    float w0;                                   /* sine frequency (30 in the paper, Sec. VI-A)   */
    float coord_lo, coord_hi;                   /* sampling range of both coordinates            */
} rinr_fit_arch;

typedef struct {
    float lr;            /* learning rate of this call's first step before decay (Sec. VI-A: 5e-4, 2e-4) */
    int32_t t0, T;       /* cosine decay: step i of this call uses lr/2 (1 + cos(pi (t0 + i) / T));
                            T <= 0 = constant rate                                                   */
    float beta1, beta2, eps;   /* Adam; 0 = the usual 0.9, 0.999, 1e-8                                */
    float loss_scale;    /* loss = loss_scale * sum of squared errors (Eq. 1); 0 = 1 / (3 H W), the mean */
} rinr_fit_opts;

typedef struct rinr_fit rinr_fit;

enum { RINR_FIT_FLAG_FP32_MFMA = 1 };   /* rinr_fit_create_ex: take the fp32 matrix-instruction kernels whatever the shape */
enum { RINR_FIT_KERNEL_FP32 = 0,        /* rinr_fit_kernel_family: fp32 operands on the fp32 matrix instructions              */
       RINR_FIT_KERNEL_SPLIT16 = 1 };   /* every fp32 operand as an exact-sum pair of halfs on the fp16 matrix instructions,
                                           three terms per product, fp32 accumulate (~22 significant bits per product)       */

/* Device state for fitting n_images models of one architecture to H x W targets (Eq. 1): parameters, Adam moments, keep
 * flags, per-image losses (3 * 4 + 1 bytes per parameter).  All images share the architecture; each has its own parameters.
 * Two families of kernels compute the same step.  The split-precision ones (the default where they are built for the
 * shape) keep the weights of all layers in one CU's LDS as fp16 hi/lo planes and the pre-activations of 16 pixels per
 * wavefront in registers: widest hidden layer <= 32: 12 linear layers, <= 48: 10, <= 64: 6.  The fp32 ones keep fp32 weights
 * in LDS: <= 32: 12 layers, <= 48: 10, <= 64: 7.  A shape only the fp32 kernels cover (7 layers x 64) takes those;
 * RINR_E_UNSUPPORTED beyond both.  These limits are narrower than the decode side's (16 layers of width 64, deep models
 * streamed) for a reason of the fit kernels' design: one Adam step keeps the weights of all layers in LDS (10 layers x 40:
 * 148 KB, 7 layers x 64: 155 KB of the 160) and the weight-gradient tiles of all layers in the owning wavefronts' registers
 * from the first pixel to the update, so gradients never touch memory; a deeper model at these widths fits neither.  The
 * paper's own shapes (Sec. VI-A: 3 x 15, 10 x 32, 10 x 40) and the benchmark's widest model (7 layers x 64) fit; a model
 * beyond the limits can still be packed and decoded, only not fitted here.
 * flags: 0 or RINR_FIT_FLAG_FP32_MFMA.  RINR_E_ARG for a bad architecture, size or flag; RINR_E_HIP on a failed allocation.
 * rinr_fit_create == rinr_fit_create_ex with flags = 0. */
int rinr_fit_create(const rinr_fit_arch *arch, int64_t n_images, int32_t H, int32_t W, rinr_fit **fit);
int rinr_fit_create_ex(const rinr_fit_arch *arch, int64_t n_images, int32_t H, int32_t W, uint32_t flags, rinr_fit **fit);
/* Which kernels this handle's steps run: RINR_FIT_KERNEL_*; RINR_E_NULL on NULL.  (Sec. VI-A fixes the method, not the
 * arithmetic; both families meet the same parity bar against the fp64 reference.) */
int rinr_fit_kernel_family(const rinr_fit *fit);
int rinr_fit_destroy(rinr_fit *fit);
int64_t rinr_fit_n_params(const rinr_fit *fit);        /* per image; < 0 on NULL */

/* Upload initial parameters (host float[n_images][n_params]); resets the Adam moments and the
 * step count to 0 and applies the current keep flags.  Synchronous. */
int rinr_fit_set_params(rinr_fit *fit, const float *params);
/* Keep flags (host uint8[n_images][n_params], NULL = keep all): a parameter with flag 0 is set
 * to 0 now and stays 0 (Sec. IV-A: the mask is applied and the model re-fitted).  Synchronous. */
int rinr_fit_set_keep(rinr_fit *fit, const uint8_t *keep);
/* Restart Adam (moments and step count to 0) without touching the parameters: a new fitting round. */
int rinr_fit_reset_optimizer(rinr_fit *fit);
/* Download the parameters (host float[n_images][n_params]).  Synchronises with `stream`. */
int rinr_fit_get_params(const rinr_fit *fit, float *params, void *stream);

/* n_steps full-batch steps (every pixel of every image each step) on `stream`: one kernel per
 * step, one workgroup per image, nothing allocated, no synchronisation.  targets: device,
 * float[n_images][3][H][W], 4-byte aligned, values on the 0..1 scale of the decoded image. */
int rinr_fit_steps(rinr_fit *fit, const float *targets, int32_t n_steps, const rinr_fit_opts *opts, void *stream);

/* Loss and gradient at the current parameters, without an update:
 * grad host float[n_images][n_params] (NULL = loss only), loss host float[n_images].  For checking
 * the kernels against a reference: allocates a device gradient buffer inside the handle on first use and
 * synchronises with `stream`.  loss_scale as in rinr_fit_opts (0 = the mean). */
int rinr_fit_loss_grad(rinr_fit *fit, const float *targets, float loss_scale, float *loss, float *grad, void *stream);
/* Per-image loss seen by the most recent step (before its update).  Synchronises with `stream`. */
int rinr_fit_last_loss(const rinr_fit *fit, float *loss, void *stream);

/* ---- reconstruction quality on the GPU --------------------------------------------------- */

/* Peak signal-to-noise ratio per image, the quantity the pruning ratio is chosen from (Sec. IV-A):
 * psnr[s] = 10 log10(peak^2 * elems / sum_k (a[s][k] - b[s][k])^2) in dB, +inf where the two are equal.
 * a, b: device float[n_images][elems] (e.g. a decoded batch and the original images, elems = 3 H W),
 * 4-byte aligned; psnr: device float[n_images]; peak: the value range (1 for 0..1 images).  One kernel on
 * `stream`, one workgroup per image, no synchronisation, nothing allocated.
 * RINR_E_NULL / RINR_E_ARG (negative sizes, peak <= 0) / RINR_E_ALIGN / RINR_E_HIP. */
int rinr_psnr_batch(const float *a, const float *b, int64_t n_images, int64_t elems, float peak, float *psnr,
                    void *stream);

/* ---- the whole encode procedure of Sec. IV in one call ----------------------------------- */

typedef struct {
    int32_t schedule;      /* PSNR-driven pruning round: 0 = Eq. 2, 1 = Eq. 3, 2 = Eq. 4 (rinr_prune_ratio)      */
    float first_ratio;     /* fixed ratio of the first pruning round (Sec. IV-A: 0.2 for the large-image sets);
                              0 = no first round (Sec. IV-A: the small-image set goes straight to the second)    */
    int32_t fit_steps;     /* steps of the initial fit                                                           */
    int32_t refit_steps;   /* steps of the re-fit after each pruning round                                       */
    float lr, refit_lr;    /* learning rates of the fit and of the re-fits ("a smaller learning rate",
                              Sec. IV-A), each cosine-decayed to 0 over its stage                                */
    int32_t hidden_bits;   /* code width of the hidden layers: 8 (Sec. IV-B), 2..8 or 16; 0 = keep them fp32     */
} rinr_encode_opts;

/* Upper bound of the blob rinr_encode_images writes for this handle's images (masks present, every weight kept). */
int rinr_encode_blob_bound(const rinr_fit *fit, int32_t hidden_bits, size_t *bytes);

/* Fit (Eq. 1), prune by magnitude at first_ratio and re-fit, prune at the ratio each image's PSNR selects (Eq. 2-4;
 * the ratio is the fraction of all entries pruned afterwards) and re-fit, quantise the hidden layers per layer
 * (Sec. IV-B), and pack every image's model into one blob for rinr_store_open.  Nothing but a sequence of the calls
 * above and of rinr_pack: the same steps issued one by one give the same bytes.
 * fit: a handle whose parameters are set (rinr_fit_set_params); its keep flags are replaced, its parameters end as the
 * final fp32 fit.  targets: device, as for rinr_fit_steps.  psnr (host float[n_images], may be NULL): PSNR in dB of that
 * final fit before quantisation, from the mean squared error over the 0..1 range.  blob: host, `capacity` bytes
 * (rinr_encode_blob_bound is always enough); *blob_bytes = bytes written.  RINR_E_SIZE if the blob does not fit (then
 * *blob_bytes is the size needed and the fit has been done).  Synchronises with `stream` several times; allocates
 * host memory proportional to n_images * n_params. */
int rinr_encode_images(rinr_fit *fit, const float *targets, const rinr_encode_opts *opts, float *psnr, void *blob,
                       size_t capacity, size_t *blob_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif

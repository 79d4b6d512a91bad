/* CPU oracle for batched INR image decode.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 statement of what decoding a Rapid-INR image means: one
 * small sine-activated MLP per image (Sec. III-A) maps every pixel's normalised
 * (x, y) to RGB (Sec. III-B); pruned weights are zero (Sec. IV-A); hidden-layer
 * weights may be stored as integer codes with a per-layer affine map while
 * other layers stay fp32 (Sec. IV-B); the activation is sin with frequency
 * w0 = 30 (Sec. VI-A).
 *
 * Nothing here is shared with the GPU library: no headers, no packing code, no
 * tables.  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it.  It reads the *unpacked* model description (one code, one keep
 * flag per weight), so a bug in the GPU library's packed format cannot hide.
 *
 * Pins (tests marked "not gpu"): dequant against exact rational arithmetic;
 * pruned == code-at-zero-point; single-sine-layer closed form in multiprecision;
 * all-zero weights; zero first layer; axis/grid ramp; resolution nesting;
 * hand-unrolled 2x2; bias periodicity; uint8 rounding properties; at depth (a
 * rectangular five-layer chain) renumbering of hidden units, oddness of the
 * activation and the small-signal limit against the affine matrix chain; and
 * agreement with a second numpy implementation.  The paper prints no decoded
 * value for any model, so none of the pins is a value from the paper.
 */
#ifndef INR_ORACLE_H
#define INR_ORACLE_H
#include <stdint.h>

typedef struct {
    int32_t n_in, n_out;
    int32_t bits;           /* 0: w_f32 holds the weights; else codes does     */
    int32_t zp;             /* zero point of the affine code map               */
    float scale;            /* w = scale * (code - zp)                         */
    const float *w_f32;     /* [n_out][n_in], used when bits == 0              */
    const uint16_t *codes;  /* [n_out][n_in], used when bits != 0              */
    const uint8_t *keep;    /* NULL = dense, else [n_out][n_in], 0 = pruned    */
    const float *bias;      /* [n_out]                                         */
} orc_layer;

typedef struct {
    int32_t n_layers;       /* linear layers; all but the last are followed by sin */
    const orc_layer *layers;
} orc_model;

/* Effective weights of one layer as doubles holding fp32-representable values. */
void orc_dequant(const orc_layer *l, double *w_out);

/* Decode slots [0, n): slot s shows model ids[s].  out_f64 is [n][3][H][W];
 * out_u8 (optional, same shape) is the 8-bit image of the clamped value.
 * clamp == 0 leaves the linear output unclamped in out_f64 (out_u8 then must be NULL).
 * Returns 0, or -1 on a bad argument (an id outside [0, n_models) included). */
int orc_decode(const orc_model *models, int64_t n_models, const int64_t *ids, int64_t n,
               int32_t H, int32_t W, double w0, double lo, double hi, int clamp,
               double *out_f64, uint8_t *out_u8, int n_threads);

/* Decode with on-GPU-style augmentation (Sec. III-B: augmentation runs on the decoded
 * batch before the backbone).  Geometric augmentation is a per-slot affine map of the
 * sampling grid, which a resolution-free decode (Sec. III-B) gets for free:
 *   (x', y') = (A[0] x + A[1] y + A[2],  A[3] x + A[4] y + A[5])
 * with (x, y) the pixel-centre coordinate; affine is [n][6] or NULL (identity).
 * Photometric normalisation is per channel, after the clamp:
 *   out = value * norm[c] + norm[3 + c];  norm is [6] or NULL (none).
 * out_u8 is not available here. */
int orc_decode_aug(const orc_model *models, int64_t n_models, const int64_t *ids, int64_t n,
                   int32_t H, int32_t W, double w0, double lo, double hi, int clamp,
                   const double *affine, const double *norm, double *out_f64, int n_threads);

#endif

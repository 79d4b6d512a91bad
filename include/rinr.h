/* rinr — batched on-GPU decode of an INR-compressed image dataset (MI355X / gfx950).
 *
 * Every image is its own small sine-activated coordinate MLP (paper Sec. III-A):
 * input the pixel's normalised (x, y), output (R, G, B).  The whole dataset is
 * uploaded to GPU memory once in weight form (Sec. III-B) and a batch of image
 * ids is decoded on the fly, at any resolution, into an NCHW RGB tensor that
 * stays on the GPU (Sec. III-B).  Weights may be pruned with a mask (Sec. IV-A)
 * and stored as integer codes with a per-layer affine map; the paper quantises
 * the hidden layers to 8 bits and keeps the first and last layer fp32
 * (Sec. IV-B).  Activation: sin with frequency w0 = 30 (Sec. VI-A).
 *
 * Plain C ABI.  Every function returns 0 (RINR_OK) or a negative RINR_E_* code;
 * nothing throws across the boundary.  "host" / "device" on a pointer says which
 * memory it must point to.  The caller owns every buffer it passes; the library
 * owns only the rinr_store handle (and one small device status word inside it).
 */
#ifndef RINR_H
#define RINR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    RINR_OK = 0,
    RINR_E_NULL = -1,        /* a required pointer is NULL                           */
    RINR_E_ARG = -2,         /* a size or option is out of range                     */
    RINR_E_MODEL = -3,       /* a model description breaks a rule listed at rinr_pack */
    RINR_E_SIZE = -4,        /* buffer too small / size overflows                    */
    RINR_E_FORMAT = -5,      /* blob header, index or a record is corrupt            */
    RINR_E_UNSUPPORTED = -6, /* valid, but wider/deeper than the kernels are built for */
    RINR_E_ALIGN = -7,       /* a device pointer is not aligned as required          */
    RINR_E_HIP = -8          /* a HIP runtime call failed (see rinr_last_hip_error)  */
};

enum { RINR_MAX_WIDTH = 64,    /* widest hidden layer the decode kernels accept        */
       RINR_MAX_LAYERS = 16 }; /* most linear layers per model                         */

/* ---- host-side description of one model (input of rinr_pack) ---------------------
 * Layer l computes y = W x + b with W stored [out][in] row-major (Sec. III-A MLP).
 * All layers but the last are followed by sin(w0 * y); the last is linear. */
typedef struct {
    int32_t in, out;        /* 1..RINR_MAX_WIDTH; first layer in == 2, last out == 3   */
    int32_t bits;           /* 0 = raw fp32 weights; 2..8 or 16 = integer codes         */
    float scale;            /* w = scale * (code - zp) (Sec. IV-B); ignored if bits==0  */
    int32_t zp;             /* 0 .. 2^bits - 1; ignored if bits == 0                    */
    const void *weights;    /* host. bits==0: float[out*in]; bits<=8: uint8_t[out*in];
                               bits==16: uint16_t[out*in]. One entry per weight, pruned
                               ones included (their value is ignored).                   */
    const uint8_t *mask;    /* host. NULL = dense; else out*in bits, bit k of the flat
                               index k = o*in + i at byte k/8, bit k%8; 1 = kept,
                               0 = pruned, i.e. the weight is exactly 0 (Sec. IV-A)      */
    const float *bias;      /* host. float[out]; never pruned or quantised             */
} rinr_layer_desc;

typedef struct {
    int32_t n_layers;               /* linear layers, 2..RINR_MAX_LAYERS (>= 1 sine layer) */
    const rinr_layer_desc *layers;  /* host                                              */
} rinr_model_desc;

/* Store-wide decode constants.  NULL where accepted means {30, -1, 1}. */
typedef struct {
    float w0;                /* sine frequency (Sec. VI-A: 30)                          */
    float coord_lo, coord_hi;/* pixel-centre grid spans [lo, hi] on both axes:
                                x_j = lo + (hi-lo)(2j+1)/(2W), y_i likewise with H.
                                The paper's text normalises to 0..1 (Sec. III-A);
                                sine-network initialisations assume -1..1 (default).      */
} rinr_store_opts;

/* ---- packing: model descriptions -> one position-independent blob ---------------
 * The blob is the dataset in "weight format": what is saved to disk and what is
 * uploaded once to the GPU (Sec. III-B).  Little-endian; offsets, no pointers.
 * Per layer it holds the mask (1 bit per weight), the codes of the KEPT weights
 * only, in ascending flat index, as one LSB-first bit stream of `bits` per code
 * (32 for raw fp32), and the fp32 biases.
 *
 * rinr_pack_size: *bytes = exact size rinr_pack will write.
 * rinr_pack: writes the blob to host_blob (capacity `bytes`, must be >= that size).
 * Both validate and return RINR_E_MODEL for: n_layers out of range; in/out out of
 * range; first in != 2; last out != 3; out of layer l != in of layer l+1; bits not
 * in {0, 2..8, 16}; zp outside [0, 2^bits); a kept code >= 2^bits; non-finite scale,
 * bias or kept fp32 weight; NULL weights or bias.  RINR_E_ARG for n_models < 0 or
 * non-finite / zero-span opts. */
int rinr_pack_size(const rinr_model_desc *models, int64_t n_models, const rinr_store_opts *opts,
                   size_t *bytes);
int rinr_pack(const rinr_model_desc *models, int64_t n_models, const rinr_store_opts *opts,
              void *host_blob, size_t bytes);

/* Inverse of rinr_pack for ONE layer of ONE model, on the host (round-trip tests,
 * tooling; not used by decode).  Reads a host copy of the blob and writes one entry
 * per weight: codes_out (uint16_t[out*in], the stored code, or 0 where pruned; for
 * bits == 0 unused and may be NULL), f32_out (float[out*in] dequantised weights,
 * 0 where pruned), keep_out (uint8_t[out*in] 0/1), bias_out (float[out]).  Any
 * output pointer may be NULL.  meta_out (may be NULL) receives
 * {in, out, bits, zp, n_kept} and *scale_out the scale. */
int rinr_unpack_layer(const void *host_blob, size_t bytes, int64_t model, int32_t layer,
                      uint16_t *codes_out, float *f32_out, uint8_t *keep_out, float *bias_out,
                      int32_t meta_out[5], float *scale_out);

/* ---- device-resident store ------------------------------------------------------ */
typedef struct rinr_store rinr_store;

/* Options of rinr_store_open_ex.  NULL, or a zero in a field, means the default. */
typedef struct {
    int32_t fp32_tile_rows;  /* MFMA tile of the fp32 kernels at padded widths 32 and 64: 32 (32x32x2, default)
                                or 16 (16x16x4).  Fixes the kernels' on-chip weight layout for this store. */
    int32_t lds_budget;      /* on-chip memory a workgroup may use, in bytes: a multiple of 16 from 20480 to 163840
                                (default: all 160 KB).  Models that do not fit it are decoded with their layers
                                streamed in groups; a small budget forces that on small models (tests).        */
} rinr_open_opts;

/* Sec. III-B: the whole dataset is moved to GPU memory once, in weight form, before training starts;
 * every batch is then selected and decoded from that resident copy.  rinr_store_open makes the resident
 * copy usable: it opens a store over a blob already in device memory (device_blob, 16-byte aligned,
 * `bytes` long).  host_blob, if not NULL, is a host copy of the same bytes and is validated in full
 * (header, index, every record's offsets and sizes) without touching the device; if NULL the blob is
 * copied back from the device once, here, for the same validation.  The store neither copies nor owns
 * the blob: it must stay allocated and unchanged until rinr_store_close.  Must be called with the
 * blob's device current.  Allocates the handle and an 8-byte device status word.
 * Every store that rinr_pack writes opens: models whose expanded weights fit the 160 KB of on-chip memory
 * are decoded from a resident copy of the whole model, deeper ones with their layers streamed through it
 * in groups (slower per pixel, same results).
 * rinr_store_open == rinr_store_open_ex with opts = NULL. */
int rinr_store_open(const void *device_blob, const void *host_blob, size_t bytes, rinr_store **store);
int rinr_store_open_ex(const void *device_blob, const void *host_blob, size_t bytes, const rinr_open_opts *opts,
                       rinr_store **store);
/* Frees the handle and its status word (Sec. III-B: the resident dataset is released by its owner, the
 * caller; the blob itself is untouched).  No decode of this store may still be running. */
int rinr_store_close(rinr_store *store);
/* Size of the resident dataset (Sec. III-A: one model per image): number of models, widest hidden layer,
 * most linear layers.  Any output pointer may be NULL. */
int rinr_store_info(const rinr_store *store, int64_t *n_models, int32_t *max_width, int32_t *max_layers);
/* Worst-case output error (absolute, before any normalisation) that the reduced-precision modes can cause
 * on this store, from its own weights: bounds[0] for RINR_FLAG_FP16_ACT, bounds[1] for RINR_FLAG_FP16_ALL.
 * With |sin'| <= 1, u = 2^-12 and R_l the largest absolute row sum of layer l:
 * d_0 = u, d_l = w0 R_l (d_{l-1} + t) + u, bound = R_out d_last  (t = 2^-11 for fp16 weights, else 0).
 * A mode is used only where its bound is at most 9.5e-4 (see the flags). */
int rinr_store_error_bounds(const rinr_store *store, float bounds[2]);

/* ---- decode ------------------------------------------------------------------------ */
enum { RINR_OUT_F32 = 1,           /* out: float [n][3][H][W], clamp(y, 0, 1)                 */
       RINR_OUT_U8 = 2,            /* out: uint8 [n][3][H][W], rint(255 * clamp(y, 0, 1))     */
       RINR_OUT_F32_AND_U8 = 3 };  /* out: float tensor, opts.out_u8: uint8 tensor            */
enum { RINR_FLAG_NO_CLAMP = 1,     /* fp32 output only: write the linear output unclamped     */
       RINR_FLAG_FP32_MFMA = 2,    /* run the layers on fp32 MFMA instead of the default
                                      split-precision fp16 MFMA (hi+lo operand pairs, fp32
                                      accumulate); same results within the stated tolerance  */
       RINR_FLAG_NORMALIZE = 4,    /* fp32 output only: out = value * norm_scale[c] + norm_shift[c]
                                      per channel c, after the clamp                          */
       RINR_FLAG_FP16_ACT = 8,     /* faster, less precise: activations travel between layers as one
                                      fp16 value (relative rounding 2^-12 each) instead of a hi+lo
                                      pair; weights, coordinates and accumulation as in the default
                                      kernel.  Honoured only on stores whose a-priori error bound
                                      (rinr_store_error_bounds) is at most 9.5e-4, so that the result stays
                                      within 1e-3 of the fp64 definition; other stores are decoded by the
                                      default kernel.  Ignored together with RINR_FLAG_FP32_MFMA, and where
                                      the store is served by the fp32 kernels anyway (operands beyond fp16
                                      range)                                                            */
       RINR_FLAG_FP16_ALL = 16,    /* fastest, least precise: RINR_FLAG_FP16_ACT, and the hidden layers'
                                      weights are rounded to fp16 as well (after dequantisation and the
                                      w0 scaling): fp16 operands with fp32 accumulation throughout the
                                      hidden layers; the first and the last layer keep their hi+lo
                                      pairs.  Honoured under the same rule with its own bound; a store that
                                      passes only the RINR_FLAG_FP16_ACT bound is decoded in that mode.     */
       RINR_FLAG_FP16_UNCHECKED = 32 };
                                   /* with one of the two flags above: use the mode whatever the bound says.
                                      The bound is a worst case that grows with the product of the layers'
                                      gains; measured errors of deep models are far below it (2e-5 .. 8e-5 on
                                      the benchmark workloads) but nothing guarantees them: the caller
                                      takes the responsibility.                                            */

/* Augmentation on the GPU, fused into the decode (Sec. III-B: decoded images are augmented
 * on the GPU before they reach the backbone).  Geometric augmentation (flip, crop + resize,
 * rotation, translation, zoom) is a per-slot affine map of the sampling grid, free for a
 * resolution-free decode:  (x', y') = (A[0] x + A[1] y + A[2],  A[3] x + A[4] y + A[5])
 * with (x, y) the pixel-centre coordinate of the H x W grid; the MLP is evaluated at (x', y').
 * Photometric normalisation is RINR_FLAG_NORMALIZE. */
typedef struct {
    int32_t out_dtype;       /* RINR_OUT_*                                              */
    int32_t flags;           /* RINR_FLAG_*                                             */
    void *out_u8;            /* device; second output for RINR_OUT_F32_AND_U8, else NULL */
    const float *affine;     /* device; float[n][6], one 2x3 map per slot, or NULL = identity.
                                Mapped coordinates must stay below 6e4 in magnitude.       */
    float norm_scale[3];     /* used with RINR_FLAG_NORMALIZE, e.g. 1/std per channel      */
    float norm_shift[3];     /* used with RINR_FLAG_NORMALIZE, e.g. -mean/std per channel  */
    void *workspace;         /* device, 4-byte aligned, or NULL.  Scratch for one call: with it, a batch from
                                a store that mixes model widths or depths is decoded heaviest model first (one
                                more small kernel orders the slots), which shortens the tail of the grid;
                                results are the same bytes.  Calls that may overlap need their own.
                                The ordering kernel is one workgroup: about 6 us per thousand slots.   */
    size_t workspace_bytes;  /* >= rinr_decode_workspace_bytes(n), else RINR_E_SIZE                    */
    /* Launch shape, for experiments and tests; 0 = chosen by the library (what the benchmarks use).     */
    int32_t launch_threads;        /* threads per workgroup: a multiple of 64 up to 768                  */
    int32_t launch_blocks_per_cu;  /* fixed grid target in workgroups per compute unit (1..1024) instead of
                                      the built-in cost model's split of each slot's pixels              */
    int32_t one_grid_min_tiles;    /* stores that mix width classes decode images of at least this many
                                      64-pixel tiles in one grid, smaller ones class by class (default 64) */
} rinr_decode_opts;

/* Bytes of rinr_decode_opts.workspace a batch of n slots needs (4 per slot). */
size_t rinr_decode_workspace_bytes(int32_t n);

/* Decodes slots s = 0..n-1 (Sec. III-B: batch select + pixel- and image-parallel
 * decode): slot s shows model image_ids[s] sampled on an H x W pixel-centre grid,
 * written to out[s][c][i][j], c = 0,1,2 = R,G,B.  image_ids: device, int64[n],
 * repeats allowed.  out: device, contiguous NCHW, 4-byte aligned for fp32.
 * stream: a hipStream_t (NULL = the default stream).  Asynchronous: enqueues one kernel
 * on `stream` and returns; never synchronises, never reads the host copy of the blob.
 * n == 0 is OK and launches nothing.  Host-detectable errors (NULL, n < 0, H or W <= 0,
 * n*3*H*W overflowing int64 / the three planes of a slot >= 2^32 pixels, misaligned out or affine, bad out_dtype,
 * NO_CLAMP or NORMALIZE with a uint8 output, non-finite norm values) are returned before
 * anything is enqueued.  An id outside
 * [0, n_models) cannot be seen from the host: that slot is written as zeros and a sticky
 * device counter is incremented (read it with rinr_store_status).
 * Domain: every sine argument w0*(Wx+b) must stay within +-512*pi (the hardware sine's
 * range; sine networks stay within a few tens of radians).  The default split-precision
 * kernels also need |w * w0/2pi| and the coordinate bounds below 6e4 (fp16 range); a store
 * that breaks this is served by the fp32 MFMA kernels automatically.
 * The handle is not const: a store keeps the launch plan and the launch record of its last decode, so one
 * store is used from one host thread at a time (different stores are independent).
 * rinr_decode_batch == rinr_decode_batch_ex with {RINR_OUT_F32, 0, NULL, NULL} and no workspace. */
int rinr_decode_batch(rinr_store *models, const int64_t *image_ids, int32_t n,
                      int32_t H, int32_t W, void *out, void *stream);
int rinr_decode_batch_ex(rinr_store *models, const int64_t *image_ids, int32_t n,
                         int32_t H, int32_t W, void *out, const rinr_decode_opts *opts, void *stream);

/* For callers that cannot allocate device memory or pass a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same as rinr_decode_batch_ex, except that the heaviest-first slot order
 * (see rinr_decode_opts.workspace, which is ignored here) is kept in a static device array of the library instead:
 * 4 bytes per slot, RINR_NOALLOC_MAX_SLOTS slots = 256 KB, held on every GPU the library is used on until the
 * process ends.  n > RINR_NOALLOC_MAX_SLOTS returns RINR_E_SIZE.  The call allocates nothing and frees nothing.
 * Every call on one GPU shares that GPU's array (whatever the store): each call rewrites the entries it reads
 * before it reads them, so calls in sequence on one stream are independent, but calls that may overlap on
 * one GPU (other streams, other host threads) race on it: use rinr_decode_batch_ex with a workspace of their own. */
enum { RINR_NOALLOC_MAX_SLOTS = 65536 };
int rinr_decode_batch_noalloc(rinr_store *models, const int64_t *image_ids, int32_t n, int32_t H, int32_t W,
                              void *out, const rinr_decode_opts *opts, void *stream);

/* Sec. III-B selects the batch on the GPU with no CPU in the loop, so an id outside the dataset can only
 * be seen by the kernel: this call synchronises `stream`, then reads (and leaves set) the count of
 * out-of-range image ids seen by decodes on this store so far. */
int rinr_store_status(const rinr_store *store, int64_t *bad_id_count, void *stream);

/* Test hooks for the expand/dequantise stage (Sec. IV-A mask, Sec. IV-B codes).  They cite no passage of their
 * own: they expose, for bit-exact checks, what the decode kernels hold on chip after running the same device
 * routine the decode uses to rebuild layer `layer` of model `id` from the packed record.  No sine pre-scaling
 * is applied.  Outputs are device pointers, row-major [out][in], 0 where pruned; bias_out (float[out]) may be NULL.
 * rinr_debug_dequant: the fp32 kernels' layout; the values are bit-comparable with scale * (code - zp) rounded
 * once to fp32.
 * rinr_debug_dequant_split: the split-precision kernels' fp16 operand blocks.  For a 2..8-bit hidden layer hi_out
 * is the integer code - zp the matrix cores multiply by, lo_out is 0 and *scale_out the multiplier applied to
 * the accumulator; for every other layer hi_out = fp16(w) and lo_out = fp16(w - hi) as floats and *scale_out = 1.
 * The first layer's operand block holds its weights several times (once per pixel tile and operand slot): an
 * entry whose copies disagree is written as NaN.  bias_out receives what the bias tile holds (bias / scale for
 * a 2..8-bit hidden layer).  fp16_weights != 0 exports the RINR_FLAG_FP16_ALL form: hi_out = fp16(w). */
int rinr_debug_dequant(const rinr_store *store, int64_t id, int32_t layer, float *device_out,
                       float *bias_out, void *stream);
int rinr_debug_dequant_split(const rinr_store *store, int64_t id, int32_t layer, int32_t fp16_weights, float *hi_out,
                             float *lo_out, float *bias_out, float *scale_out, void *stream);

/* Grid the last decode on this store used (diagnostics / benchmarks):
 * info[0] = kernel launches, info[1] = workgroups, info[2] = threads per workgroup,
 * info[3] = dynamic LDS bytes per workgroup, info[4] = kernels that ran: 0 split precision (default),
 * 1 fp32 MFMA, 2 fp16 activations, 3 fp16 weights and activations, info[5] = 1 if the layers were streamed
 * through on-chip memory in groups (a model too deep to be resident), else 0. */
int rinr_last_launch_info(const rinr_store *store, int32_t info[6]);

const char *rinr_strerror(int code);
/* hipError_t of the last failed HIP call on this thread (0 if none), as an int. */
int rinr_last_hip_error(void);
const char *rinr_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RINR_H */

// Fitting one sine MLP per image on the GPU (Eq. 1): full-batch gradient of the squared error by forward and backward
// passes on the matrix cores, Adam update fused into the same kernel.  This file: the handle, the fp32 kernels described
// next, the host side of both families; the split-precision kernels (fp16 hi/lo operand pairs) are rinr_fit16.hip.h.
//
// One workgroup per image, one launch per step.  The image's weights live in LDS (bias folded in as an
// extra input column that multiplies a row of ones), pixels are taken in chunks of PC, and every
// contraction of a chunk is a set of 16x16 output tiles computed with v_mfma_f32_16x16x4_f32 from LDS
// operands:
//     forward        Z_l [d_out x PC]  = W_l [d_out x d_in+1] . H_l [d_in+1 x PC]        H_{l+1} = sin(w0 Z_l)
//     weight grads   dW_l [d_out x d_in+1] += D_l [d_out x PC] . H_l^T                   (contraction over pixels)
//     backward       D_{l-1} = (W_l^T . D_l) * w0 cos(w0 Z_{l-1})
// In LDS the sine layers' weights and biases are held times w0 / 2pi, so that Z comes out in revolutions, the unit of
// the hardware sine and cosine, and the error is carried as E_l = c_l D_l with c_{L-1} = 1, c_{L-2} = 1 / w0,
// c_{l-1} = c_l / 2pi below that: then E_{l-1} = (W_l^T . E_l) * cos(2pi Z'_{l-1}) with the LDS weights, one multiply per
// element, and the accumulated sum over pixels of E_l H_l^T is c_l times the gradient: the factor 1 / c_l is applied
// once per parameter at the end.
// The weight-gradient tiles stay in registers for the whole step (each wavefront owns a fixed set of
// tiles of every layer), so gradients never touch memory: at the end of the step the owner of an entry
// applies Adam to it in place.  Nothing is allocated and nothing leaves the workgroup except the
// parameters, the moments and one loss value.
#include "../../include/rinr_fit.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxL = RINR_FIT_MAX_LAYERS;
// The kernels are built per hidden width rounded up to a multiple of 8 (WQ) and per depth bucket.
// Row tiles of a hidden layer: MT = ceil(WQ / 16).
constexpr int fit_tiles(int wq) { return (wq + 15) / 16; }
// Wavefronts per workgroup (= per image).  Every phase between two barriers is a short dependent chain per
// wavefront, so what fills the matrix pipe is other wavefronts: 4 at widths <= 16, whose 4 tiles per layer do not feed
// more, and several images per CU; 8 at widths <= 32, two images per CU; 12 at widths <= 48, one wavefront per tile of
// their 12-tile layers (LDS holds one image); 16 above, one per forward tile, so that the 20 gradient tiles of a
// width-64 layer take two rounds instead of three (+3 %, a few spilled registers notwithstanding).
constexpr int fit_waves(int wq) { return fit_tiles(wq) == 1 ? 4 : (fit_tiles(wq) == 2 ? 8 : (fit_tiles(wq) == 3 ? 12 : 16)); }
// Wavefronts per SIMD the kernel is compiled for (the register budget follows): at widths <= 32 two workgroups
// share a CU (10 x 32 at 224 x 224, 512 images: 26.8 -> 20.3 ms per step).
constexpr int fit_waves_per_simd(int wq) { return fit_tiles(wq) == 1 ? 3 : (fit_tiles(wq) == 3 ? 3 : 4); }
// Layer counts the kernels are built for: the accumulators of all layers stay in registers, so the depth
// is a compile-time bound and a shallow model takes the kernel with the smaller one.
constexpr int fit_depth_lo(int wq) { return fit_tiles(wq) == 1 ? 4 : (fit_tiles(wq) == 4 ? 7 : 10); }
constexpr int fit_depth_hi(int wq) { return fit_tiles(wq) <= 2 ? kMaxL : fit_depth_lo(wq); }
constexpr uint32_t kLdsLimit = 160 * 1024;

thread_local int g_fit_last_hip = 0;
inline bool hip_fail(hipError_t e) {
    if (e == hipSuccess) return false;
    g_fit_last_hip = (int)e;
    return true;
}
#define FIT_HIP(call) do { if (hip_fail(call)) return RINR_E_HIP; } while (0)

// Shapes for hidden widths <= WQ (a multiple of 8) and the LDS layout in floats.  Padding is with zero weights, which
// leaves values and gradients of the real entries unchanged (a padded unit outputs sin(0) = 0 and receives no
// error), so every hidden layer has the same compile-time shape whatever its true width.  Pixels are taken 64 at a time.
// A layer's input is a block of four rows (ones, and three rows whose weights are zero) followed by the activations:
// the bias is the weight of the row of ones, the contraction over the inputs takes 1 + WQ / 4 k-steps of four rows, and
// what lies beyond row 4 + WQ is never read.  The first layer's block is (ones, x, y, zero) and is its whole input.
// LDS has 32 banks and serves a wavefront's 4-byte accesses in two halves of 32 lanes; a half that hits a bank
// twice takes a second cycle.  The MFMA operands are read in two patterns, lane (m, kq) -> (row m, column kq) and
// -> (row kq, column m), so a half covers 16 rows x 2 columns or 2 rows x 16 columns.  Weight rows have stride
// LD = 2 * odd, which makes the first pattern conflict-free.  Pixel-buffer rows come in pairs: row r starts at
// prow(r) = (r / 2) * PAIR + (r % 2) * ODD with PAIR = 2 * odd and ODD = 16 (mod 32), so that 16 consecutive rows
// start in 16 different even banks and the two rows of a pair are 16 banks apart: both patterns conflict-free
// (ODD = 80 is the first such value that holds 64 pixels, PAIR = 146 the first that holds two rows).
//   W0  [RO][6]        first layer: columns bias, x, y, 0
//   Wh  [RO][LD] each  layers 1..L-2: columns bias, 0, 0, 0, then the weights (RO = 16 MT rows, zero beyond the width)
//   Wl  [16][LD]       last layer (3 real rows)
//   B0, B1, B2 [KR rows] three pixel buffers.  Forward: the input of layer l is B[l & 1] (row 0 ones, rows 4.. the
//       activations; B0 rows 1..3 hold x, y, 0).  Backward: B0 holds the restored input of the layer at hand; B1 / B2
//       the back-propagated error with row = unit, ping-pong (so B1's row of ones is written again for every chunk).
//   B3 [KR rows]       with PIPE: the restored layer inputs alternate between B0 and B3.
// Pre-activations are not stashed in LDS: the wavefront that computed a tile keeps it in registers until the
// backward pass has used it (sine again for the weight gradient's operand, cosine for the error).
template <int WQ> struct Shape {
    static constexpr int PC = 64, PT = PC / 16;
    static constexpr int MT = fit_tiles(WQ), RO = 16 * MT, LD = RO + 6, KR = RO + 4;
    static constexpr int KSF = 1 + WQ / 4;                          // k-steps of a hidden layer's forward contraction
    static constexpr int KSB = WQ / 4;                              // ... of the backward one (over the layer's outputs)
    static constexpr int NIT = (4 + WQ + 15) / 16;                  // column tiles of a hidden weight gradient (block of four + inputs)
    static constexpr int PAIR = 146, ODD = 80;
    static __host__ __device__ constexpr int prow(int r) { return (r >> 1) * PAIR + (r & 1) * ODD; }
    static constexpr int ML = fit_depth_hi(WQ);                     // deepest model: register budget (and LDS at width 64)
    static constexpr int NW = fit_waves(WQ), NTHREADS = NW * 64;
    static constexpr int ZSLOTS = (MT * PT + NW - 1) / NW;  // forward tiles a wavefront owns per layer
    static constexpr int GSLOTS = (MT * NIT + NW - 1) / NW; // gradient tiles a wavefront owns per layer
    static __host__ __device__ constexpr int w_off(int l) { return l == 0 ? 0 : RO * 6 + (l - 1) * RO * LD; }
    static __host__ __device__ constexpr int w_end(int L) { return RO * 6 + (L - 2) * RO * LD + 16 * LD; }
    static __host__ __device__ constexpr int buf(int b, int L) { return w_end(L) + b * prow(KR); }
    // A fourth buffer, where LDS has room for it (one image per CU at widths 33..48, small models at widths <= 16):
    // the backward pass then restores the next layer's input while it works on this one, one barrier less per layer.
    static constexpr bool PIPE = MT == 1 || MT == 3;
    static __host__ __device__ constexpr int total(int L) { return buf(PIPE ? 4 : 3, L); }
};

struct FitArgs {
    float *params, *m, *v;        // [n_images][n_params]
    const uint8_t *keep;          // [n_images][n_params] or null
    const float *target;          // [n_images][3][HW]
    float *loss;                  // [n_images]
    float *emag;                  // [n_images] root-mean-square output error the last step saw (split-precision kernel's error scale); may be null
    float *grad_out;              // null: Adam update; else the gradient is written here and nothing is updated
    int64_t n_params;
    uint32_t HW, W;
    float inv2W, inv2H, lo, span, w0rev;        // w0rev = w0 / 2pi
    float loss_scale;
    float neg1;                   // -1, as data: keeps x - float(half) a single mixed-precision fma in the split kernels
    float lr, c1inv, c2inv, b1, b2, eps;
    int32_t L;
    int32_t d[kMaxL + 1];         // true widths
    int32_t p_off[kMaxL];         // offset of W_l in the parameter vector
    float gscale[kMaxL];          // what the accumulated weight gradient of layer l is multiplied by (see the kernel)
};

__device__ __forceinline__ f32x4 mfma4(float a, float b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }

// acc += sum over KSTEPS k-steps of A(ks) x B(ks): one float per lane from LDS at ap[ks * AS], bp[ks * BS].
// Trip count and strides are compile-time, so the loads become immediate-offset reads issued ahead of the MFMAs
// (in groups of eight, which bounds the registers held).
// ZERO: the sum starts at 0 (as the first MFMA's inline-constant C operand: no registers are cleared).
template <int KSTEPS, int AS, int BS, bool ZERO>
__device__ __forceinline__ f32x4 contract(const float *ap, const float *bp, f32x4 acc) {
#pragma unroll
    for (int k0 = 0; k0 < KSTEPS; k0 += 8) {
        constexpr int G = 8;
        float av[G], bv[G];
#pragma unroll
        for (int u = 0; u < G; ++u)
            if (k0 + u < KSTEPS) {
                av[u] = ap[(k0 + u) * AS];
                bv[u] = bp[(k0 + u) * BS];
            }
#pragma unroll
        for (int u = 0; u < G; ++u)
            if (k0 + u < KSTEPS) acc = mfma4(av[u], bv[u], (ZERO && k0 + u == 0) ? (f32x4){0.0f, 0.0f, 0.0f, 0.0f} : acc);
    }
    return acc;
}

}  // namespace
#include "rinr_fit16.hip.h"
namespace {

// Where entry (o, i) of layer l's weight-gradient tile lives in the parameter vector, or -1 (padding).
// Column 0 is the bias; input j is column 1 + j of the first layer and column 4 + j of the others.
__device__ __forceinline__ int param_index(const FitArgs &a, int l, int o, int i) {
    const int din = a.d[l], dout = a.d[l + 1];
    if (o >= dout) return -1;
    if (i == 0) return a.p_off[l] + dout * din + o;
    const int j = i - (l == 0 ? 1 : 4);
    if (j >= 0 && j < din) return a.p_off[l] + o * din + j;
    return -1;
}

template <int WQ, int ML>
__global__ __launch_bounds__(Shape<WQ>::NTHREADS, fit_waves_per_simd(WQ)) void fit_step_kernel(const FitArgs a) {
    typedef Shape<WQ> S;
    constexpr int MT = S::MT, LD = S::LD, KR = S::KR, KSF = S::KSF, KSB = S::KSB, PC = S::PC, PT = S::PT, NIT = S::NIT;
    constexpr int PSTEP = 2 * S::PAIR;       // prow(r + 4) - prow(r): one k-step down a pixel buffer
    constexpr int ZSLOTS = S::ZSLOTS, GSLOTS = S::GSLOTS, kWaves = S::NW, kThreads = S::NTHREADS;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    __shared__ float red[kWaves];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, m = lane & 15, kq = lane >> 4;
    const size_t img = blockIdx.x;
    float *P = a.params + img * a.n_params;
    const f32x4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    constexpr bool PIPE = S::PIPE;
    float *const B0 = lds + S::buf(0, a.L), *const B1 = lds + S::buf(1, a.L), *const B2 = lds + S::buf(2, a.L);
    float *const B3 = PIPE ? lds + S::buf(3, a.L) : B0;

    // ---- set up: zero everything, then the weights (sine layers times w0 / 2pi) behind their bias column
    for (int q = tid; q < S::total(a.L); q += kThreads) lds[q] = 0.0f;
    __syncthreads();
    for (int l = 0; l < a.L; ++l) {
        const int din = a.d[l], dout = a.d[l + 1], ld = l == 0 ? 6 : LD, first = l == 0 ? 1 : 4;
        float *Wt = lds + S::w_off(l);
        const float *src = P + a.p_off[l];
        const float sc = l < a.L - 1 ? a.w0rev : 1.0f;
        for (int e = tid; e < dout * din; e += kThreads) Wt[(e / din) * ld + first + e % din] = src[e] * sc;
        for (int o = tid; o < dout; o += kThreads) Wt[o * ld] = src[dout * din + o] * sc;
    }
    if (PIPE && tid < PC) B3[S::prow(0) + tid] = 1.0f;       // its row of ones; nothing else ever writes its rows 0..3
    __syncthreads();

    f32x4 acc[ML][GSLOTS];          // weight-gradient tiles, whole step
    f32x4 zst[ML][ZSLOTS];          // pre-activation tiles of the chunk at hand
#pragma unroll
    for (int l = 0; l < ML; ++l) {
#pragma unroll
        for (int s = 0; s < GSLOTS; ++s) acc[l][s] = zero4;
#pragma unroll
        for (int s = 0; s < ZSLOTS; ++s) zst[l][s] = zero4;
    }
    float loss_part = 0.0f;

    // rows ones, x, y, zero of B0: the first layer's input at the chunk's pixel centres (a ragged last chunk
    // repeats the last pixel; its error is zeroed)
    auto put_coords = [&](uint32_t c) {
        if (tid < PC) {
            uint32_t p = c * PC + tid;
            p = p < a.HW ? p : a.HW - 1;
            const uint32_t row = p / a.W, col = p - row * a.W;
            B0[S::prow(0) + tid] = 1.0f;
            B0[S::prow(1) + tid] = fmaf(a.span, (float)(2 * col + 1) * a.inv2W, a.lo);
            B0[S::prow(2) + tid] = fmaf(a.span, (float)(2 * row + 1) * a.inv2H, a.lo);
            B0[S::prow(3) + tid] = 0.0f;
        }
    };

    const uint32_t nchunks = (a.HW + PC - 1) / PC;
    for (uint32_t c = 0; c < nchunks; ++c) {
        // the layer count is read afresh per chunk: otherwise every "l < L" and "l == L - 1" of the unrolled layers is
        // kept as a lane mask across the loop, and the masks spill out of the scalar registers
        int L = a.L;
        asm volatile("" : "+s"(L));
        put_coords(c);
        if (tid >= kThreads - PC) B1[S::prow(0) + tid - (kThreads - PC)] = 1.0f;     // the backward pass kept errors here
        __syncthreads();
        // ---- forward: Z_l = W_l H_l, one 16x16 tile (rows mt, pixels nt) per task; H_{l+1} = sin(2pi Z_l)
#pragma unroll
        for (int l = 0; l < ML; ++l) {
            if (l < L) {
                const bool last = l == L - 1;
                const float *in = (l & 1) ? B1 : B0;
                float *out = (l & 1) ? B0 : B1;
                const int ntasks = (last ? 1 : MT) * PT;
#pragma unroll
                for (int s = 0; s < ZSLOTS; ++s) {
                    const int task = wave + s * kWaves;
                    if (task < ntasks) {
                        const int mt = task / PT, nt = task - mt * PT, col = nt * 16 + m;
                        f32x4 z;
                        if (l == 0)
                            z = contract<1, 4, PSTEP, true>(lds + S::w_off(0) + (mt * 16 + m) * 6 + kq, in + S::prow(kq) + col, zero4);
                        else
                            z = contract<KSF, 4, PSTEP, true>(lds + S::w_off(l) + (mt * 16 + m) * LD + kq, in + S::prow(kq) + col, zero4);
                        if (!last) {
                            zst[l][s] = z;
#pragma unroll
                            for (int v = 0; v < 4; ++v) out[S::prow(4 + mt * 16 + 4 * kq + v) + col] = __builtin_amdgcn_sinf(z[v]);
                        } else {
                            const uint32_t pix = c * PC + col;
#pragma unroll
                            for (int v = 0; v < 4; ++v) {
                                const int o = 4 * kq + v;
                                float e = 0.0f;
                                if (o < 3 && pix < a.HW) e = z[v] - a.target[(img * 3 + o) * a.HW + pix];
                                loss_part = fmaf(e, e, loss_part);
                                B2[S::prow(o) + col] = 2.0f * a.loss_scale * e;
                            }
                        }
                    }
                }
                __syncthreads();
            }
        }
        // ---- backward, layer by layer: restore H_l (the layer's input); then dW_l += E_l H_l^T into this wavefront's
        //      accumulators (tile rows ot, columns it) and E_{l-1} = (W_l^T E_l) * cos(2pi z_{l-1}) (tile rows it, pixels nt).
        //      With PIPE only the first of these layers restores its own input ahead; every layer restores the next one's
        //      into the other H buffer while it computes.
        auto restore = [&](int l, float *H) {          // l is a constant after unrolling
            if (l == 0) {
                put_coords(c);                         // B0, which is where layer 0's input is expected
            } else {
#pragma unroll
                for (int s = 0; s < ZSLOTS; ++s) {
                    const int task = wave + s * kWaves;
                    if (task < MT * PT) {
                        const int mt = task / PT, nt = task - mt * PT, col = nt * 16 + m;
#pragma unroll
                        for (int v = 0; v < 4; ++v) H[S::prow(4 + mt * 16 + 4 * kq + v) + col] = __builtin_amdgcn_sinf(zst[l - 1][s][v]);
                    }
                }
            }
        };
        float *Dc = B2, *Dn = B1;
#pragma unroll
        for (int l = ML - 1; l >= 0; --l) {
            if (l < L) {
                const bool last = l == L - 1;
                float *const Hc = (PIPE && (l & 1)) ? B3 : B0;      // holds H_l
                float *const Hn = (PIPE && !(l & 1)) ? B3 : B0;     // PIPE: receives H_{l-1}
                if (!PIPE || last) {
                    restore(l, Hc);
                    __syncthreads();
                }
                if (l == 0) {
#pragma unroll
                    for (int s = 0; s < GSLOTS; ++s) {
                        const int ot = wave + s * kWaves;        // columns ones, x, y; the other lanes read the zero row
                        if (ot < MT) acc[0][s] = contract<PC / 4, 4, 4, false>(Dc + S::prow(ot * 16 + m) + kq, Hc + S::prow(m < 4 ? m : 3) + kq, acc[0][s]);
                    }
                } else {
                    const int ntasks = (last ? 1 : MT) * NIT;
#pragma unroll
                    for (int s = 0; s < GSLOTS; ++s) {
                        const int task = wave + s * kWaves;
                        if (task < ntasks) {
                            const int ot = task / NIT, it = task - ot * NIT, i = it * 16 + m;
                            // columns beyond the buffer's rows read the buffer's zero row
                            acc[l][s] = contract<PC / 4, 4, 4, false>(Dc + S::prow(ot * 16 + m) + kq, Hc + S::prow(i < KR ? i : 3) + kq, acc[l][s]);
                        }
                    }
                    const float *Wt = lds + S::w_off(l);
#pragma unroll
                    for (int s = 0; s < ZSLOTS; ++s) {
                        const int task = wave + s * kWaves;
                        if (task < MT * PT) {
                            const int it = task / PT, nt = task - it * PT, col = nt * 16 + m;
                            const float *ap = Wt + kq * LD + 4 + it * 16 + m, *bp = Dc + S::prow(kq) + col;
                            const f32x4 g = last ? contract<1, 4 * LD, PSTEP, true>(ap, bp, zero4) : contract<KSB, 4 * LD, PSTEP, true>(ap, bp, zero4);
#pragma unroll
                            for (int v = 0; v < 4; ++v)
                                Dn[S::prow(it * 16 + 4 * kq + v) + col] = g[v] * __builtin_amdgcn_cosf(zst[l - 1][s][v]);
                        }
                    }
                    if (PIPE) restore(l - 1, Hn);
                }
                __syncthreads();
                float *t = Dc;
                Dc = Dn;
                Dn = t;
            }
        }
    }
    const int L = a.L;

    // ---- loss of this step's parameters
    for (int off = 32; off > 0; off >>= 1) loss_part += __shfl_xor(loss_part, off, 64);
    if (lane == 0) red[wave] = loss_part;
    __syncthreads();
    if (tid == 0) {
        float s = 0.0f;
        for (int w = 0; w < kWaves; ++w) s += red[w];
        a.loss[img] = a.loss_scale * s;
    }

    // ---- every gradient entry is in exactly one lane: Adam in place (or hand the gradient out)
    float *M = a.m + img * a.n_params, *V = a.v + img * a.n_params;
    const uint8_t *K = a.keep ? a.keep + img * a.n_params : nullptr;
    float *G = a.grad_out ? a.grad_out + img * a.n_params : nullptr;
#pragma unroll
    for (int l = 0; l < ML; ++l) {
        if (l < L) {
            const int nit = l == 0 ? 1 : NIT, ntasks = (l == L - 1 ? 1 : MT) * nit;
#pragma unroll
            for (int s = 0; s < GSLOTS; ++s) {
                const int task = wave + s * kWaves;
                if (task < ntasks) {
                    const int ot = task / nit, it = task - ot * nit;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int at = param_index(a, l, ot * 16 + 4 * kq + v, it * 16 + m);
                        if (at >= 0) {
                            const bool kept = !K || K[at];
                            const float g = kept ? acc[l][s][v] * a.gscale[l] : 0.0f;
                            if (G) {
                                G[at] = g;
                            } else if (kept) {
                                const float mm = a.b1 * M[at] + (1.0f - a.b1) * g;
                                const float vv = a.b2 * V[at] + (1.0f - a.b2) * g * g;
                                M[at] = mm;
                                V[at] = vv;
                                P[at] -= a.lr * (mm * a.c1inv) / (sqrtf(vv * a.c2inv) + a.eps);
                            } else {
                                P[at] = 0.0f;
                            }
                        }
                    }
                }
            }
        }
    }
}

typedef void (*fit_fn)(const FitArgs);

template <int WQ> fit_fn kernel_of(int L) {
    if (L <= fit_depth_lo(WQ)) return fit_step_kernel<WQ, fit_depth_lo(WQ)>;
    return fit_step_kernel<WQ, fit_depth_hi(WQ)>;
}
// wq: the widest hidden layer rounded up to a multiple of 8
fit_fn kernel_for(int wq, int L) {
    switch (wq) {
        case 8: return kernel_of<8>(L);
        case 16: return kernel_of<16>(L);
        case 24: return kernel_of<24>(L);
        case 32: return kernel_of<32>(L);
        case 40: return kernel_of<40>(L);
        case 48: return kernel_of<48>(L);
        case 56: return kernel_of<56>(L);
        default: return kernel_of<64>(L);
    }
}
template <int WQ> int lds_floats_of(int L) { return L <= Shape<WQ>::ML ? Shape<WQ>::total(L) : 0; }
// LDS floats of a model of L linear layers at rounded width wq, or 0 if no kernel is built that deep
int lds_floats(int wq, int L) {
    switch (wq) {
        case 8: return lds_floats_of<8>(L);
        case 16: return lds_floats_of<16>(L);
        case 24: return lds_floats_of<24>(L);
        case 32: return lds_floats_of<32>(L);
        case 40: return lds_floats_of<40>(L);
        case 48: return lds_floats_of<48>(L);
        case 56: return lds_floats_of<56>(L);
        default: return lds_floats_of<64>(L);
    }
}


// ---- the split-precision kernels (rinr_fit16.hip.h): built per hidden width rounded up to a multiple of 16 and per depth bucket
constexpr int fit16_depth_lo(int wp) { return wp == 16 ? 4 : 6; }
constexpr int fit16_depth_hi(int wp) { return wp <= 32 ? kMaxL : (wp == 48 ? 10 : 6); }
// Plane sets: two layers per pair of barriers where LDS holds two sets of pixel planes (padded widths 16 and 32), else one.
template <int WP, int PL> fit_fn kernel16_of(int L) {
    if (L <= fit16_depth_lo(WP)) return fit16::fit16_step_kernel<WP, fit16_depth_lo(WP), PL>;
    return fit16::fit16_step_kernel<WP, fit16_depth_hi(WP), PL>;
}
fit_fn kernel16_for(int wp, int L, int pl) {
    switch (wp) {
        case 16: return pl == 2 ? kernel16_of<16, 2>(L) : kernel16_of<16, 1>(L);
        case 32: return pl == 2 ? kernel16_of<32, 2>(L) : kernel16_of<32, 1>(L);
        case 48: return kernel16_of<48, 1>(L);
        default: return kernel16_of<64, 1>(L);
    }
}
// LDS bytes of a model of L linear layers at padded width wp with pl plane sets, or 0 if no split kernel is built that deep
uint32_t lds_bytes16(int wp, int L, int pl) {
    if (L > fit16_depth_hi(wp) || (pl == 2 && wp > 32)) return 0;
    switch (wp) {
        case 16: return pl == 2 ? fit16::Shape<16, 2>::total(L) : fit16::Shape<16, 1>::total(L);
        case 32: return pl == 2 ? fit16::Shape<32, 2>::total(L) : fit16::Shape<32, 1>::total(L);
        case 48: return fit16::Shape<48, 1>::total(L);
        default: return fit16::Shape<64, 1>::total(L);
    }
}

}  // namespace

struct rinr_fit {
    rinr_fit_arch arch;
    int64_t n_images, n_params;
    int32_t H, W;
    int wq, lds_floats;         // wq: widest hidden layer rounded up to a multiple of 8 (fp32 kernels); lds_floats 0 = no fp32 kernel fits
    int family;                 // RINR_FIT_KERNEL_FP32 or RINR_FIT_KERNEL_SPLIT16: the kernels this handle's steps run
    int wp;                     // widest hidden layer rounded up to a multiple of 16 (split kernels)
    uint32_t lds16;             // their LDS bytes
    int pl16;                   // their plane sets (layers per pair of barriers)
    float *emag;                // [n_images] error size seen by the last step (split kernels' error scale); 0 = none yet
    int32_t p_off[kMaxL];
    float *params, *m, *v, *loss, *scratch_grad;
    uint8_t *keep;            // null until set
    bool has_keep;
    int64_t t;                // Adam steps taken
};

extern "C" int rinr_fit_create_ex(const rinr_fit_arch *arch, int64_t n_images, int32_t H, int32_t W, uint32_t flags, rinr_fit **out) {
    if (!arch || !out) return RINR_E_NULL;
    *out = nullptr;
    if (arch->n_layers < 2 || arch->n_layers > kMaxL || n_images < 0 || H <= 0 || W <= 0) return RINR_E_ARG;
    if (flags & ~(uint32_t)RINR_FIT_FLAG_FP32_MFMA) return RINR_E_ARG;
    if ((int64_t)H * W >= ((int64_t)1 << 31) || n_images > ((int64_t)1 << 31) - 1) return RINR_E_SIZE;
    if (arch->widths[0] != 2 || arch->widths[arch->n_layers] != 3) return RINR_E_ARG;
    for (int l = 1; l < arch->n_layers; ++l)
        if (arch->widths[l] < 1 || arch->widths[l] > RINR_MAX_WIDTH) return RINR_E_ARG;
    if (!(arch->coord_hi > arch->coord_lo) || !std::isfinite(arch->w0) || !std::isfinite(arch->coord_lo) ||
        !std::isfinite(arch->coord_hi))
        return RINR_E_ARG;
    rinr_fit *f = new (std::nothrow) rinr_fit();
    if (!f) return RINR_E_SIZE;
    f->arch = *arch;
    f->n_images = n_images;
    f->H = H;
    f->W = W;
    int wmax = 1;
    for (int l = 1; l < arch->n_layers; ++l) wmax = arch->widths[l] > wmax ? arch->widths[l] : wmax;
    f->wq = (wmax + 7) / 8 * 8;
    f->wp = (wmax + 15) / 16 * 16;
    f->lds_floats = lds_floats(f->wq, arch->n_layers);
    if ((size_t)f->lds_floats * 4 + 256 > kLdsLimit) f->lds_floats = 0;
    f->pl16 = 2;
    f->lds16 = lds_bytes16(f->wp, arch->n_layers, 2);
    if (f->lds16 == 0 || (size_t)f->lds16 + 256 > kLdsLimit) {
        f->pl16 = 1;
        f->lds16 = lds_bytes16(f->wp, arch->n_layers, 1);
        if ((size_t)f->lds16 + 256 > kLdsLimit) f->lds16 = 0;
    }
    // the split-precision kernels where they are built for the shape, the fp32 ones otherwise or on request
    f->family = (f->lds16 && !(flags & RINR_FIT_FLAG_FP32_MFMA)) ? RINR_FIT_KERNEL_SPLIT16 : RINR_FIT_KERNEL_FP32;
    if (f->family == RINR_FIT_KERNEL_FP32 && f->lds_floats == 0) { delete f; return RINR_E_UNSUPPORTED; }
    f->n_params = 0;
    for (int l = 0; l < arch->n_layers; ++l) {
        f->p_off[l] = (int32_t)f->n_params;
        f->n_params += (int64_t)arch->widths[l + 1] * (arch->widths[l] + 1);
    }
    const size_t ni = (size_t)(n_images > 0 ? n_images : 1);
    const size_t np = ni * (size_t)f->n_params;
    f->params = f->m = f->v = f->loss = f->scratch_grad = f->emag = nullptr;
    f->keep = nullptr;
    f->has_keep = false;
    f->t = 0;
    const void *fn = f->family == RINR_FIT_KERNEL_SPLIT16 ? (const void *)kernel16_for(f->wp, arch->n_layers, f->pl16)
                                                         : (const void *)kernel_for(f->wq, arch->n_layers);
    if (hip_fail(hipMalloc((void **)&f->params, np * 4)) || hip_fail(hipMalloc((void **)&f->m, np * 4)) ||
        hip_fail(hipMalloc((void **)&f->v, np * 4)) || hip_fail(hipMalloc((void **)&f->keep, np)) ||
        hip_fail(hipMalloc((void **)&f->loss, ni * 4)) || hip_fail(hipMalloc((void **)&f->emag, ni * 4)) ||
        hip_fail(hipMemset(f->params, 0, np * 4)) || hip_fail(hipMemset(f->m, 0, np * 4)) ||
        hip_fail(hipMemset(f->v, 0, np * 4)) || hip_fail(hipMemset(f->loss, 0, ni * 4)) || hip_fail(hipMemset(f->emag, 0, ni * 4)) ||
        hip_fail(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit - 256))) {
        rinr_fit_destroy(f);
        return RINR_E_HIP;
    }
    *out = f;
    return RINR_OK;
}

extern "C" int rinr_fit_create(const rinr_fit_arch *arch, int64_t n_images, int32_t H, int32_t W, rinr_fit **out) {
    return rinr_fit_create_ex(arch, n_images, H, W, 0u, out);
}

extern "C" int rinr_fit_kernel_family(const rinr_fit *f) { return f ? f->family : RINR_E_NULL; }

extern "C" int rinr_fit_destroy(rinr_fit *f) {
    if (!f) return RINR_OK;
    (void)hipFree(f->params);
    (void)hipFree(f->m);
    (void)hipFree(f->v);
    (void)hipFree(f->keep);
    (void)hipFree(f->loss);
    (void)hipFree(f->scratch_grad);
    (void)hipFree(f->emag);
    delete f;
    return RINR_OK;
}

extern "C" int64_t rinr_fit_n_params(const rinr_fit *f) { return f ? f->n_params : -1; }

namespace {
// masked parameters are zero: done on the host copy before upload, or by a download/upload round trip
int apply_keep_to_device_params(rinr_fit *f, const uint8_t *keep_host) {
    const size_t np = (size_t)f->n_images * (size_t)f->n_params;
    if (np == 0) return RINR_OK;
    std::vector<float> p;
    try { p.resize(np); } catch (const std::bad_alloc &) { return RINR_E_SIZE; }
    FIT_HIP(hipMemcpy(p.data(), f->params, np * 4, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < np; ++i)
        if (!keep_host[i]) p[i] = 0.0f;
    FIT_HIP(hipMemcpy(f->params, p.data(), np * 4, hipMemcpyHostToDevice));
    return RINR_OK;
}
}  // namespace

extern "C" int rinr_fit_reset_optimizer(rinr_fit *f) {
    if (!f) return RINR_E_NULL;
    const size_t np = (size_t)f->n_images * (size_t)f->n_params;
    FIT_HIP(hipDeviceSynchronize());
    if (np) {
        FIT_HIP(hipMemset(f->m, 0, np * 4));
        FIT_HIP(hipMemset(f->v, 0, np * 4));
    }
    if (f->n_images) FIT_HIP(hipMemset(f->emag, 0, (size_t)f->n_images * 4));      // a new round: no error history
    f->t = 0;
    return RINR_OK;
}

extern "C" int rinr_fit_set_params(rinr_fit *f, const float *params) {
    if (!f || (!params && f->n_images > 0)) return RINR_E_NULL;
    const size_t np = (size_t)f->n_images * (size_t)f->n_params;
    FIT_HIP(hipDeviceSynchronize());
    if (np) FIT_HIP(hipMemcpy(f->params, params, np * 4, hipMemcpyHostToDevice));
    int rc = rinr_fit_reset_optimizer(f);
    if (rc) return rc;
    if (f->has_keep && np) {
        std::vector<uint8_t> k;
        try { k.resize(np); } catch (const std::bad_alloc &) { return RINR_E_SIZE; }
        FIT_HIP(hipMemcpy(k.data(), f->keep, np, hipMemcpyDeviceToHost));
        return apply_keep_to_device_params(f, k.data());
    }
    return RINR_OK;
}

extern "C" int rinr_fit_set_keep(rinr_fit *f, const uint8_t *keep) {
    if (!f) return RINR_E_NULL;
    const size_t np = (size_t)f->n_images * (size_t)f->n_params;
    FIT_HIP(hipDeviceSynchronize());
    if (f->n_images) FIT_HIP(hipMemset(f->emag, 0, (size_t)f->n_images * 4));
    if (!keep) { f->has_keep = false; return RINR_OK; }
    if (np) FIT_HIP(hipMemcpy(f->keep, keep, np, hipMemcpyHostToDevice));
    f->has_keep = true;
    return np ? apply_keep_to_device_params(f, keep) : RINR_OK;
}

extern "C" int rinr_fit_get_params(const rinr_fit *f, float *params, void *stream) {
    if (!f || (!params && f->n_images > 0)) return RINR_E_NULL;
    const size_t np = (size_t)f->n_images * (size_t)f->n_params;
    FIT_HIP(hipStreamSynchronize((hipStream_t)stream));
    if (np) FIT_HIP(hipMemcpy(params, f->params, np * 4, hipMemcpyDeviceToHost));
    return RINR_OK;
}

namespace {
int launch(rinr_fit *f, const float *targets, float loss_scale, float lr, int64_t t, float b1, float b2, float eps,
           float *grad_out, hipStream_t stream) {
    FitArgs a;
    a.params = f->params; a.m = f->m; a.v = f->v;
    a.keep = f->has_keep ? f->keep : nullptr;
    a.target = targets;
    a.loss = f->loss;
    a.emag = f->emag;
    a.grad_out = grad_out;
    a.n_params = f->n_params;
    a.HW = (uint32_t)(f->H * f->W);
    a.W = (uint32_t)f->W;
    a.inv2W = 1.0f / (2.0f * (float)f->W);
    a.inv2H = 1.0f / (2.0f * (float)f->H);
    a.lo = f->arch.coord_lo;
    a.span = f->arch.coord_hi - f->arch.coord_lo;
    a.w0rev = (float)((double)f->arch.w0 / (2.0 * 3.14159265358979323846));
    a.loss_scale = loss_scale;
    a.neg1 = -1.0f;
    {
        const int L = f->arch.n_layers;
        double c = 1.0;                                   // 1 / c_l
        for (int l = L - 1; l >= 0; --l) {
            a.gscale[l] = (float)c;
            c = l == L - 1 ? (double)f->arch.w0 : c * 2.0 * 3.14159265358979323846;
        }
    }
    a.lr = lr;
    a.c1inv = (float)(1.0 / (1.0 - std::pow((double)b1, (double)t)));
    a.c2inv = (float)(1.0 / (1.0 - std::pow((double)b2, (double)t)));
    a.b1 = b1; a.b2 = b2; a.eps = eps;
    a.L = f->arch.n_layers;
    for (int l = 0; l <= a.L; ++l) a.d[l] = f->arch.widths[l];
    for (int l = 0; l < a.L; ++l) a.p_off[l] = f->p_off[l];
    if (f->family == RINR_FIT_KERNEL_SPLIT16)
        hipLaunchKernelGGL(kernel16_for(f->wp, f->arch.n_layers, f->pl16), dim3((uint32_t)f->n_images), dim3(64 * fit16::fit16_waves(f->wp)), (size_t)f->lds16, stream, a);
    else
        hipLaunchKernelGGL(kernel_for(f->wq, f->arch.n_layers), dim3((uint32_t)f->n_images), dim3(64 * fit_waves(f->wq)), (size_t)f->lds_floats * 4, stream, a);
    FIT_HIP(hipGetLastError());
    return RINR_OK;
}
}  // namespace

extern "C" int rinr_fit_steps(rinr_fit *f, const float *targets, int32_t n_steps, const rinr_fit_opts *o, void *stream) {
    if (!f || !o || (!targets && f->n_images > 0)) return RINR_E_NULL;
    if (n_steps < 0 || !(o->lr >= 0.0f) || o->t0 < 0) return RINR_E_ARG;
    if (((uintptr_t)targets & 3) != 0) return RINR_E_ALIGN;
    const float b1 = o->beta1 != 0.0f ? o->beta1 : 0.9f, b2 = o->beta2 != 0.0f ? o->beta2 : 0.999f;
    const float eps = o->eps != 0.0f ? o->eps : 1e-8f;
    if (!(b1 > 0.0f && b1 < 1.0f && b2 > 0.0f && b2 < 1.0f && eps > 0.0f) || !(o->loss_scale >= 0.0f)) return RINR_E_ARG;
    const float ls = o->loss_scale != 0.0f ? o->loss_scale : (float)(1.0 / (3.0 * (double)f->H * (double)f->W));
    if (f->n_images == 0) { f->t += n_steps; return RINR_OK; }
    for (int32_t i = 0; i < n_steps; ++i) {
        double lr = o->lr;
        if (o->T > 0) lr = 0.5 * lr * (1.0 + std::cos(3.14159265358979323846 * (double)(o->t0 + i) / (double)o->T));
        f->t += 1;
        const int rc = launch(f, targets, ls, (float)lr, f->t, b1, b2, eps, nullptr, (hipStream_t)stream);
        if (rc) return rc;
    }
    return RINR_OK;
}

extern "C" int rinr_fit_loss_grad(rinr_fit *f, const float *targets, float loss_scale, float *loss, float *grad, void *stream) {
    if (!f || !loss || (!targets && f->n_images > 0)) return RINR_E_NULL;
    if (((uintptr_t)targets & 3) != 0) return RINR_E_ALIGN;
    if (!(loss_scale >= 0.0f)) return RINR_E_ARG;
    if (f->n_images == 0) return RINR_OK;
    const size_t np = (size_t)f->n_images * (size_t)f->n_params;
    if (!f->scratch_grad) FIT_HIP(hipMalloc((void **)&f->scratch_grad, np * 4));
    const float ls = loss_scale != 0.0f ? loss_scale : (float)(1.0 / (3.0 * (double)f->H * (double)f->W));
    const int rc = launch(f, targets, ls, 0.0f, 1, 0.9f, 0.999f, 1e-8f, f->scratch_grad, (hipStream_t)stream);
    if (rc) return rc;
    FIT_HIP(hipStreamSynchronize((hipStream_t)stream));
    FIT_HIP(hipMemcpy(loss, f->loss, (size_t)f->n_images * 4, hipMemcpyDeviceToHost));
    if (grad) FIT_HIP(hipMemcpy(grad, f->scratch_grad, np * 4, hipMemcpyDeviceToHost));
    return RINR_OK;
}

extern "C" int rinr_fit_last_loss(const rinr_fit *f, float *loss, void *stream) {
    if (!f || (!loss && f->n_images > 0)) return RINR_E_NULL;
    FIT_HIP(hipStreamSynchronize((hipStream_t)stream));
    if (f->n_images) FIT_HIP(hipMemcpy(loss, f->loss, (size_t)f->n_images * 4, hipMemcpyDeviceToHost));
    return RINR_OK;
}

// ---- PSNR per image: a streaming reduction, bound by HBM (8 bytes read per element)
namespace {
__global__ __launch_bounds__(1024) void psnr_kernel(const float *a, const float *b, int64_t elems, float peak, float *out) {
    __shared__ double red[16];
    const float *pa = a + (size_t)blockIdx.x * (size_t)elems, *pb = b + (size_t)blockIdx.x * (size_t)elems;
    const int tid = threadIdx.x;
    double acc = 0.0;
    // groups of 4 floats where both rows are 16-byte aligned, singly otherwise
    const bool vec = ((((uintptr_t)pa) | ((uintptr_t)pb)) & 15) == 0;
    const int64_t nv = vec ? elems / 4 : 0;
    float part = 0.0f;
    int since = 0;
    for (int64_t q = tid; q < nv; q += 1024) {
        const float4 x = ((const float4 *)pa)[q], y = ((const float4 *)pb)[q];
        const float d0 = x.x - y.x, d1 = x.y - y.y, d2 = x.z - y.z, d3 = x.w - y.w;
        part += d0 * d0 + d1 * d1 + d2 * d2 + d3 * d3;
        if (++since == 64) { acc += (double)part; part = 0.0f; since = 0; }     // keep the fp32 partial sums short
    }
    for (int64_t k = nv * 4 + tid; k < elems; k += 1024) {
        const float d = pa[k] - pb[k];
        part += d * d;
    }
    acc += (double)part;
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if ((tid & 63) == 0) red[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) {
        double s = 0.0;
        for (int w = 0; w < 16; ++w) s += red[w];
        out[blockIdx.x] = s > 0.0 ? (float)(10.0 * log10((double)peak * (double)peak * (double)elems / s)) : INFINITY;
    }
}
}  // namespace

extern "C" int rinr_psnr_batch(const float *a, const float *b, int64_t n_images, int64_t elems, float peak, float *psnr,
                               void *stream) {
    if (n_images < 0 || elems < 0 || !(peak > 0.0f) || n_images > ((int64_t)1 << 31) - 1) return RINR_E_ARG;
    if (n_images == 0) return RINR_OK;
    if (!psnr || (elems > 0 && (!a || !b))) return RINR_E_NULL;
    if ((((uintptr_t)a) | ((uintptr_t)b) | ((uintptr_t)psnr)) & 3) return RINR_E_ALIGN;
    hipLaunchKernelGGL(psnr_kernel, dim3((uint32_t)n_images), dim3(1024), 0, (hipStream_t)stream, a, b, elems, peak, psnr);
    FIT_HIP(hipGetLastError());
    return RINR_OK;
}

// ---- Sec. IV as one call: fit, prune (fixed round, then the PSNR-driven one), re-fit, quantise, pack -------------
namespace {

struct EncodeModels {                       // host-side model descriptions of every image, in rinr_pack's terms
    std::vector<float> params;              // [n][n_params]
    std::vector<uint8_t> keep;              // [n][n_params] (biases: 1)
    std::vector<uint8_t> maskbits, codes8;
    std::vector<uint16_t> codes16;
    std::vector<rinr_layer_desc> layers;
    std::vector<rinr_model_desc> models;
};

// keep flags of every weight matrix of every image after pruning `ratio[i]` of image i's entries by magnitude
int prune_round(const rinr_fit *f, const std::vector<float> &params, const std::vector<double> &ratio, std::vector<uint8_t> &keep,
                bool have_keep) {
    const int L = f->arch.n_layers;
    std::vector<uint8_t> out;
    for (int64_t i = 0; i < f->n_images; ++i) {
        const float *p = params.data() + (size_t)i * (size_t)f->n_params;
        uint8_t *k = keep.data() + (size_t)i * (size_t)f->n_params;
        for (int l = 0; l < L; ++l) {
            const int64_t nw = (int64_t)f->arch.widths[l] * f->arch.widths[l + 1];
            out.resize((size_t)nw);
            const int rc = rinr_l1_mask(p + f->p_off[l], nw, ratio[(size_t)i], have_keep ? k + f->p_off[l] : nullptr, out.data());
            if (rc) return rc;
            std::memcpy(k + f->p_off[l], out.data(), (size_t)nw);
        }
    }
    return RINR_OK;
}

int psnr_now(rinr_fit *f, const float *targets, std::vector<double> &psnr, void *stream) {
    std::vector<float> loss((size_t)f->n_images);
    const int rc = rinr_fit_loss_grad(f, targets, 0.0f, loss.data(), nullptr, stream);      // mean squared error
    if (rc) return rc;
    psnr.resize(loss.size());
    for (size_t i = 0; i < loss.size(); ++i) psnr[i] = loss[i] > 0.0f ? -10.0 * std::log10((double)loss[i]) : INFINITY;
    return RINR_OK;
}

int check_encode_opts(const rinr_encode_opts *o) {
    if (!o) return RINR_E_NULL;
    if (o->schedule < 0 || o->schedule > 2 || o->fit_steps < 0 || o->refit_steps < 0) return RINR_E_ARG;
    if (!(o->first_ratio >= 0.0f && o->first_ratio <= 1.0f) || !(o->lr > 0.0f) || !(o->refit_lr > 0.0f)) return RINR_E_ARG;
    if (!(o->hidden_bits == 0 || (o->hidden_bits >= 2 && o->hidden_bits <= 8) || o->hidden_bits == 16)) return RINR_E_ARG;
    return RINR_OK;
}

// descriptions for rinr_pack: hidden layers as codes of `bits` bits, first and last layer fp32 (Sec. IV-B)
int describe(const rinr_fit *f, int bits, EncodeModels &e) {
    const int L = f->arch.n_layers;
    const int64_t n = f->n_images;
    size_t wtot = 0, mtot = 0;
    for (int l = 0; l < L; ++l) {
        const size_t nw = (size_t)f->arch.widths[l] * (size_t)f->arch.widths[l + 1];
        wtot += nw;
        mtot += (nw + 7) / 8;
    }
    e.maskbits.assign((size_t)n * mtot, 0);
    if (bits && bits <= 8) e.codes8.assign((size_t)n * wtot, 0);
    if (bits == 16) e.codes16.assign((size_t)n * wtot, 0);
    e.layers.resize((size_t)n * (size_t)L);
    e.models.resize((size_t)n);
    std::vector<uint16_t> codes;
    for (int64_t i = 0; i < n; ++i) {
        const float *p = e.params.data() + (size_t)i * (size_t)f->n_params;
        const uint8_t *k = e.keep.data() + (size_t)i * (size_t)f->n_params;
        size_t woff = 0, moff = 0;
        for (int l = 0; l < L; ++l) {
            const int din = f->arch.widths[l], dout = f->arch.widths[l + 1];
            const size_t nw = (size_t)din * (size_t)dout;
            uint8_t *mb = e.maskbits.data() + (size_t)i * mtot + moff;
            for (size_t q = 0; q < nw; ++q)
                if (k[f->p_off[l] + q]) mb[q >> 3] |= (uint8_t)(1u << (q & 7));
            rinr_layer_desc &d = e.layers[(size_t)i * (size_t)L + (size_t)l];
            d.in = din;
            d.out = dout;
            d.bits = 0;
            d.scale = 1.0f;
            d.zp = 0;
            d.weights = p + f->p_off[l];
            d.mask = mb;
            d.bias = p + f->p_off[l] + nw;
            if (bits && l > 0 && l < L - 1) {
                codes.resize(nw);
                const int rc = rinr_quantize_layer(p + f->p_off[l], k + f->p_off[l], (int64_t)nw, bits, &d.scale, &d.zp, codes.data());
                if (rc) return rc;
                d.bits = bits;
                if (bits <= 8) {
                    uint8_t *c8 = e.codes8.data() + (size_t)i * wtot + woff;
                    for (size_t q = 0; q < nw; ++q) c8[q] = (uint8_t)codes[q];
                    d.weights = c8;
                } else {
                    uint16_t *c16 = e.codes16.data() + (size_t)i * wtot + woff;
                    std::memcpy(c16, codes.data(), nw * 2);
                    d.weights = c16;
                }
            }
            woff += nw;
            moff += (nw + 7) / 8;
        }
        e.models[(size_t)i].n_layers = L;
        e.models[(size_t)i].layers = e.layers.data() + (size_t)i * (size_t)L;
    }
    return RINR_OK;
}

}  // namespace

extern "C" int rinr_encode_blob_bound(const rinr_fit *f, int32_t hidden_bits, size_t *bytes) {
    if (!f || !bytes) return RINR_E_NULL;
    if (!(hidden_bits == 0 || (hidden_bits >= 2 && hidden_bits <= 8) || hidden_bits == 16)) return RINR_E_ARG;
    try {
        EncodeModels e;
        e.params.assign((size_t)f->n_images * (size_t)f->n_params, 0.0f);
        e.keep.assign((size_t)f->n_images * (size_t)f->n_params, 1);     // masks present, everything kept: the largest record
        const int rc = describe(f, hidden_bits, e);
        if (rc) return rc;
        const rinr_store_opts so = {f->arch.w0, f->arch.coord_lo, f->arch.coord_hi};
        return rinr_pack_size(e.models.data(), f->n_images, &so, bytes);
    } catch (const std::bad_alloc &) {
        return RINR_E_SIZE;
    }
}

extern "C" int rinr_encode_images(rinr_fit *f, const float *targets, const rinr_encode_opts *o, float *psnr_out, void *blob,
                                  size_t capacity, size_t *blob_bytes, void *stream) {
    if (!f || !blob_bytes || (!targets && f->n_images > 0)) return RINR_E_NULL;
    int rc = check_encode_opts(o);
    if (rc) return rc;
    try {
        const int64_t n = f->n_images;
        EncodeModels e;
        e.params.resize((size_t)n * (size_t)f->n_params);
        e.keep.assign((size_t)n * (size_t)f->n_params, 1);
        std::vector<double> psnr, ratio((size_t)n);
        bool have_keep = false;
        // the fit itself (Eq. 1; cosine decay over the stage)
        rinr_fit_opts fo = {o->lr, 0, o->fit_steps, 0.0f, 0.0f, 0.0f, 0.0f};
        if ((rc = rinr_fit_set_keep(f, nullptr)) || (rc = rinr_fit_steps(f, targets, o->fit_steps, &fo, stream))) return rc;
        // pruning rounds (Sec. IV-A): a fixed ratio first (large images only), then the ratio chosen from each image's PSNR;
        // after each, the mask is applied and the model re-fitted from a fresh optimiser at the smaller rate
        for (int round = 0; round < 2; ++round) {
            if (round == 0 && !(o->first_ratio > 0.0f)) continue;
            if (round == 0) {
                std::fill(ratio.begin(), ratio.end(), (double)o->first_ratio);
            } else {
                if ((rc = psnr_now(f, targets, psnr, stream))) return rc;
                for (int64_t i = 0; i < n; ++i) ratio[(size_t)i] = rinr_prune_ratio(o->schedule, psnr[(size_t)i]);
            }
            if ((rc = rinr_fit_get_params(f, e.params.data(), stream))) return rc;
            if ((rc = prune_round(f, e.params, ratio, e.keep, have_keep))) return rc;
            have_keep = true;
            fo.lr = o->refit_lr;
            fo.T = o->refit_steps;
            if ((rc = rinr_fit_set_keep(f, e.keep.data())) || (rc = rinr_fit_reset_optimizer(f)) ||
                (rc = rinr_fit_steps(f, targets, o->refit_steps, &fo, stream)))
                return rc;
        }
        if ((rc = psnr_now(f, targets, psnr, stream))) return rc;
        if (psnr_out)
            for (int64_t i = 0; i < n; ++i) psnr_out[i] = (float)psnr[(size_t)i];
        if ((rc = rinr_fit_get_params(f, e.params.data(), stream))) return rc;
        // hidden layers to codes, first and last layer fp32 (Sec. IV-B); one blob for the decode side
        if ((rc = describe(f, o->hidden_bits, e))) return rc;
        const rinr_store_opts so = {f->arch.w0, f->arch.coord_lo, f->arch.coord_hi};
        if ((rc = rinr_pack_size(e.models.data(), n, &so, blob_bytes))) return rc;
        if (!blob || capacity < *blob_bytes) return RINR_E_SIZE;
        return rinr_pack(e.models.data(), n, &so, blob, *blob_bytes);
    } catch (const std::bad_alloc &) {
        return RINR_E_SIZE;
    }
}

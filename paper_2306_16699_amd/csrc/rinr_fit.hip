// Fitting one sine MLP per image on the GPU (Eq. 1): full-batch gradient of the squared error by
// forward and backward passes on the fp32 matrix cores, Adam update fused into the same kernel.
//
// One workgroup per image, one launch per step.  The image's weights live in LDS (bias folded in as an
// extra input column that multiplies a row of ones), pixels are taken in chunks of PC, and every
// contraction of a chunk is a set of 16x16 output tiles computed with v_mfma_f32_16x16x4_f32 from LDS
// operands:
//     forward        Z_l [d_out x PC]  = W_l [d_out x d_in+1] . H_l [d_in+1 x PC]        H_{l+1} = sin(w0 Z_l)
//     weight grads   dW_l [d_out x d_in+1] += D_l [d_out x PC] . H_l^T                   (contraction over pixels)
//     backward       D_{l-1} = (W_l^T . D_l) * w0 cos(w0 Z_{l-1})
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
constexpr int kWaves = 8, kThreads = kWaves * 64;
constexpr int kSlots = 3;                          // weight-gradient tiles a wavefront owns per layer: ceil(4 * 5 / 8)
constexpr uint32_t kLdsLimit = 160 * 1024;

thread_local int g_fit_last_hip = 0;
inline bool hip_fail(hipError_t e) {
    if (e == hipSuccess) return false;
    g_fit_last_hip = (int)e;
    return true;
}
#define FIT_HIP(call) do { if (hip_fail(call)) return RINR_E_HIP; } while (0)

// LDS layout of one workgroup, in floats.  Row stride of the pixel arrays is PC + 1 and of the weight
// arrays an odd number too, so that the strided operand reads of the three contractions spread over banks.
struct Layout {
    int32_t L, PC, PS;
    int32_t d[kMaxL + 1];
    int32_t KP[kMaxL];        // d_in + 1 rounded up to the MFMA depth 4
    int32_t MP[kMaxL];        // d_out rounded up to 16
    int32_t NT[kMaxL];        // 16-wide tiles over the d_in + 1 columns of the weight gradient
    int32_t IT[kMaxL];        // 16-row tiles over d_in (backward contraction output)
    int32_t w_off[kMaxL], w_ld[kMaxL];   // weights  [MP][w_ld]: column d_in is the bias
    int32_t h_off[kMaxL];     // layer input [KP][PS]: rows < d_in activations, row d_in ones, rest zero
    int32_t c_off[kMaxL];     // w0 cos(w0 z_{l-1}) [d_in][PS], l >= 1
    int32_t d_off[2];         // two buffers [max MP][PS] for the back-propagated error
    int32_t p_off[kMaxL];     // offset of W_l in the parameter vector
    int32_t total;            // floats
};

inline bool make_layout(const rinr_fit_arch &arch, int PC, Layout &ly) {
    std::memset(&ly, 0, sizeof ly);
    ly.L = arch.n_layers;
    ly.PC = PC;
    ly.PS = PC + 1;
    int off = 0, poff = 0, max_mp = 0;
    for (int l = 0; l <= ly.L; ++l) ly.d[l] = arch.widths[l];
    for (int l = 0; l < ly.L; ++l) {
        const int din = ly.d[l], dout = ly.d[l + 1];
        ly.KP[l] = (din + 1 + 3) / 4 * 4;
        ly.MP[l] = (dout + 15) / 16 * 16;
        ly.NT[l] = (din + 1 + 15) / 16;
        ly.IT[l] = (din + 15) / 16;
        ly.w_ld[l] = (ly.KP[l] > ly.IT[l] * 16 ? ly.KP[l] : ly.IT[l] * 16) + 1;
        ly.w_off[l] = off;
        off += ly.MP[l] * ly.w_ld[l];
        ly.p_off[l] = poff;
        poff += dout * din + dout;
        if (ly.MP[l] > max_mp) max_mp = ly.MP[l];
        if ((ly.MP[l] / 16) * ly.NT[l] > kSlots * kWaves) return false;
    }
    for (int l = 0; l < ly.L; ++l) { ly.h_off[l] = off; off += ly.KP[l] * ly.PS; }
    for (int l = 1; l < ly.L; ++l) { ly.c_off[l] = off; off += ly.d[l] * ly.PS; }
    for (int b = 0; b < 2; ++b) { ly.d_off[b] = off; off += max_mp * ly.PS; }
    ly.total = off;
    return true;
}

struct FitArgs {
    float *params, *m, *v;        // [n_images][n_params]
    const uint8_t *keep;          // [n_images][n_params] or null
    const float *target;          // [n_images][3][HW]
    float *loss;                  // [n_images]
    float *grad_out;              // null: Adam update; else the gradient is written here and nothing is updated
    int64_t n_params;
    uint32_t HW, W;
    float inv2W, inv2H, lo, span, w0, w0rev;
    float loss_scale;
    float lr, c1inv, c2inv, b1, b2, eps;
    Layout ly;
};

__device__ __forceinline__ f32x4 mfma4(float a, float b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }

template <int PC>
__global__ __launch_bounds__(kThreads) void fit_step_kernel(const FitArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    __shared__ float red[kWaves];
    const Layout &ly = a.ly;
    constexpr int PS = PC + 1, PT = PC / 16;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, m = lane & 15, kq = lane >> 4;
    const int L = ly.L;
    const size_t img = blockIdx.x;
    float *P = a.params + img * a.n_params;

    // ---- set up: zero everything, weights with the bias as column d_in, rows of ones
    for (int q = tid; q < ly.total; q += kThreads) lds[q] = 0.0f;
    __syncthreads();
    for (int l = 0; l < L; ++l) {
        const int din = ly.d[l], dout = ly.d[l + 1], ld = ly.w_ld[l];
        float *Wt = lds + ly.w_off[l];
        const float *src = P + ly.p_off[l];
        for (int e = tid; e < dout * din; e += kThreads) Wt[(e / din) * ld + e % din] = src[e];
        for (int o = tid; o < dout; o += kThreads) Wt[o * ld + din] = src[dout * din + o];
        float *Hl = lds + ly.h_off[l];
        for (int p = tid; p < PC; p += kThreads) Hl[din * PS + p] = 1.0f;
    }
    __syncthreads();

    f32x4 acc[kMaxL][kSlots];
#pragma unroll
    for (int l = 0; l < kMaxL; ++l)
#pragma unroll
        for (int s = 0; s < kSlots; ++s) acc[l][s] = (f32x4){0.0f, 0.0f, 0.0f, 0.0f};
    float loss_part = 0.0f;

    const uint32_t nchunks = (a.HW + PC - 1) / PC;
    for (uint32_t c = 0; c < nchunks; ++c) {
        // ---- pixel-centre coordinates of the chunk (a ragged last chunk repeats the last pixel; its error is zeroed)
        if (tid < PC) {
            uint32_t p = c * PC + tid;
            p = p < a.HW ? p : a.HW - 1;
            const uint32_t row = p / a.W, col = p - row * a.W;
            float *H0 = lds + ly.h_off[0];
            H0[tid] = fmaf(a.span, (float)(2 * col + 1) * a.inv2W, a.lo);
            H0[PS + tid] = fmaf(a.span, (float)(2 * row + 1) * a.inv2H, a.lo);
        }
        __syncthreads();
        // ---- forward
        for (int l = 0; l < L; ++l) {
            const int dout = ly.d[l + 1], ld = ly.w_ld[l], ksteps = ly.KP[l] >> 2;
            const float *Wt = lds + ly.w_off[l], *Hl = lds + ly.h_off[l];
            const int ntasks = (ly.MP[l] >> 4) * PT;
            for (int task = wave; task < ntasks; task += kWaves) {
                const int mt = task / PT, nt = task - mt * PT;
                const float *ap = Wt + (mt * 16 + m) * ld + kq, *bp = Hl + kq * PS + nt * 16 + m;
                f32x4 z = {0.0f, 0.0f, 0.0f, 0.0f};
                for (int ks = 0; ks < ksteps; ++ks) z = mfma4(ap[ks * 4], bp[ks * 4 * PS], z);
                const int col = nt * 16 + m;
                if (l < L - 1) {
                    float *Hn = lds + ly.h_off[l + 1], *Cn = lds + ly.c_off[l + 1];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int o = mt * 16 + 4 * kq + v;
                        if (o < dout) {
                            const float r = z[v] * a.w0rev;
                            Hn[o * PS + col] = __builtin_amdgcn_sinf(r);
                            Cn[o * PS + col] = a.w0 * __builtin_amdgcn_cosf(r);
                        }
                    }
                } else {
                    float *D0 = lds + ly.d_off[0];
                    const uint32_t pix = c * PC + col;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int o = mt * 16 + 4 * kq + v;
                        float e = 0.0f;
                        if (o < dout && pix < a.HW) e = z[v] - a.target[(img * 3 + o) * a.HW + pix];
                        loss_part = fmaf(e, e, loss_part);
                        D0[o * PS + col] = 2.0f * a.loss_scale * e;
                    }
                }
            }
            __syncthreads();
        }
        // ---- backward: weight-gradient tiles into this wavefront's accumulators, error to the layer below
        int cur = 0;
#pragma unroll
        for (int l = kMaxL - 1; l >= 0; --l) {
            if (l < L) {
                const int din = ly.d[l], ld = ly.w_ld[l], KP = ly.KP[l], NT = ly.NT[l];
                const float *Wt = lds + ly.w_off[l], *Hl = lds + ly.h_off[l], *Dc = lds + ly.d_off[cur];
                const int ntasks = (ly.MP[l] >> 4) * NT;
#pragma unroll
                for (int s = 0; s < kSlots; ++s) {
                    const int task = wave + s * kWaves;
                    if (task < ntasks) {
                        const int ot = task / NT, it = task - ot * NT;
                        const int i = it * 16 + m;
                        const bool live = i < KP;
                        const float *ap = Dc + (ot * 16 + m) * PS + kq, *bp = Hl + (live ? i : 0) * PS + kq;
                        f32x4 g = acc[l][s];
#pragma unroll
                        for (int ks = 0; ks < PC / 4; ++ks) g = mfma4(ap[ks * 4], live ? bp[ks * 4] : 0.0f, g);
                        acc[l][s] = g;
                    }
                }
                if (l > 0) {
                    float *Dn = lds + ly.d_off[cur ^ 1];
                    const float *Cl = lds + ly.c_off[l];
                    const int ksteps = ly.MP[l] >> 2;
                    const int nt2 = ly.IT[l] * PT;
                    for (int task = wave; task < nt2; task += kWaves) {
                        const int it = task / PT, nt = task - it * PT;
                        const float *ap = Wt + kq * ld + it * 16 + m, *bp = Dc + kq * PS + nt * 16 + m;
                        f32x4 g = {0.0f, 0.0f, 0.0f, 0.0f};
                        for (int ks = 0; ks < ksteps; ++ks) g = mfma4(ap[ks * 4 * ld], bp[ks * 4 * PS], g);
                        const int col = nt * 16 + m;
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int i = it * 16 + 4 * kq + v;
                            Dn[i * PS + col] = i < din ? g[v] * Cl[i * PS + col] : 0.0f;
                        }
                    }
                }
                __syncthreads();
                cur ^= 1;
            }
        }
    }

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
    for (int l = 0; l < kMaxL; ++l) {
        if (l < L) {
            const int din = ly.d[l], dout = ly.d[l + 1], NT = ly.NT[l];
            const int ntasks = (ly.MP[l] >> 4) * NT;
#pragma unroll
            for (int s = 0; s < kSlots; ++s) {
                const int task = wave + s * kWaves;
                if (task < ntasks) {
                    const int ot = task / NT, it = task - ot * NT;
                    const int i = it * 16 + m;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int o = ot * 16 + 4 * kq + v;
                        if (o < dout && i <= din) {
                            const int at = ly.p_off[l] + (i < din ? o * din + i : dout * din + o);
                            const bool kept = !K || K[at];
                            const float g = kept ? acc[l][s][v] : 0.0f;
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

}  // namespace

struct rinr_fit {
    rinr_fit_arch arch;
    int64_t n_images, n_params;
    int32_t H, W;
    int PC;
    Layout ly;
    float *params, *m, *v, *loss, *scratch_grad;
    uint8_t *keep;            // null until set
    bool has_keep;
    int64_t t;                // Adam steps taken
};

static fit_fn kernel_for(int PC) {
    switch (PC) {
        case 64: return fit_step_kernel<64>;
        case 32: return fit_step_kernel<32>;
        default: return fit_step_kernel<16>;
    }
}

extern "C" int rinr_fit_create(const rinr_fit_arch *arch, int64_t n_images, int32_t H, int32_t W, rinr_fit **out) {
    if (!arch || !out) return RINR_E_NULL;
    *out = nullptr;
    if (arch->n_layers < 2 || arch->n_layers > kMaxL || n_images < 0 || H <= 0 || W <= 0) return RINR_E_ARG;
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
    f->PC = 0;
    const int HW = H * W;
    for (int pc : {64, 32, 16}) {
        if (pc > 16 && pc / 2 >= HW) continue;          // no point in a chunk mostly beyond the image
        Layout ly;
        if (!make_layout(*arch, pc, ly)) { delete f; return RINR_E_UNSUPPORTED; }
        if ((size_t)ly.total * 4 + 256 <= kLdsLimit) { f->PC = pc; f->ly = ly; break; }
    }
    if (!f->PC) { delete f; return RINR_E_UNSUPPORTED; }
    f->n_params = 0;
    for (int l = 0; l < arch->n_layers; ++l) f->n_params += (int64_t)arch->widths[l + 1] * (arch->widths[l] + 1);
    const size_t np = (size_t)(n_images > 0 ? n_images : 1) * (size_t)f->n_params;
    f->params = f->m = f->v = f->loss = f->scratch_grad = nullptr;
    f->keep = nullptr;
    f->has_keep = false;
    f->t = 0;
    if (hip_fail(hipMalloc((void **)&f->params, np * 4)) || hip_fail(hipMalloc((void **)&f->m, np * 4)) ||
        hip_fail(hipMalloc((void **)&f->v, np * 4)) || hip_fail(hipMalloc((void **)&f->keep, np)) ||
        hip_fail(hipMalloc((void **)&f->loss, (size_t)(n_images > 0 ? n_images : 1) * 4)) ||
        hip_fail(hipMemset(f->params, 0, np * 4)) || hip_fail(hipMemset(f->m, 0, np * 4)) ||
        hip_fail(hipMemset(f->v, 0, np * 4)) || hip_fail(hipMemset(f->loss, 0, (size_t)(n_images > 0 ? n_images : 1) * 4)) ||
        hip_fail(hipFuncSetAttribute((const void *)kernel_for(f->PC), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)kLdsLimit - 256))) {
        rinr_fit_destroy(f);
        return RINR_E_HIP;
    }
    *out = f;
    return RINR_OK;
}

extern "C" int rinr_fit_destroy(rinr_fit *f) {
    if (!f) return RINR_OK;
    (void)hipFree(f->params);
    (void)hipFree(f->m);
    (void)hipFree(f->v);
    (void)hipFree(f->keep);
    (void)hipFree(f->loss);
    (void)hipFree(f->scratch_grad);
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
    a.grad_out = grad_out;
    a.n_params = f->n_params;
    a.HW = (uint32_t)(f->H * f->W);
    a.W = (uint32_t)f->W;
    a.inv2W = 1.0f / (2.0f * (float)f->W);
    a.inv2H = 1.0f / (2.0f * (float)f->H);
    a.lo = f->arch.coord_lo;
    a.span = f->arch.coord_hi - f->arch.coord_lo;
    a.w0 = f->arch.w0;
    a.w0rev = (float)((double)f->arch.w0 / (2.0 * 3.14159265358979323846));
    a.loss_scale = loss_scale;
    a.lr = lr;
    a.c1inv = (float)(1.0 / (1.0 - std::pow((double)b1, (double)t)));
    a.c2inv = (float)(1.0 / (1.0 - std::pow((double)b2, (double)t)));
    a.b1 = b1; a.b2 = b2; a.eps = eps;
    a.ly = f->ly;
    hipLaunchKernelGGL(kernel_for(f->PC), dim3((uint32_t)f->n_images), dim3(kThreads), (size_t)f->ly.total * 4, stream, a);
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

// Split-precision decode kernel: the layers' contractions run on the fp16 matrix cores
// (v_mfma_f32_16x16x32_f16 / 16x16x16_f16, fp32 accumulate) with every fp32 operand carried
// as an exact-sum pair of halfs, hi = fp16(x), lo = fp16(x - hi), so a product keeps ~22
// significant bits:  W*h ~= Wh*hh + Wh*hl + Wl*hh   (the dropped Wl*hl is 2^-22 relative).
// A hidden layer stored as 2..8-bit codes (Sec. IV-B) needs no low part at all: its integers
// q - zp are exact in fp16, so W*h = scale * (Q*hh + Q*hl) and the scale moves into the sine
// epilogue.  Unlike fp32 MFMA, the fp16 matrix pipe runs concurrently with the vector ALU on
// this chip, so the sine + split work of one wavefront hides behind the matrix work of
// another; the method and its results (Sec. III-B decode) are unchanged.
//
// Same structure as the fp32 kernel: workgroup = (slot, range of 64-pixel tiles), model
// expanded once into LDS, activations register-resident across layers.  Tile = 16 rows x 16
// pixels, lane = (n = lane % 16, g = lane / 16); accumulator register v of a lane holds row
// 4g + v of its tile.  A 32-deep k-step takes from lane group g the 8 activations that group
// holds of two consecutive row tiles (2j, 2j+1), so again nothing crosses lanes.
#pragma once
#include "rinr_kernels.hip.h"

namespace rinr {

typedef _Float16 h2v __attribute__((ext_vector_type(2)));
typedef _Float16 h4v __attribute__((ext_vector_type(4)));
typedef _Float16 h8v __attribute__((ext_vector_type(8)));
typedef float f2v __attribute__((ext_vector_type(2)));

// A hidden layer takes the two-term integer form when its codes are exact in fp16 and the
// scale is a usable multiplier; otherwise its dequantised fp32 weights are split hi/lo.
__host__ __device__ inline bool xdl_int_layer(uint32_t bits, float scale_pre) {
    const float a = scale_pre < 0 ? -scale_pre : scale_pre;
    return bits >= 2 && bits <= 8 && a >= 1e-12f && a <= 1e12f;
}

struct XLayer {            // one entry per linear layer, built in LDS by the workgroup
    uint32_t off_hi;       // byte offset of the fp16 operand block
    uint32_t off_lo;       // byte offset of the low-part block, 0 = none (integer layer)
    float scale;           // multiplies the accumulator before the sine (1 unless integer layer)
    uint32_t off_bias;     // byte offset of the fp32 bias tile(s)
};

template <int MT> struct XLayout {
    static constexpr int WP = 16 * MT;
    static constexpr int KJ = MT / 2;              // 32-deep k-steps of a hidden layer
    static constexpr int K16 = MT % 2;             // plus one 16-deep step for an odd last tile
    static constexpr int TABLE = 16 * 16;          // bytes: one XLayer per linear layer, 16 at most
    static constexpr int HID = 256 * MT * MT * 2;  // bytes of one hidden operand block
    static constexpr int FIRST = MT * 64 * 16;     // bytes: [mt][lane][8 halfs], hi and lo in one k-step
    static constexpr int OUT = (KJ * 64 * 16 + K16 * 64 * 8);   // bytes: one 16-row tile
    // half index of hidden weight (o, i) inside its block
    static __device__ __forceinline__ int idx_hidden(int o, int i) {
        const int mt = o >> 4, m = o & 15, t = i >> 4, g = (i >> 2) & 3, v = i & 3;
        if (t < 2 * KJ) return (((t >> 1) * MT + mt) * 64 + g * 16 + m) * 8 + (t & 1) * 4 + v;
        return KJ * MT * 512 + (mt * 64 + g * 16 + m) * 4 + v;
    }
    static __device__ __forceinline__ int idx_first(int o, int e) { return ((o >> 4) * 64 + (o & 15)) * 8 + e; }
    // output channel c sits in row 4c of the single output tile, i.e. lane group c, register 0
    static __device__ __forceinline__ int idx_out(int c, int i) {
        const int t = i >> 4, g = (i >> 2) & 3, v = i & 3, lane = g * 16 + 4 * c;
        if (t < 2 * KJ) return ((t >> 1) * 64 + lane) * 8 + (t & 1) * 4 + v;
        return KJ * 512 + lane * 4 + v;
    }
    static __device__ __forceinline__ int idx_bias(int o) { return ((o >> 4) * 4 + ((o >> 2) & 3)) * 4 + (o & 3); }
};

// Bytes of LDS the expanded model needs (without the staging copy of the record).
// n_int = hidden layers in integer form, n_raw = hidden layers split hi/lo.
__host__ __device__ inline uint32_t xdl_model_bytes(int mt, int n_layers, int n_int, int n_raw) {
    const uint32_t wp = 16u * mt, hid = 512u * mt * mt;
    const uint32_t out = (uint32_t)((mt / 2) * 1024 + (mt % 2) * 512);
    return 16u * 16u + ((uint32_t)(n_layers - 1) * wp + 16u) * 4u + (uint32_t)mt * 1024u +
           hid * (uint32_t)(n_int + 2 * n_raw) + 2u * out;
}

template <int MT>
__device__ __forceinline__ void xdl_expand_model(char *lds, const uint32_t *rec, int L, float pre, int tid, int nthreads,
                                                 uint32_t total_bytes) {
    typedef XLayout<MT> LY;
    XLayer *tab = (XLayer *)lds;
    for (uint32_t q = tid; q < (total_bytes >> 2); q += nthreads) ((uint32_t *)lds)[q] = 0u;
    __syncthreads();
    if (tid == 0) {
        uint32_t bias = LY::TABLE;
        uint32_t cur = LY::TABLE + ((uint32_t)(L - 1) * LY::WP + 16u) * 4u;
        for (int l = 0; l < L; ++l) {
            const LayerRec r = *(const LayerRec *)(rec + l * (sizeof(LayerRec) / 4));
            XLayer e;
            e.off_bias = bias;
            bias += (l < L - 1 ? LY::WP : 16) * 4;
            e.scale = 1.0f;
            e.off_hi = cur;
            e.off_lo = 0;
            if (l == 0) cur += LY::FIRST;
            else if (l == L - 1) { e.off_lo = cur + LY::OUT; cur += 2 * LY::OUT; }
            else if (xdl_int_layer(r.bits, r.scale * pre)) { e.scale = r.scale * pre; cur += LY::HID; }
            else { e.off_lo = cur + LY::HID; cur += 2 * LY::HID; }
            tab[l] = e;
        }
    }
    __syncthreads();
    const int wave = tid >> 6, lane = tid & 63, nwaves = nthreads >> 6;
    for (int l = wave; l < L; l += nwaves) {
        const LayerRec r = *(const LayerRec *)(rec + l * (sizeof(LayerRec) / 4));
        const XLayer e = tab[l];
        _Float16 *hi = (_Float16 *)(lds + e.off_hi), *lo = (_Float16 *)(lds + e.off_lo);
        float *bt = (float *)(lds + e.off_bias);
        if (l == L - 1) {
            expand_layer(rec, r, lane,
                         [=](int o, int i, float v, int) {
                             const _Float16 h = (_Float16)v;
                             hi[LY::idx_out(o, i)] = h;
                             lo[LY::idx_out(o, i)] = (_Float16)(v - (float)h);
                         },
                         [=](int o, float v) { bt[o * 4] = v; });
        } else if (l == 0) {
            expand_layer(rec, r, lane,
                         [=](int o, int i, float v, int) {
                             const float w = v * pre;
                             const _Float16 h = (_Float16)w, lw = (_Float16)(w - (float)h);
                             hi[LY::idx_first(o, i)] = h;          // pairs with the coordinate's high half
                             hi[LY::idx_first(o, 2 + i)] = h;      // ... with its low half
                             hi[LY::idx_first(o, 4 + i)] = lw;     // low weight part x high coordinate half
                         },
                         [=](int o, float v) { bt[LY::idx_bias(o)] = v * pre; });
        } else if (e.off_lo == 0) {
            const float inv = 1.0f / e.scale;
            expand_layer(rec, r, lane, [=](int o, int i, float, int q) { hi[LY::idx_hidden(o, i)] = (_Float16)(float)q; },
                         [=](int o, float v) { bt[LY::idx_bias(o)] = v * pre * inv; });
        } else {
            expand_layer(rec, r, lane,
                         [=](int o, int i, float v, int) {
                             const float w = v * pre;
                             const _Float16 h = (_Float16)w;
                             hi[LY::idx_hidden(o, i)] = h;
                             lo[LY::idx_hidden(o, i)] = (_Float16)(w - (float)h);
                         },
                         [=](int o, float v) { bt[LY::idx_bias(o)] = v * pre; });
        }
    }
    __syncthreads();
}

__device__ __forceinline__ f32x4 mfma32h(h8v a, h8v b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
__device__ __forceinline__ f32x4 mfma16h(h4v a, h4v b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x16f16(a, b, c, 0, 0, 0); }

// sine of the four accumulator values of one tile, then the exact hi/lo split of the results.
// neg1 is -1.0f passed as data so that h - float(hi) stays a single mixed-precision fma.
__device__ __forceinline__ void sine_split(const f32x4 d, float scale, float neg1, h4v &hi, h4v &lo) {
    const f2v p0 = {sin_rev(d[0] * scale), sin_rev(d[1] * scale)};
    const f2v p1 = {sin_rev(d[2] * scale), sin_rev(d[3] * scale)};
    const h2v a0 = __builtin_convertvector(p0, h2v), a1 = __builtin_convertvector(p1, h2v);
    const f2v r0 = {__builtin_fmaf((float)a0[0], neg1, p0[0]), __builtin_fmaf((float)a0[1], neg1, p0[1])};
    const f2v r1 = {__builtin_fmaf((float)a1[0], neg1, p1[0]), __builtin_fmaf((float)a1[1], neg1, p1[1])};
    const h2v b0 = __builtin_convertvector(r0, h2v), b1 = __builtin_convertvector(r1, h2v);
    hi = (h4v){a0[0], a0[1], a1[0], a1[1]};
    lo = (h4v){b0[0], b0[1], b1[0], b1[1]};
}

// ---- per-wavefront state of one half (two 16-pixel tiles = 32 pixels) of a 64-pixel tile ----------
template <int MT> struct XHalf {
    static constexpr int KJ = MT / 2, KJA = KJ ? KJ : 1;
    h8v Hh[2][KJA], Hl[2][KJA];     // activations as fp16 hi / lo, operand of the 32-deep k-steps
    h4v Hh4[2], Hl4[2];             // ... of the 16-deep step (odd MT)
    f32x4 D[2][MT];                 // accumulators
};

// sine + split of all accumulators of a half: 32*MT VALU instructions (x4 with the scale multiply)
template <int MT>
__device__ __forceinline__ void xdl_epilogue(XHalf<MT> &H, float scale, float neg1) {
    constexpr int KJ = MT / 2;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            h4v hi, lo;
            sine_split(H.D[nt][t], scale, neg1, hi, lo);
            if (t < 2 * KJ) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    H.Hh[nt][t >> 1][(t & 1) * 4 + v] = hi[v];
                    H.Hl[nt][t >> 1][(t & 1) * 4 + v] = lo[v];
                }
            } else { H.Hh4[nt] = hi; H.Hl4[nt] = lo; }
        }
}

// MFMAs of one hidden layer for a half.  LO: the layer has a low weight part (three terms).
template <int MT, bool LO>
__device__ __forceinline__ void xdl_hidden(XHalf<MT> &H, const char *lds, const XLayer el, int lane, int g) {
    constexpr int KJ = MT / 2, K16 = MT % 2;
    const h8v *ah = (const h8v *)(lds + el.off_hi) + lane;
    const h8v *al = (const h8v *)(lds + el.off_lo) + lane;
    const h4v *ah4 = (const h4v *)(lds + el.off_hi + KJ * MT * 1024) + lane;
    const h4v *al4 = (const h4v *)(lds + el.off_lo + KJ * MT * 1024) + lane;
    const f32x4 *bt = (const f32x4 *)(lds + el.off_bias) + g;
#pragma unroll
    for (int j = 0; j < KJ; ++j)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const h8v av = ah[(j * MT + mt) * 64];
            h8v aw;
            if (LO) aw = al[(j * MT + mt) * 64];
            f32x4 c;
            if (j == 0) c = bt[mt * 4];
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) H.D[nt][mt] = mfma32h(av, H.Hh[nt][j], j == 0 ? c : H.D[nt][mt]);
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) H.D[nt][mt] = mfma32h(av, H.Hl[nt][j], H.D[nt][mt]);
            if (LO) {
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) H.D[nt][mt] = mfma32h(aw, H.Hh[nt][j], H.D[nt][mt]);
            }
        }
    if (K16) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const h4v av = ah4[mt * 64];
            h4v aw;
            if (LO) aw = al4[mt * 64];
            f32x4 c;
            if (KJ == 0) c = bt[mt * 4];
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) H.D[nt][mt] = mfma16h(av, H.Hh4[nt], KJ == 0 ? c : H.D[nt][mt]);
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) H.D[nt][mt] = mfma16h(av, H.Hl4[nt], H.D[nt][mt]);
            if (LO) {
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) H.D[nt][mt] = mfma16h(aw, H.Hh4[nt], H.D[nt][mt]);
            }
        }
    }
}

// Tell the scheduler to issue the block just written as: a first batch of LDS reads, then NM x
// (1 MFMA, its share of the NV vector-ALU ops), feeding the remaining NDS LDS reads in between,
// so that the matrix pipe works on one half while the ALU does the other half's sine and split.
template <int NM, int NV, int NDS, int I> struct XInterleave {
    static __device__ __forceinline__ void run() {
        constexpr int FIRST = NDS < 6 ? NDS : 6;
        constexpr int PER = (NV * (I + 1)) / NM - (NV * I) / NM;
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if constexpr (PER > 0) __builtin_amdgcn_sched_group_barrier(0x002, PER, 0);
        if constexpr (FIRST + I < NDS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        XInterleave<NM, NV, NDS, I + 1>::run();
    }
};
template <int NM, int NV, int NDS> struct XInterleave<NM, NV, NDS, NM> {
    static __device__ __forceinline__ void run() {}
};
template <int NM, int NV, int NDS> __device__ __forceinline__ void xdl_interleave() {
    constexpr int FIRST = NDS < 6 ? NDS : 6;
    __builtin_amdgcn_sched_group_barrier(0x100, FIRST, 0);
    XInterleave<NM, NV, NDS, 0>::run();
}

template <int MT>
__device__ __forceinline__ void xdl_body(const DecodeArgs &a, const Work &w, float *lds_f) {
    typedef XLayout<MT> LY;
    constexpr int KJ = LY::KJ, K16 = LY::K16;
    constexpr int NM_INT = 2 * MT * (KJ + K16) * 2, NM_RAW = 2 * MT * (KJ + K16) * 3;   // MFMAs per half-layer
    constexpr int NV = 32 * MT;                 // ALU ops of a half's epilogue: 8*MT activations x (mul, sin, cvt/2, fma, cvt/2)
    constexpr int ND_INT = (KJ + K16) * MT + MT, ND_RAW = 2 * (KJ + K16) * MT + MT;     // LDS reads per half-layer
    char *lds = (char *)lds_f;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const uint32_t slot = w.slot, tile0 = w.tile0, tile1 = w.tile1;
    const size_t plane0 = w.plane0;
    const IndexEntry e = w.e;
    const int L = e.n_layers;

    uint32_t *stage = (uint32_t *)(lds_f + a.stage_off[MT]);
    {
        const uint4 *src = (const uint4 *)(a.blob + e.off);
        uint4 *dst = (uint4 *)stage;
        for (uint32_t q = tid; q < (e.nbytes >> 4); q += nthreads) dst[q] = src[q];
    }
    // Tiles are handed out through a counter in LDS (it reuses the first word of the staging area,
    // which is dead once the model is expanded): the SIMD arbiter favours its older wavefront, so
    // with a fixed split the favoured waves would finish early and leave the others running alone.
    xdl_expand_model<MT>(lds, stage, L, a.pre, tid, nthreads, a.stage_off[MT] << 2);
    uint32_t *next_tile = stage;
    if (tid == 0) *next_tile = tile0 + (nthreads >> 6);
    __syncthreads();

    const int lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, n = lane & 15;
    const XLayer *tab = (const XLayer *)lds;
    const float neg1 = a.neg1;
    const XLayer e0 = tab[0], eo = tab[L - 1];
    float af[6] = {1.0f, 0.0f, 0.0f, 0.0f, 1.0f, 0.0f};      // augmentation: this slot's map of the sampling grid
    if (a.affine)
        for (int q = 0; q < 6; ++q) af[q] = a.affine[(size_t)slot * 6 + q];
    const float nsc = g == 0 ? a.ns[0] : (g == 1 ? a.ns[1] : a.ns[2]);     // lane group g stores channel g
    const float nsh = g == 0 ? a.nb[0] : (g == 1 ? a.nb[1] : a.nb[2]);

    for (uint32_t tile = tile0 + wave; tile < tile1;) {
        XHalf<MT> X, Y;
        // ---- first layer: coordinates as hi/lo halfs in lane group 0; k slots (xh, yh, xl, yl, xh, yh, 0, 0)
        {
            const h8v *a0 = (const h8v *)(lds + e0.off_hi) + lane;
            const f32x4 *bt = (const f32x4 *)(lds + e0.off_bias) + g;
            h8v b0[4];
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                uint32_t p = (tile << 6) + nt * 16 + n;
                p = min(p, a.HW - 1);
                const uint32_t row = a.wmagic ? (__umulhi(p, a.wmagic) >> a.wshift) : p, col = p - row * a.W;
                const float x0 = fmaf(a.span, (float)(2 * col + 1) * a.inv2W, a.lo);
                const float y0 = fmaf(a.span, (float)(2 * row + 1) * a.inv2H, a.lo);
                const float x = fmaf(af[0], x0, fmaf(af[1], y0, af[2])), y = fmaf(af[3], x0, fmaf(af[4], y0, af[5]));
                const _Float16 xh = (_Float16)x, yh = (_Float16)y;
                const _Float16 xl = (_Float16)(x - (float)xh), yl = (_Float16)(y - (float)yh);
                const _Float16 z = (_Float16)0.0f;
                b0[nt] = g == 0 ? (h8v){xh, yh, xl, yl, xh, yh, z, z} : (h8v){z, z, z, z, z, z, z, z};
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const h8v av = a0[mt * 64];
                const f32x4 c = bt[mt * 4];
                X.D[0][mt] = mfma32h(av, b0[0], c);
                X.D[1][mt] = mfma32h(av, b0[1], c);
                Y.D[0][mt] = mfma32h(av, b0[2], c);
                Y.D[1][mt] = mfma32h(av, b0[3], c);
            }
        }
        xdl_epilogue<MT>(X, 1.0f, neg1);
        // ---- hidden layers, software-pipelined over the two halves:
        //      matrix work of X(l) with the sine/split of Y(l-1), then matrix work of Y(l) with the sine/split of X(l)
        float scale_prev = 1.0f;
        for (int l = 1; l < L - 1; ++l) {
            const XLayer el = tab[l];
            if (el.off_lo == 0) {
                xdl_hidden<MT, false>(X, lds, el, lane, g);
                xdl_epilogue<MT>(Y, scale_prev, neg1);
                xdl_interleave<NM_INT, NV, ND_INT>();
                __builtin_amdgcn_sched_barrier(0);
                xdl_hidden<MT, false>(Y, lds, el, lane, g);
                xdl_epilogue<MT>(X, el.scale, neg1);
                xdl_interleave<NM_INT, NV, ND_INT>();
            } else {
                xdl_hidden<MT, true>(X, lds, el, lane, g);
                xdl_epilogue<MT>(Y, scale_prev, neg1);
                xdl_interleave<NM_RAW, NV, ND_RAW>();
                __builtin_amdgcn_sched_barrier(0);
                xdl_hidden<MT, true>(Y, lds, el, lane, g);
                xdl_epilogue<MT>(X, el.scale, neg1);
                xdl_interleave<NM_RAW, NV, ND_RAW>();
            }
            scale_prev = el.scale;
        }
        xdl_epilogue<MT>(Y, scale_prev, neg1);
        // ---- output layer width -> 3: one 16-row tile, channel c in row 4c = lane group c, register 0
        {
            const h8v *ah = (const h8v *)(lds + eo.off_hi) + lane;
            const h8v *al = (const h8v *)(lds + eo.off_lo) + lane;
            const h4v *ah4 = (const h4v *)(lds + eo.off_hi + KJ * 1024) + lane;
            const h4v *al4 = (const h4v *)(lds + eo.off_lo + KJ * 1024) + lane;
            const f32x4 c = ((const f32x4 *)(lds + eo.off_bias))[g];
            f32x4 O[4] = {c, c, c, c};
#pragma unroll
            for (int j = 0; j < KJ; ++j) {
                const h8v av = ah[j * 64], aw = al[j * 64];
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) {
                    const h8v bh = nt < 2 ? X.Hh[nt][j] : Y.Hh[nt - 2][j];
                    const h8v bl = nt < 2 ? X.Hl[nt][j] : Y.Hl[nt - 2][j];
                    O[nt] = mfma32h(av, bh, O[nt]);
                    O[nt] = mfma32h(av, bl, O[nt]);
                    O[nt] = mfma32h(aw, bh, O[nt]);
                }
            }
            if (K16) {
                const h4v av = ah4[0], aw = al4[0];
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) {
                    const h4v bh = nt < 2 ? X.Hh4[nt] : Y.Hh4[nt - 2];
                    const h4v bl = nt < 2 ? X.Hl4[nt] : Y.Hl4[nt - 2];
                    O[nt] = mfma16h(av, bh, O[nt]);
                    O[nt] = mfma16h(av, bl, O[nt]);
                    O[nt] = mfma16h(aw, bh, O[nt]);
                }
            }
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                float r = O[nt][0];
                if (!a.no_clamp) r = fminf(fmaxf(r, 0.0f), 1.0f);
                if (a.normalize) r = fmaf(r, nsc, nsh);
                const uint32_t p = (tile << 6) + nt * 16 + n;
                if (g < 3 && p < a.HW) {
                    const size_t at = plane0 + (size_t)g * a.HW + p;
                    if (a.out_f32) a.out_f32[at] = r;
                    if (a.out_u8) a.out_u8[at] = (uint8_t)rintf(255.0f * r);
                }
            }
        }
        uint32_t nt_ = 0;
        if (lane == 0) nt_ = atomicAdd(next_tile, 1u);
        tile = __builtin_amdgcn_readfirstlane(nt_);
    }
}

template <int MT, int NTHREADS>
__global__ __launch_bounds__(NTHREADS) void decode_xdl_kernel(const DecodeArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds_f[];
    Work w;
    if (!decode_prologue(a, w)) return;
    xdl_body<MT>(a, w, lds_f);
}

// every width class in one launch (a.cls == 0)
template <int NTHREADS>
__global__ __launch_bounds__(NTHREADS) void decode_xdl_any_kernel(const DecodeArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds_f[];
    Work w;
    if (!decode_prologue(a, w)) return;
    switch (w.cls) {
        case 1: xdl_body<1>(a, w, lds_f); break;
        case 2: xdl_body<2>(a, w, lds_f); break;
        case 3: xdl_body<3>(a, w, lds_f); break;
        default: xdl_body<4>(a, w, lds_f); break;
    }
}

}  // namespace rinr

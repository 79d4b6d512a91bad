// Split-precision decode kernel: the layers' contractions run on the fp16 matrix cores
// (v_mfma_f32_32x32x16_f16 / 16x16x32_f16 / 16x16x16_f16, fp32 accumulate) with every fp32
// operand carried as an exact-sum pair of halfs, hi = fp16(x), lo = fp16(x - hi), so a product
// keeps ~22 significant bits:  W*h ~= Wh*hh + Wh*hl + Wl*hh   (the dropped Wl*hl is 2^-22 relative).
// A hidden layer stored as 2..8-bit codes (Sec. IV-B) needs no low part at all: its integers
// q - zp are exact in fp16, so W*h = scale * (Q*hh + Q*hl) and the scale moves into the sine
// epilogue.  Unlike fp32 MFMA, the fp16 matrix pipe runs concurrently with the vector ALU on
// this chip, so the sine + split work hides the matrix work; the method and its results
// (Sec. III-B decode) are unchanged.
//
// Same structure as the fp32 kernel: workgroup = (slot, range of 64-pixel tiles), model
// expanded once into LDS, activations register-resident across layers.  Tile = TM rows x TM
// pixels (TM = 32 at padded width 32, and at 64 in the all-class kernel; else 16), lane = (n = lane % TM, g = lane / TM).
// A lane's accumulator registers come in quads of four consecutive rows; quad Q (counted over
// all row tiles of the layer) holds rows
//     TM = 16:  16 Q + 4 g + b            TM = 32:  32 (Q / 4) + 8 (Q % 4) + 4 g + b,   b = 0..3.
// One MFMA k-step takes 8 halfs per lane = quads 2j and 2j+1 of every lane group, i.e. exactly the
// activations the lanes already hold, so again nothing crosses lanes between layers.  An odd last quad (padded widths
// 16 and 48) takes a half-depth step, v_mfma_f32_16x16x16_f16, on the same accumulators.
// Two MFMAs of different depth must not follow each other closely on one accumulator: with a 16x16x16 step issued
// right behind a 16x16x32 step that writes its C operand (one vector instruction between them, no wait states
// added by the compiler) the second read the accumulator before the first had written it, and the first step's
// contribution was lost.  So all full-depth steps of a layer are issued first, then 20 idle cycles of this wavefront
// (one more than the longest wait the instruction set documents between dependent matrix instructions of different
// kinds; the SIMD's other wavefronts issue meanwhile), then all half-depth steps,
// the order being forced through the accumulators themselves (xdl_touch).  tests/test_gpu_parity.py pins it with a
// model whose output must contain a term that only the full-depth step supplies.
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

// MFMA tile rows the split-precision kernel uses for a width class (padded width = 16 * cls).
// The 32-row instruction does twice the work per issue slot; at padded width 32 that pays, at 64 the
// 16-register accumulator tuples cost more in register pressure than the issue slots give back.
__host__ __device__ constexpr int xdl_tile_rows(int cls) { return cls == 2 ? 32 : 16; }

// What kinds of hidden layer the models served by a launch have (the host knows it from the store): a kernel
// for one kind runs a layer loop without a branch on the kind.  With the branch inside, the compiler hoists and
// sinks the two halves' common epilogue code out of the branches, away from the MFMAs it is meant to run under.
enum { kHiddenAllInt = 0, kHiddenAllRaw = 1, kHiddenMixed = 2 };
// Added to the kind: activations travel as one fp16 value instead of a hi+lo pair (RINR_FLAG_FP16_ACT): one MFMA
// term less per layer and a two-instruction epilogue, at 2^-12 relative rounding per activation.
enum { kAct16 = 4 };
// Added to kAct16 (the kind is then irrelevant): the hidden layers' weights are single fp16 values too, fp16(w * w0 / 2pi)
// whether the layer is stored as codes or as fp32, so every hidden layer is one MFMA term and its epilogue is
// sine + conversion (RINR_FLAG_FP16_ALL): fp16 operands with fp32 accumulation throughout the hidden layers.
enum { kWeight16 = 8 };

struct XLayer {            // one entry per linear layer, built in LDS by the workgroup
    uint32_t off_hi;       // byte offset of the fp16 operand block
    uint32_t off_lo;       // byte offset of the low-part block, 0 = none (integer layer)
    float scale;           // multiplies the accumulator before the sine (1 unless integer layer)
    uint32_t off_bias;     // byte offset of the fp32 bias tile(s)
};

template <int TM, int WP> struct XLayout {
    static constexpr int G = 64 / TM;              // lane groups
    static constexpr int RV = TM * TM / 64;        // accumulator registers per tile
    static constexpr int MT = WP / TM;             // row tiles per layer
    static constexpr int NQ = WP / (4 * G);        // quads per lane over the layer's rows
    static constexpr int KJ = NQ / 2;              // full k-steps (8 halfs per lane) of a hidden layer
    static constexpr int K16 = NQ % 2;             // plus one half-depth step for an odd last quad (TM = 16 only)
    static constexpr int TABLE = 16 * 16;          // bytes: one XLayer per linear layer, 16 at most
    static constexpr int HID = WP * WP * 2;        // bytes of one hidden operand block
    static constexpr int FIRST = G * MT * 64 * 16; // bytes: [pixel tile q][mt][lane][8 halfs], hi and lo in one k-step; variant q has the
                                                   // weights in lane group q's k-slots only, so that group q's coordinates alone count
    static constexpr int OUT = KJ * 64 * 16 + K16 * 64 * 8;   // bytes: one TM-row tile
    static constexpr int OUTB = TM * 4;            // bytes of the output layer's bias tile
    static_assert(WP % TM == 0 && (TM == 16 || K16 == 0), "layout");

    // row r of the layer -> (quad, lane group, position in the quad)
    static __device__ __forceinline__ void locate(int r, int &q, int &g, int &b) {
        b = r & 3;
        if (TM == 16) { q = r >> 4; g = (r >> 2) & 3; }
        else { q = ((r >> 5) << 2) | ((r >> 3) & 3); g = (r >> 2) & 1; }
    }
    // half index of hidden weight (o, i) inside its block: [k-step][row tile][lane][8]
    static __device__ __forceinline__ int idx_hidden(int o, int i) {
        const int mt = o / TM, m = o % TM;
        int q, g, b;
        locate(i, q, g, b);
        if (q < 2 * KJ) return (((q >> 1) * MT + mt) * 64 + g * TM + m) * 8 + (q & 1) * 4 + b;
        return KJ * MT * 512 + (mt * 64 + g * TM + m) * 4 + b;
    }
    static __device__ __forceinline__ int idx_first(int q, int o, int e) { return (((q * MT + o / TM) * 64) + q * TM + (o % TM)) * 8 + e; }
    // output channel c sits in row 4c of the single output tile
    static __device__ __forceinline__ int idx_out(int c, int i) {
        int q, g, b;
        locate(i, q, g, b);
        const int lane = g * TM + 4 * c;
        if (q < 2 * KJ) return ((q >> 1) * 64 + lane) * 8 + (q & 1) * 4 + b;
        return KJ * 512 + lane * 4 + b;
    }
    // bias tiles are accumulator shaped: [row tile][lane group][register]
    static __device__ __forceinline__ int idx_bias(int o) {
        int q, g, b;
        locate(o % TM, q, g, b);
        return ((o / TM) * G + g) * RV + q * 4 + b;
    }
};

// Bytes of LDS the expanded model of width class `cls` needs (without the staging copy of the
// record).  n_int = hidden layers in integer form, n_raw = hidden layers split hi/lo.
__host__ __device__ inline uint32_t xdl_model_bytes(int cls, int n_layers, int n_int, int n_raw) {
    const uint32_t tm = (uint32_t)xdl_tile_rows(cls), wp = 16u * cls, g = 64u / tm, nq = wp / (4u * g);
    const uint32_t out = (nq / 2) * 1024u + (nq % 2) * 512u;
    return 16u * 16u + ((uint32_t)(n_layers - 1) * wp + tm) * 4u + g * (wp / tm) * 1024u +
           wp * wp * 2u * (uint32_t)(n_int + 2 * n_raw) + 2u * out;
}

// Builds the operand blocks of layers [l0, l1) in LDS and their XLayer entries tab[l].  `rec` is the model record:
// the staged copy in LDS, or the record itself in global memory.
//   SLOTTED == false (resident model, l0 = 0, l1 = L): table, all bias tiles, then the blocks back to back.
//   SLOTTED == true  (streamed model): table, then one fixed-size slot per layer of the group: bias tile, blocks.
// zero_bytes from the start of LDS are cleared first (padding rows and columns, pruned weights).  Ends with a barrier.
template <int TM, int WP> struct XSlot {
    typedef XLayout<TM, WP> LY;
    static constexpr int BLOCKS = 2 * LY::HID > LY::FIRST ? (2 * LY::HID > 2 * LY::OUT ? 2 * LY::HID : 2 * LY::OUT)
                                                          : (LY::FIRST > 2 * LY::OUT ? LY::FIRST : 2 * LY::OUT);
    static constexpr int BIAS = WP * 4 > LY::OUTB ? WP * 4 : LY::OUTB;
    static constexpr int BYTES = BIAS + BLOCKS;
};

template <int TM, int WP, bool W16, bool SLOTTED>
__device__ __forceinline__ void xdl_expand_layers(char *lds, const uint32_t *rec, int L, int l0, int l1, float pre, int tid,
                                                  int nthreads, uint32_t zero_bytes) {
    typedef XLayout<TM, WP> LY;
    XLayer *tab = (XLayer *)lds;
    for (uint32_t q = tid; q < (zero_bytes >> 4); q += nthreads) ((uint4 *)lds)[q] = make_uint4(0u, 0u, 0u, 0u);   // zero_bytes is a multiple of 16
    __syncthreads();
    if (tid == 0) {
        uint32_t bias = LY::TABLE;
        uint32_t cur = LY::TABLE + (uint32_t)(L - 1) * WP * 4u + LY::OUTB;
        for (int l = l0; l < l1; ++l) {
            const LayerRec r = *(const LayerRec *)(rec + l * (sizeof(LayerRec) / 4));
            if (SLOTTED) {
                bias = LY::TABLE + (uint32_t)(l - l0) * XSlot<TM, WP>::BYTES;
                cur = bias + XSlot<TM, WP>::BIAS;
            }
            XLayer e;
            e.off_bias = bias;
            bias += l < L - 1 ? WP * 4 : LY::OUTB;
            e.scale = 1.0f;
            e.off_hi = cur;
            e.off_lo = 0;
            if (l == 0) cur += LY::FIRST;
            else if (l == L - 1) { e.off_lo = cur + LY::OUT; cur += 2 * LY::OUT; }
            else if (W16) cur += LY::HID;
            else if (xdl_int_layer(r.bits, r.scale * pre)) { e.scale = r.scale * pre; cur += LY::HID; }
            else { e.off_lo = cur + LY::HID; cur += 2 * LY::HID; }
            tab[l] = e;
        }
    }
    __syncthreads();
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, nwaves = nthreads >> 6;
    ExpandShare sh = expand_share(rec, l0, l1, wave, nwaves);
    for (int l = l0; l < l1; ++l) {
        const LayerRec r = *(const LayerRec *)(rec + l * (sizeof(LayerRec) / 4));
        const XLayer e = tab[l];
        _Float16 *hi = (_Float16 *)(lds + e.off_hi), *lo = (_Float16 *)(lds + e.off_lo);
        float *bt = (float *)(lds + e.off_bias);
        if (l == L - 1) {
            expand_layer(rec, r, lane, sh,
                         [=](int o, int i, float v, int) {
                             const _Float16 h = (_Float16)v;
                             hi[LY::idx_out(o, i)] = h;
                             lo[LY::idx_out(o, i)] = (_Float16)(v - (float)h);
                         },
                         [=](int o, float v) { bt[LY::idx_bias(4 * o)] = v; });
        } else if (l == 0) {
            expand_layer(rec, r, lane, sh,
                         [=](int o, int i, float v, int) {
                             const float w = v * pre;
                             const _Float16 h = (_Float16)w, lw = (_Float16)(w - (float)h);
                             for (int q = 0; q < LY::G; ++q) {
                                 hi[LY::idx_first(q, o, i)] = h;          // pairs with the coordinate's high half
                                 hi[LY::idx_first(q, o, 2 + i)] = h;      // ... with its low half
                                 hi[LY::idx_first(q, o, 4 + i)] = lw;     // low weight part x high coordinate half
                             }
                         },
                         [=](int o, float v) { bt[LY::idx_bias(o)] = v * pre; });
        } else if (W16) {
            expand_layer(rec, r, lane, sh, [=](int o, int i, float v, int) { hi[LY::idx_hidden(o, i)] = (_Float16)(v * pre); },
                         [=](int o, float v) { bt[LY::idx_bias(o)] = v * pre; });
        } else if (e.off_lo == 0) {
            const float inv = 1.0f / e.scale;
            expand_layer(rec, r, lane, sh, [=](int o, int i, float, int q) { hi[LY::idx_hidden(o, i)] = (_Float16)(float)q; },
                         [=](int o, float v) { bt[LY::idx_bias(o)] = v * pre * inv; });
        } else {
            expand_layer(rec, r, lane, sh,
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

// Values every lane holds alike, moved to scalar registers
__device__ __forceinline__ float uniform_f(float v) { return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v))); }
__device__ __forceinline__ XLayer uniform_layer(const XLayer e) {
    XLayer u;
    u.off_hi = __builtin_amdgcn_readfirstlane(e.off_hi);
    u.off_lo = __builtin_amdgcn_readfirstlane(e.off_lo);
    u.scale = uniform_f(e.scale);
    u.off_bias = __builtin_amdgcn_readfirstlane(e.off_bias);
    return u;
}

// ---- MFMA wrappers per tile shape -------------------------------------------------------------------
template <int TM> struct XTile;
template <> struct XTile<16> {
    typedef f32x4 acc_t;
    static __device__ __forceinline__ acc_t mfma(h8v a, h8v b, acc_t c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ acc_t mfma_half(h4v a, h4v b, acc_t c) { return __builtin_amdgcn_mfma_f32_16x16x16f16(a, b, c, 0, 0, 0); }
};
template <> struct XTile<32> {
    typedef f32x16 acc_t;
    static __device__ __forceinline__ acc_t mfma(h8v a, h8v b, acc_t c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ acc_t mfma_half(h4v, h4v, acc_t c) { return c; }     // never used: no odd quad at TM = 32
};

// sine of four accumulator values (one quad), then the exact hi/lo split of the results.
// neg1 is -1.0f passed as data so that h - float(hi) stays a single mixed-precision fma.
__device__ __forceinline__ void sine_split(float d0, float d1, float d2, float d3, float scale, float neg1, h4v &hi, h4v &lo) {
    const f2v p0 = {sin_rev(d0 * scale), sin_rev(d1 * scale)};
    const f2v p1 = {sin_rev(d2 * scale), sin_rev(d3 * scale)};
    const h2v a0 = __builtin_convertvector(p0, h2v), a1 = __builtin_convertvector(p1, h2v);
    const f2v r0 = {__builtin_fmaf((float)a0[0], neg1, p0[0]), __builtin_fmaf((float)a0[1], neg1, p0[1])};
    const f2v r1 = {__builtin_fmaf((float)a1[0], neg1, p1[0]), __builtin_fmaf((float)a1[1], neg1, p1[1])};
    const h2v b0 = __builtin_convertvector(r0, h2v), b1 = __builtin_convertvector(r1, h2v);
    hi = (h4v){a0[0], a0[1], a1[0], a1[1]};
    lo = (h4v){b0[0], b0[1], b1[0], b1[1]};
}

// sine of four accumulator values rounded to fp16 (single-term activations)
__device__ __forceinline__ void sine_hi(float d0, float d1, float d2, float d3, float scale, h4v &hi) {
    const f2v p0 = {sin_rev(d0 * scale), sin_rev(d1 * scale)};
    const f2v p1 = {sin_rev(d2 * scale), sin_rev(d3 * scale)};
    const h2v a0 = __builtin_convertvector(p0, h2v), a1 = __builtin_convertvector(p1, h2v);
    hi = (h4v){a0[0], a0[1], a1[0], a1[1]};
}

// Between the full-depth and the half-depth MFMAs of one set of accumulators: 20 wait states that no MFMA of the set
// can cross.  The empty asm statements make every accumulator an operand: the full-depth steps that produce it must
// come before the first, the half-depth steps that consume it after the last, and volatile asm statements keep their
// order, so the idle cycles sit between the two groups whatever the scheduler does with the rest.
template <class Acc> __device__ __forceinline__ void xdl_touch(Acc &acc) { asm volatile("" : "+v"(acc)); }
__device__ __forceinline__ void xdl_wait_states() { asm volatile("s_nop 15\n\ts_nop 3"); }

// ---- per-wavefront state of one half (32 pixels) of a 64-pixel tile ------------------------------------
template <int TM, int WP> struct XHalf {
    typedef XLayout<TM, WP> LY;
    static constexpr int NTH = 32 / TM;            // pixel tiles in a half: two of 16 pixels, or one of 32
    static constexpr int KJA = LY::KJ ? LY::KJ : 1;
    h8v Hh[NTH][KJA], Hl[NTH][KJA];                // activations as fp16 hi / lo, one entry per full k-step
    h4v Hh4[NTH], Hl4[NTH];                        // ... of the half-depth step (odd last quad)
    typename XTile<TM>::acc_t D[NTH][LY::MT];      // accumulators
};

// sine + split of all accumulators of a half: WP/2 activations per lane, 4 VALU instructions each
template <int TM, int WP, bool A16>
__device__ __forceinline__ void xdl_epilogue(XHalf<TM, WP> &H, float scale, float neg1) {
    typedef XLayout<TM, WP> LY;
    constexpr int QT = LY::RV / 4;                 // quads per tile
#pragma unroll
    for (int nt = 0; nt < XHalf<TM, WP>::NTH; ++nt)
#pragma unroll
        for (int t = 0; t < LY::MT; ++t)
#pragma unroll
            for (int qq = 0; qq < QT; ++qq) {
                const int q = t * QT + qq;         // quad index over the layer's rows
                h4v hi, lo;
                if (A16) sine_hi(H.D[nt][t][qq * 4 + 0], H.D[nt][t][qq * 4 + 1], H.D[nt][t][qq * 4 + 2], H.D[nt][t][qq * 4 + 3], scale, hi);
                else sine_split(H.D[nt][t][qq * 4 + 0], H.D[nt][t][qq * 4 + 1], H.D[nt][t][qq * 4 + 2], H.D[nt][t][qq * 4 + 3], scale, neg1,
                                hi, lo);
                if (q < 2 * LY::KJ) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        H.Hh[nt][q >> 1][(q & 1) * 4 + v] = hi[v];
                        if (!A16) H.Hl[nt][q >> 1][(q & 1) * 4 + v] = lo[v];
                    }
                } else {
                    H.Hh4[nt] = hi;
                    if (!A16) H.Hl4[nt] = lo;
                }
            }
}

// MFMAs of one hidden layer for a half.  LO: the layer has a low weight part (one more term).  A16: no low activation part.
template <int TM, int WP, bool LO, bool A16>
__device__ __forceinline__ void xdl_hidden(XHalf<TM, WP> &H, const char *lds, const XLayer el, int lane, int g) {
    typedef XLayout<TM, WP> LY;
    typedef XTile<TM> T;
    typedef typename T::acc_t acc_t;
    constexpr int KJ = LY::KJ, K16 = LY::K16, MT = LY::MT, NTH = XHalf<TM, WP>::NTH;
    const h8v *ah = (const h8v *)(lds + el.off_hi) + lane;
    const h8v *al = (const h8v *)(lds + el.off_lo) + lane;
    const h4v *ah4 = (const h4v *)(lds + el.off_hi + KJ * MT * 1024) + lane;
    const h4v *al4 = (const h4v *)(lds + el.off_lo + KJ * MT * 1024) + lane;
    const acc_t *bt = (const acc_t *)(lds + el.off_bias) + g;
#pragma unroll
    for (int j = 0; j < KJ; ++j)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const h8v av = ah[(j * MT + mt) * 64];
            h8v aw;
            if (LO) aw = al[(j * MT + mt) * 64];
            acc_t c;
            if (j == 0) c = bt[mt * LY::G];
#pragma unroll
            for (int nt = 0; nt < NTH; ++nt) H.D[nt][mt] = T::mfma(av, H.Hh[nt][j], j == 0 ? c : H.D[nt][mt]);
            if (!A16) {
#pragma unroll
                for (int nt = 0; nt < NTH; ++nt) H.D[nt][mt] = T::mfma(av, H.Hl[nt][j], H.D[nt][mt]);
            }
            if (LO) {
#pragma unroll
                for (int nt = 0; nt < NTH; ++nt) H.D[nt][mt] = T::mfma(aw, H.Hh[nt][j], H.D[nt][mt]);
            }
        }
    if (K16) {
        if (KJ) {
#pragma unroll
            for (int nt = 0; nt < NTH; ++nt)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) xdl_touch(H.D[nt][mt]);
            xdl_wait_states();
#pragma unroll
            for (int nt = 0; nt < NTH; ++nt)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) xdl_touch(H.D[nt][mt]);
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const h4v av = ah4[mt * 64];
            h4v aw;
            if (LO) aw = al4[mt * 64];
            acc_t c;
            if (KJ == 0) c = bt[mt * LY::G];
#pragma unroll
            for (int nt = 0; nt < NTH; ++nt) H.D[nt][mt] = T::mfma_half(av, H.Hh4[nt], KJ == 0 ? c : H.D[nt][mt]);
            if (!A16) {
#pragma unroll
                for (int nt = 0; nt < NTH; ++nt) H.D[nt][mt] = T::mfma_half(av, H.Hl4[nt], H.D[nt][mt]);
            }
            if (LO) {
#pragma unroll
                for (int nt = 0; nt < NTH; ++nt) H.D[nt][mt] = T::mfma_half(aw, H.Hh4[nt], H.D[nt][mt]);
            }
        }
    }
}

// One hidden layer for both halves of a 64-pixel tile, software-pipelined: the matrix work of X(l) is issued
// together with the sine/split of Y(l-1), then the matrix work of Y(l) with the sine/split of X(l).
template <int TM, int WP, bool LO, bool A16>
__device__ __forceinline__ void xdl_layer(XHalf<TM, WP> &X, XHalf<TM, WP> &Y, const char *lds, const XLayer el, int lane, int g,
                                          float scale_prev, float scale, float neg1) {
    xdl_hidden<TM, WP, LO, A16>(X, lds, el, lane, g);
    xdl_epilogue<TM, WP, A16>(Y, scale_prev, neg1);
    __builtin_amdgcn_sched_barrier(0);
    xdl_hidden<TM, WP, LO, A16>(Y, lds, el, lane, g);
    xdl_epilogue<TM, WP, A16>(X, scale, neg1);
}

// The slot's augmentation map (every lane holds it alike), in scalar registers.
struct XUniform {
    float af0, af1, af2, af3, af4, af5;
};
__device__ __forceinline__ XUniform xdl_uniform(const DecodeArgs &a, uint32_t slot) {
    XUniform u;
    u.af0 = 1.0f; u.af1 = 0.0f; u.af2 = 0.0f; u.af3 = 0.0f; u.af4 = 1.0f; u.af5 = 0.0f;   // augmentation: this slot's map of the sampling grid
    if (a.affine) {
        const float *m = a.affine + (size_t)slot * 6;
        u.af0 = uniform_f(m[0]); u.af1 = uniform_f(m[1]); u.af2 = uniform_f(m[2]);
        u.af3 = uniform_f(m[3]); u.af4 = uniform_f(m[4]); u.af5 = uniform_f(m[5]);
    }
    return u;
}

// ---- first layer: every lane forms the coordinates of one pixel of the tile as hi/lo halfs in
//      k slots (xh, yh, xl, yl, xh, yh, 0, 0); the MFMA of pixel tile q uses the weight variant whose
//      non-zero k slots are lane group q's, so one operand register set serves all pixel tiles.
//      Per-lane values that only the first and the last layer use are derived again for every tile
//      (the empty asm keeps them from being hoisted): held across the hidden layers they would
//      push the kernel over its register budget.
template <int TM, int WP>
__device__ __forceinline__ void xdl_first(XHalf<TM, WP> &X, XHalf<TM, WP> &Y, const DecodeArgs &a, const XUniform &u, const char *lds,
                                          const XLayer e0, uint32_t tile, int lane) {
    typedef XLayout<TM, WP> LY;
    typedef XTile<TM> T;
    typedef typename T::acc_t acc_t;
    constexpr int MT = LY::MT, G = LY::G, NTH = XHalf<TM, WP>::NTH;
    const int g = lane / TM;
    float lo_v = a.lo, af2 = u.af2, af5 = u.af5;        // second uniform operand of an fma: copied to a vector register at the use
    asm volatile("" : "+s"(lo_v), "+s"(af2), "+s"(af5));
    const h8v *a0 = (const h8v *)(lds + e0.off_hi) + lane;
    const acc_t *bt = (const acc_t *)(lds + e0.off_bias) + g;
    // lane (pixel tile q = lane / TM, column n = lane % TM) feeds pixel n * (64 / TM) + q of the 64: a lane's columns of the
    // pixel tiles are then consecutive pixels, which the output layer stores as one vector
    uint32_t p = (tile << 6) + (uint32_t)(lane % TM) * (64 / TM) + (uint32_t)(lane / TM);
    p = min(p, a.HW - 1);
    const uint32_t row = a.wmagic ? (__umulhi(p, a.wmagic) >> a.wshift) : p, col = p - row * a.W;
    const float x0 = fmaf(a.span, (float)(2 * col + 1) * a.inv2W, lo_v);
    const float y0 = fmaf(a.span, (float)(2 * row + 1) * a.inv2H, lo_v);
    const float x = fmaf(u.af0, x0, fmaf(u.af1, y0, af2)), y = fmaf(u.af3, x0, fmaf(u.af4, y0, af5));
    const _Float16 xh = (_Float16)x, yh = (_Float16)y;
    const _Float16 xl = (_Float16)(x - (float)xh), yl = (_Float16)(y - (float)yh);
    const _Float16 z = (_Float16)0.0f;
    const h8v b0 = {xh, yh, xl, yl, xh, yh, z, z};
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const acc_t c = bt[mt * G];
#pragma unroll
        for (int nt = 0; nt < NTH; ++nt) {
            X.D[nt][mt] = T::mfma(a0[(nt * MT + mt) * 64], b0, c);
            Y.D[nt][mt] = T::mfma(a0[((NTH + nt) * MT + mt) * 64], b0, c);
        }
    }
}

// ---- output layer width -> 3: one TM-row tile with channel c in row 4c.  At TM = 16 that is
//      register 0 of lane group c; at TM = 32 registers 0 (R) and 4 (B) of group 0, register 0 (G) of group 1.
//      Then clamp, optional normalisation and the NCHW store.
template <int TM, int WP, bool A16>
__device__ __forceinline__ void xdl_output(const XHalf<TM, WP> &X, const XHalf<TM, WP> &Y, const DecodeArgs &a, float ns0, float ns1,
                                           float ns2, float nb0, float nb1, float nb2, const char *lds, const XLayer eo,
                                           uint32_t tile, int lane, size_t plane0) {
    typedef XLayout<TM, WP> LY;
    typedef XTile<TM> T;
    typedef typename T::acc_t acc_t;
    constexpr int KJ = LY::KJ, K16 = LY::K16, NTH = XHalf<TM, WP>::NTH;
    const int go = lane / TM, no = lane % TM;
    const h8v *ah = (const h8v *)(lds + eo.off_hi) + lane;
    const h8v *al = (const h8v *)(lds + eo.off_lo) + lane;
    const h4v *ah4 = (const h4v *)(lds + eo.off_hi + KJ * 1024) + lane;
    const h4v *al4 = (const h4v *)(lds + eo.off_lo + KJ * 1024) + lane;
    const acc_t c = ((const acc_t *)(lds + eo.off_bias))[go];
    acc_t O[2 * NTH];
#pragma unroll
    for (int nt = 0; nt < 2 * NTH; ++nt) O[nt] = c;
#pragma unroll
    for (int j = 0; j < KJ; ++j) {
        const h8v av = ah[j * 64], aw = al[j * 64];
#pragma unroll
        for (int nt = 0; nt < 2 * NTH; ++nt) {
            const h8v bh = nt < NTH ? X.Hh[nt % NTH][j] : Y.Hh[nt % NTH][j];
            O[nt] = T::mfma(av, bh, O[nt]);
            if (!A16) O[nt] = T::mfma(av, nt < NTH ? X.Hl[nt % NTH][j] : Y.Hl[nt % NTH][j], O[nt]);
            O[nt] = T::mfma(aw, bh, O[nt]);
        }
    }
    if (K16) {
        if (KJ) {
#pragma unroll
            for (int nt = 0; nt < 2 * NTH; ++nt) xdl_touch(O[nt]);
            xdl_wait_states();
#pragma unroll
            for (int nt = 0; nt < 2 * NTH; ++nt) xdl_touch(O[nt]);
        }
        const h4v av = ah4[0], aw = al4[0];
#pragma unroll
        for (int nt = 0; nt < 2 * NTH; ++nt) {
            const h4v bh = nt < NTH ? X.Hh4[nt % NTH] : Y.Hh4[nt % NTH];
            O[nt] = T::mfma_half(av, bh, O[nt]);
            if (!A16) O[nt] = T::mfma_half(av, nt < NTH ? X.Hl4[nt % NTH] : Y.Hl4[nt % NTH], O[nt]);
            O[nt] = T::mfma_half(aw, bh, O[nt]);
        }
    }
    // lane (go, no) holds column `no` of every pixel tile: pixels p0 .. p0 + NT - 1 of the image, NT = 64 / TM
    constexpr int NT = 2 * NTH;
    constexpr int NS = TM == 16 ? 1 : 2;         // channels a lane stores: TM = 16: channel go; TM = 32: R and B (group 0), G (group 1)
    const uint32_t p0 = (tile << 6) + (uint32_t)no * NT;
#pragma unroll
    for (int k = 0; k < NS; ++k) {
        const int ch = TM == 16 ? go : (go == 0 ? 2 * k : 1);
        const bool live = TM == 16 ? go < 3 : (go == 0 || k == 0);
        float r[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            r[nt] = O[nt][TM == 16 ? 0 : 4 * k];
            if (!a.no_clamp) r[nt] = fminf(fmaxf(r[nt], 0.0f), 1.0f);
            if (a.normalize) r[nt] = fmaf(r[nt], ch == 0 ? ns0 : (ch == 1 ? ns1 : ns2), ch == 0 ? nb0 : (ch == 1 ? nb1 : nb2));
        }
        const uint32_t at = (uint32_t)ch * a.HW + p0;       // within the slot's three planes: 3 HW < 2^32 is checked by the host
        if (a.vec_store) {                                  // HW is a multiple of 4 and the outputs are aligned: whole vectors
            if (live && p0 < a.HW) {
                if (a.out_f32) {
                    float *dst = a.out_f32 + plane0 + at;
                    if constexpr (NT == 4) *(f32x4 *)dst = (f32x4){r[0], r[1], r[2], r[3]};
                    else *(f2v *)dst = (f2v){r[0], r[1]};
                }
                if (a.out_u8) {
                    uint32_t pk = 0u;
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) pk = __builtin_amdgcn_cvt_pk_u8_f32(255.0f * r[nt], nt, pk);   // round to nearest even, packed
                    uint8_t *dst = a.out_u8 + plane0 + at;
                    if constexpr (NT == 4) *(uint32_t *)dst = pk;
                    else *(uint16_t *)dst = (uint16_t)pk;
                }
            }
        } else {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                if (live && p0 + nt < a.HW) {
                    if (a.out_f32) (a.out_f32 + plane0)[at + nt] = r[nt];
                    if (a.out_u8) (a.out_u8 + plane0)[at + nt] = (uint8_t)rintf(255.0f * r[nt]);
                }
        }
    }
}

// Resident form: the model is expanded once per workgroup; a wavefront takes one 64-pixel tile at a time through all
// layers.
template <int TM, int WP, int MODE_>
__device__ __forceinline__ void xdl_body(const DecodeArgs &a, const Work &w, float *lds_f) {
    constexpr bool W16 = (MODE_ & kWeight16) != 0;
    constexpr int MODE = W16 ? (int)kHiddenAllRaw : (MODE_ & 3);      // all-fp16: one form for every hidden layer, no scale
    constexpr bool A16 = (MODE_ & kAct16) != 0 || W16;
    typedef XHalf<TM, WP> Half;
    char *lds = (char *)lds_f;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const uint32_t tile0 = w.tile0, tile1 = w.tile1;
    const size_t plane0 = w.plane0;
    const IndexEntry e = w.e;
    const int L = e.n_layers;

    // the packed record is staged at the end of the workgroup's LDS, the operand blocks are built at the start
    uint32_t *stage = (uint32_t *)(lds + (a.lds_bytes - e.nbytes));
    {
        const uint4 *src = (const uint4 *)(a.blob + e.off);
        uint4 *dst = (uint4 *)stage;
        for (uint32_t q = tid; q < (e.nbytes >> 4); q += nthreads) dst[q] = src[q];
    }
    // Tiles are handed out through a counter in LDS (it reuses the first word of the staging area,
    // which is dead once the model is expanded): the SIMD arbiter favours its older wavefront, so
    // with a fixed split the favoured waves would finish early and leave the others running alone.
    xdl_expand_layers<TM, WP, W16, false>(lds, stage, L, 0, L, a.pre, tid, nthreads, a.lds_bytes - e.nbytes);
    uint32_t *next_tile = stage;
    if (tid == 0) *next_tile = tile0 + (nthreads >> 6);
    __syncthreads();

    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const XLayer *tab = (const XLayer *)lds;
    const float neg1 = a.neg1;
    const XLayer e0 = uniform_layer(tab[0]), eo = uniform_layer(tab[L - 1]);
    const XUniform u = xdl_uniform(a, w.slot);
    // per-channel normalisation constants as values (not as an address chosen per lane)
    const float ns0 = uniform_f(a.ns[0]), ns1 = uniform_f(a.ns[1]), ns2 = uniform_f(a.ns[2]);
    const float nb0 = uniform_f(a.nb[0]), nb1 = uniform_f(a.nb[1]), nb2 = uniform_f(a.nb[2]);

    for (uint32_t tile = tile0 + wave; tile < tile1;) {
        Half X, Y;
        uint32_t ones = ~0u;
        asm volatile("" : "+s"(ones));
        int lane = (int)__builtin_amdgcn_mbcnt_hi(ones, __builtin_amdgcn_mbcnt_lo(ones, 0u));
        xdl_first<TM, WP>(X, Y, a, u, lds, e0, tile, lane);
        xdl_epilogue<TM, WP, A16>(X, 1.0f, neg1);
        // ---- hidden layers, software-pipelined over the two halves:
        //      matrix work of X(l) with the sine/split of Y(l-1), then matrix work of Y(l) with the sine/split of X(l)
        float scale_prev = 1.0f;
        int l = 1;
        if (MODE == kHiddenAllInt && L > 2) {      // first hidden layer on its own: the first layer's outputs carry no scale
            const XLayer el = uniform_layer(tab[1]);
            int ll = lane;
            asm volatile("" : "+v"(ll));
            xdl_layer<TM, WP, false, A16>(X, Y, lds, el, ll, ll / TM, 1.0f, el.scale, neg1);
            scale_prev = el.scale;
            l = 2;
        }
        for (; l < L - 1; ++l) {
            const XLayer el = uniform_layer(tab[l]);
            int ll = lane;                       // the lane group is derived from the lane index per layer, not kept
            asm volatile("" : "+v"(ll));
            if constexpr (MODE == kHiddenAllInt) {
                xdl_layer<TM, WP, false, A16>(X, Y, lds, el, ll, ll / TM, scale_prev, el.scale, neg1);
            } else if constexpr (MODE == kHiddenAllRaw) {
                xdl_layer<TM, WP, !W16, A16>(X, Y, lds, el, ll, ll / TM, 1.0f, 1.0f, neg1);
            } else {
                if (el.off_lo == 0) xdl_layer<TM, WP, false, A16>(X, Y, lds, el, ll, ll / TM, scale_prev, el.scale, neg1);
                else xdl_layer<TM, WP, true, A16>(X, Y, lds, el, ll, ll / TM, scale_prev, el.scale, neg1);
            }
            scale_prev = el.scale;
        }
        xdl_epilogue<TM, WP, A16>(Y, scale_prev, neg1);
        asm volatile("" : "+s"(ones));           // pixel indices and addresses: derived again rather than kept
        lane = (int)__builtin_amdgcn_mbcnt_hi(ones, __builtin_amdgcn_mbcnt_lo(ones, 0u));
        xdl_output<TM, WP, A16>(X, Y, a, ns0, ns1, ns2, nb0, nb1, nb2, lds, eo, tile, lane, plane0);
        uint32_t nt_ = 0;
        if (lane == 0) nt_ = atomicAdd(next_tile, 1u);
        tile = __builtin_amdgcn_readfirstlane(nt_);
    }
}

// Streamed form, for a model whose operand blocks do not fit LDS: the layers go through LDS in groups of as many
// slots as fit.  Every wavefront keeps one tile in registers (both halves, mid-pipeline: X holds activations, Y
// accumulators awaiting their sine); for each group the workgroup builds the group's blocks straight from the
// packed record in global memory, then every wavefront takes its tile through the group's layers.
template <int TM, int WP, int MODE_>
__device__ __forceinline__ void xdl_stream_body(const DecodeArgs &a, const Work &w, float *lds_f) {
    constexpr bool W16 = (MODE_ & kWeight16) != 0;
    constexpr bool A16 = (MODE_ & kAct16) != 0 || W16;
    typedef XLayout<TM, WP> LY;
    typedef XHalf<TM, WP> Half;
    char *lds = (char *)lds_f;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = nthreads >> 6;
    const IndexEntry e = w.e;
    const int L = e.n_layers;
    const int K = (int)((a.lds_bytes - LY::TABLE) / (uint32_t)XSlot<TM, WP>::BYTES);   // layers per group (>= 1 by the host's launch size)
    const uint32_t *rec = (const uint32_t *)(a.blob + e.off);
    const XLayer *tab = (const XLayer *)lds;
    const float neg1 = a.neg1;
    const XUniform u = xdl_uniform(a, w.slot);
    // per-channel normalisation constants as values (not as an address chosen per lane)
    const float ns0 = uniform_f(a.ns[0]), ns1 = uniform_f(a.ns[1]), ns2 = uniform_f(a.ns[2]);
    const float nb0 = uniform_f(a.nb[0]), nb1 = uniform_f(a.nb[1]), nb2 = uniform_f(a.nb[2]);

    for (uint32_t t0 = w.tile0; t0 < w.tile1; t0 += (uint32_t)nwaves) {
        const uint32_t tile = t0 + (uint32_t)wave;
        const bool active = tile < w.tile1;                            // the same for a whole wavefront
        Half X, Y;
        float scale_prev = 1.0f;
        for (int l0 = 0; l0 < L; l0 += K) {
            const int l1 = l0 + K < L ? l0 + K : L;
            __syncthreads();                                           // every wavefront is done with the previous group
            xdl_expand_layers<TM, WP, W16, true>(lds, rec, L, l0, l1, a.pre, tid, nthreads,
                                                 LY::TABLE + (uint32_t)(l1 - l0) * XSlot<TM, WP>::BYTES);
            if (!active) continue;
            for (int l = l0; l < l1; ++l) {
                const XLayer el = uniform_layer(tab[l]);
                if (l == 0) {
                    xdl_first<TM, WP>(X, Y, a, u, lds, el, tile, lane);
                    xdl_epilogue<TM, WP, A16>(X, 1.0f, neg1);
                } else if (l < L - 1) {
                    if (W16) xdl_layer<TM, WP, false, A16>(X, Y, lds, el, lane, lane / TM, 1.0f, 1.0f, neg1);
                    else if (el.off_lo == 0) xdl_layer<TM, WP, false, A16>(X, Y, lds, el, lane, lane / TM, scale_prev, el.scale, neg1);
                    else xdl_layer<TM, WP, true, A16>(X, Y, lds, el, lane, lane / TM, scale_prev, el.scale, neg1);
                    scale_prev = W16 ? 1.0f : el.scale;
                } else {
                    xdl_epilogue<TM, WP, A16>(Y, scale_prev, neg1);
                    xdl_output<TM, WP, A16>(X, Y, a, ns0, ns1, ns2, nb0, nb1, nb2, lds, el, tile, lane, w.plane0);
                }
            }
        }
    }
}

// One width class per launch (a.cls != 0) ...
template <int CLS, int NTHREADS, int MODE>
__global__ __launch_bounds__(NTHREADS) void decode_xdl_kernel(const DecodeArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds_f[];
    Work w;
    if (!decode_prologue(a, w)) return;
    xdl_body<xdl_tile_rows(CLS), 16 * CLS, MODE>(a, w, lds_f);
}

// ... or every width class in one launch (a.cls == 0)
template <int NTHREADS, int MODE>
__global__ __launch_bounds__(NTHREADS) void decode_xdl_any_kernel(const DecodeArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds_f[];
    Work w;
    if (!decode_prologue(a, w)) return;
    switch (w.cls) {
        case 1: xdl_body<xdl_tile_rows(1), 16, MODE>(a, w, lds_f); break;
        case 2: xdl_body<xdl_tile_rows(2), 32, MODE>(a, w, lds_f); break;
        case 3: xdl_body<xdl_tile_rows(3), 48, MODE>(a, w, lds_f); break;
        default: xdl_body<32, 64, MODE>(a, w, lds_f); break;    // 32-row tiles: measured faster here, slower in the one-class kernel;
                                                                // the layout is smaller than the 16-row one the host sizes LDS for
    }
}

// The streamed form: one width class per launch, one wavefront per SIMD.  MODE: 0 (hi+lo activations, any kind of
// hidden layer), kAct16, or kAct16 | kWeight16.
template <int CLS, int MODE>
__global__ __launch_bounds__(kStreamThreads) void decode_xdl_stream_kernel(const DecodeArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds_f[];
    Work w;
    if (!decode_prologue(a, w)) return;
    xdl_stream_body<xdl_tile_rows(CLS), 16 * CLS, MODE>(a, w, lds_f);
}

// ---- debug export of the split-precision operand blocks (see rinr_debug_dequant_split) ----------------------------
template <int TM, int WP, bool W16>
__global__ __launch_bounds__(256) void xdl_debug_kernel(const uint8_t *blob, int64_t id, int layer, uint32_t lds_bytes,
                                                        float *hi_out, float *lo_out, float *bias_out, float *scale_out) {
    typedef XLayout<TM, WP> LY;
    extern __shared__ __attribute__((aligned(16))) float lds_f[];
    char *lds = (char *)lds_f;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const IndexEntry e = *(const IndexEntry *)(blob + sizeof(StoreHeader) + (size_t)id * sizeof(IndexEntry));
    const int L = e.n_layers;
    const uint32_t *rec = (const uint32_t *)(blob + e.off);
    // one layer at a time in the slotted layout, straight from global memory: any depth fits
    xdl_expand_layers<TM, WP, W16, true>(lds, rec, L, layer, layer + 1, 1.0f, tid, nthreads, lds_bytes);
    const XLayer el = ((const XLayer *)lds)[layer];
    const LayerRec r = *(const LayerRec *)(rec + layer * (sizeof(LayerRec) / 4));
    const _Float16 *hi = (const _Float16 *)(lds + el.off_hi), *lo = (const _Float16 *)(lds + el.off_lo);
    const float *bt = (const float *)(lds + el.off_bias);
    const int n_in = r.n_in, cnt = r.n_in * r.n_out;
    const float nan = __uint_as_float(0x7FC00000u);
    for (int k = tid; k < cnt; k += nthreads) {
        const int o = k / n_in, i = k - o * n_in;
        float h, l;
        if (layer == L - 1) {
            h = (float)hi[LY::idx_out(o, i)];
            l = (float)lo[LY::idx_out(o, i)];
        } else if (layer == 0) {
            h = (float)hi[LY::idx_first(0, o, i)];
            l = (float)hi[LY::idx_first(0, o, 4 + i)];
            for (int q = 0; q < LY::G; ++q) {          // every copy must agree
                if ((float)hi[LY::idx_first(q, o, i)] != h || (float)hi[LY::idx_first(q, o, 2 + i)] != h) h = nan;
                if ((float)hi[LY::idx_first(q, o, 4 + i)] != l) l = nan;
            }
        } else {
            h = (float)hi[LY::idx_hidden(o, i)];
            l = el.off_lo ? (float)lo[LY::idx_hidden(o, i)] : 0.0f;
        }
        hi_out[k] = h;
        lo_out[k] = l;
    }
    if (bias_out)
        for (int o = tid; o < r.n_out; o += nthreads) bias_out[o] = bt[LY::idx_bias(layer == L - 1 ? 4 * o : o)];
    if (scale_out && tid == 0) *scale_out = el.scale;
}

}  // namespace rinr

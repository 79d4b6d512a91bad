// Device code of the decode path: on-chip weight layout, expand/dequantise stage and the
// fused per-pixel MLP kernel.  gfx950 (CDNA4) only: 64-lane wavefronts, fp32 MFMA.
//
// Method (paper Sec. III-B): every pixel of every image of the batch is decoded in
// parallel by pushing its normalised (x, y) through that image's own MLP.  Here one
// workgroup owns (batch slot, range of pixel tiles).  It rebuilds the image's fp32
// weights once into LDS from the packed record (mask + kept-code stream + affine map,
// Sec. IV-A/B), then each wavefront walks its tiles of 64 pixels through all layers with
// the activations held in registers from the first layer to the RGB store.
//
// Layers are evaluated transposed, Hout[width x pixels] = Wmat[width x width] * Hin, with
// the weights as the MFMA A operand and pixels along the N axis.  The rows of an
// accumulator tile that a lane owns are then exactly the contraction indices that lane
// must supply as B operand of the next layer, provided the next layer's weights are laid
// out in LDS with the matching permutation of k.  So bias (as the C operand of the first
// k-step) and sin are applied in place and nothing crosses lanes between layers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "rinr_format.h"

namespace rinr {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// ---- MFMA tile traits --------------------------------------------------------------------
// TM = rows (and pixel columns) of one tile.  A lane is (n = lane % TM, g = lane / TM).
//   A operand: lane supplies A[row n][k = g]      B operand: lane supplies B[k = g][col n]
//   D tile   : RV registers per lane; register v holds row (v>>2)*4G + 4g + (v&3), column n
template <int TM> struct Tile;
template <> struct Tile<16> {
    static constexpr int G = 4, RV = 4;
    typedef f32x4 acc_t;
    static __device__ __forceinline__ acc_t mfma(float a, float b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
};
template <> struct Tile<32> {
    static constexpr int G = 2, RV = 16;
    typedef f32x16 acc_t;
    static __device__ __forceinline__ acc_t mfma(float a, float b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
};

// ---- LDS layout of one expanded model --------------------------------------------------
// WP = padded width (multiple of TM).  All indices are in floats.
template <int TM, int WP> struct Layout {
    typedef Tile<TM> T;
    static constexpr int G = T::G, RV = T::RV;
    static constexpr int MT = WP / TM;                 // row tiles per layer
    static constexpr int MTS = (MT == 3) ? 4 : MT;     // stride of the per-lane A vector
    static constexpr int KSTEPS = WP / G;              // MFMA k-steps of a hidden layer
    static constexpr int FIRST = 64 * MTS;             // first layer: one k-step
    static constexpr int HIDDEN = KSTEPS * 64 * MTS;   // one hidden layer
    static constexpr int OUTW = 4 * WP;                // output layer, float4 per (g, r)
    static_assert(WP % TM == 0, "padded width must be whole tiles");

    // row-in-tile rr -> (lane group g, accumulator register v)
    static __device__ __forceinline__ void split(int rr, int &g, int &v) {
        if (TM == 16) { g = rr >> 2; v = rr & 3; }
        else { g = (rr >> 2) & 1; v = ((rr >> 3) << 2) | (rr & 3); }
    }
    static __device__ __forceinline__ int idx_first(int o, int i) {       // i in {0, 1}
        const int mt = o / TM, mr = o % TM;
        return (i * TM + mr) * MTS + mt;
    }
    static __device__ __forceinline__ int idx_hidden(int o, int i) {
        const int mt = o / TM, mr = o % TM, t = i / TM;
        int g, v;
        split(i % TM, g, v);
        return ((t * RV + v) * 64 + g * TM + mr) * MTS + mt;
    }
    static __device__ __forceinline__ int idx_bias(int o) {
        int g, v;
        split(o % TM, g, v);
        return ((o / TM) * G + g) * RV + v;
    }
    static __device__ __forceinline__ int idx_out(int c, int i) {
        int g, v;
        split(i % TM, g, v);
        return (g * KSTEPS + (i / TM) * RV + v) * 4 + c;
    }
    // offsets of the segments for a model with L linear layers (L >= 2)
    static __device__ __host__ __forceinline__ int off_first() { return 0; }
    static __device__ __host__ __forceinline__ int off_bias(int l) { return FIRST + l * WP; }
    static __device__ __host__ __forceinline__ int off_hidden(int L, int l) { return FIRST + (L - 1) * WP + (l - 1) * HIDDEN; }
    static __device__ __host__ __forceinline__ int off_out(int L) { return off_hidden(L, L - 1); }
    static __device__ __host__ __forceinline__ int off_outb(int L) { return off_out(L) + OUTW; }
    static __device__ __host__ __forceinline__ int total(int L) { return off_outb(L) + 4; }
};

// ---- expand + dequantise (Sec. IV-A mask, Sec. IV-B codes) -----------------------------
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    return x;
}

__device__ __forceinline__ uint32_t take_code(const uint32_t *cs, uint32_t rank, uint32_t cb) {
    const uint32_t bit = rank * cb;
    const uint32_t w = bit >> 5, sh = bit & 31;
    const uint64_t two = (uint64_t)cs[w] | ((uint64_t)cs[w + 1] << 32);
    const uint32_t m = cb == 32 ? 0xFFFFFFFFu : ((1u << cb) - 1u);
    return (uint32_t)(two >> sh) & m;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t x) {
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) x += __shfl_xor(x, d, 64);
    return x;
}

// The weights of a model are cut into blocks of 64 consecutive flat indices, layer after layer, and the workgroup's
// wavefronts share the blocks of the layers at hand (the whole model, or one group of its layers) evenly: wavefront w
// of nw takes blocks [B w / nw, B (w + 1) / nw) of the B blocks counted over those layers, so a wavefront touches one
// or two layers whatever the depth and the widths.
struct ExpandShare {
    uint32_t g0, g1;      // this wavefront's range of blocks, counted over all layers
    uint32_t base;        // blocks of the layers before the one at hand (advanced by expand_layer)
};
__device__ __forceinline__ ExpandShare expand_share(const uint32_t *rec, int l0, int l1, int wave, int nwaves) {
    uint32_t total = 0;
    for (int l = l0; l < l1; ++l) {
        const LayerRec *r = (const LayerRec *)(rec + l * (sizeof(LayerRec) / 4));
        total += ((uint32_t)r->n_in * r->n_out + 63) >> 6;
    }
    ExpandShare s;
    s.g0 = total * (uint32_t)wave / (uint32_t)nwaves;
    s.g1 = total * (uint32_t)(wave + 1) / (uint32_t)nwaves;
    s.base = 0;
    return s;
}

// This wavefront's part of one layer, one weight per lane.  `rec` is the model record (words; the staged copy in LDS,
// or the record itself in global memory).  Over the workgroup, put(o, i, w, q) receives every KEPT weight of the true
// n_out x n_in matrix exactly once: w the fp32 value and q the integer code - zp of a coded layer (0 for fp32 layers);
// pruned weights are not reported (the caller's area starts out as zeros); putb(o, b) receives every bias (from the
// wavefront that holds the layer's first block).  A kept weight's code is found by its rank among the kept ones: the
// count before the wavefront's first block by one reduction over the mask words, then, per block of 64 weights, the
// block's keep bits as one 64-bit lane mask (a ballot), the lane's rank by a masked bit count, and the running count in
// a scalar register.
template <class PutW, class PutB>
__device__ __forceinline__ void expand_layer(const uint32_t *rec, const LayerRec &r, int lane, ExpandShare &sh, PutW put, PutB putb) {
    const uint32_t n_in = r.n_in, cnt = (uint32_t)r.n_in * r.n_out;
    const uint32_t nwords = (cnt + 31) >> 5, nblocks = (cnt + 63) >> 6;
    const uint32_t first = sh.base, last = sh.base + nblocks;
    sh.base = last;
    if (sh.g1 <= first || sh.g0 >= last) return;
    const uint32_t b0 = sh.g0 > first ? sh.g0 - first : 0u, b1 = (sh.g1 < last ? sh.g1 : last) - first;
    const uint32_t *mw = rec + (r.mask_off >> 2);
    const uint32_t *cs = rec + (r.code_off >> 2);
    const uint32_t cb = r.bits ? r.bits : 32u;
    const uint32_t magic = n_in > 1 ? 0xFFFFFFFFu / n_in + 1u : 0u;     // ceil(2^32 / n_in): k / n_in == umulhi(k, magic) for k < 2^16
    const bool has_mask = r.has_mask != 0;
    uint32_t running = 0;
    if (b0) {
        if (has_mask) {
            uint32_t part = 0;
            for (uint32_t wi = lane; wi < 2 * b0; wi += 64) part += __popc(wi < nwords ? mw[wi] : 0u);
            running = (uint32_t)__builtin_amdgcn_readfirstlane((int)wave_sum(part));
        } else {
            running = b0 << 6;          // dense: every weight before the block is kept (b0 < nblocks, so all of them exist)
        }
    }
    for (uint32_t b = b0; b < b1; ++b) {
        const uint32_t k = (b << 6) + (uint32_t)lane;
        bool kept = k < cnt;
        if (has_mask) {
            const uint32_t wi = k >> 5;
            const uint32_t word = wi < nwords ? mw[wi] : 0u;      // bits past the layer's end are zero in a valid record
            kept = (word >> ((uint32_t)lane & 31u)) & 1u;
        }
        const uint64_t keep64 = __ballot(kept);
        const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(keep64 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)keep64, running));
        running += (uint32_t)__popcll(keep64);
        if (kept) {
            uint32_t code;
            if (cb == 8u) code = ((const uint8_t *)cs)[rank];
            else if (cb == 32u) code = cs[rank];
            else if (cb == 16u) code = ((const uint16_t *)cs)[rank];
            else code = take_code(cs, rank, cb);
            const uint32_t o = n_in == 1 ? k : __umulhi(k, magic), i = k - o * n_in;
            float val;
            int32_t q = 0;
            if (r.bits) { q = (int32_t)code - r.zp; val = r.scale * (float)q; }
            else val = __uint_as_float(code);
            put((int)o, (int)i, val, q);
        }
    }
    if (b0 == 0) {
        const float *bias = (const float *)(rec + (r.bias_off >> 2));
        for (uint32_t o = (uint32_t)lane; o < r.n_out; o += 64u) putb((int)o, bias[o]);
    }
}

// Whole model: zero the expanded area, then every wavefront its share of the blocks.  `pre` scales the
// weights and biases of the sine layers (w0 / 2pi, so that the pre-activation is in
// revolutions); the output layer is never scaled.  Ends with a workgroup barrier.
template <int TM, int WP>
__device__ __forceinline__ void expand_model(float *lds, const uint32_t *rec, int L, float pre, int tid, int nthreads) {
    typedef Layout<TM, WP> LY;
    const int total = LY::total(L);
    for (int q = tid; q < total; q += nthreads) lds[q] = 0.0f;
    __syncthreads();
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, nwaves = nthreads >> 6;
    ExpandShare sh = expand_share(rec, 0, L, wave, nwaves);
    for (int l = 0; l < L; ++l) {
        const LayerRec r = *(const LayerRec *)(rec + l * (sizeof(LayerRec) / 4));
        if (l == L - 1) {
            float *w = lds + LY::off_out(L), *b = lds + LY::off_outb(L);
            expand_layer(rec, r, lane, sh, [=](int o, int i, float v, int) { w[LY::idx_out(o, i)] = v; },
                         [=](int o, float v) { b[o] = v; });
        } else if (l == 0) {
            float *w = lds + LY::off_first(), *b = lds + LY::off_bias(0);
            expand_layer(rec, r, lane, sh, [=](int o, int i, float v, int) { w[LY::idx_first(o, i)] = v * pre; },
                         [=](int o, float v) { b[LY::idx_bias(o)] = v * pre; });
        } else {
            float *w = lds + LY::off_hidden(L, l), *b = lds + LY::off_bias(l);
            expand_layer(rec, r, lane, sh, [=](int o, int i, float v, int) { w[LY::idx_hidden(o, i)] = v * pre; },
                         [=](int o, float v) { b[LY::idx_bias(o)] = v * pre; });
        }
    }
    __syncthreads();
}

// ---- which models are decoded from a resident copy -----------------------------------------------
// A model is resident when its expanded weights and the staged copy of its packed record fit the LDS of one
// workgroup together; the host (launch sizes) and the kernels (which workgroups a launch serves) use this one rule.
constexpr uint32_t kLdsLimit = 160 * 1024;   // LDS per workgroup on gfx950
enum { kFitFp32 = 0,        // fp32 kernels: 4 bytes per padded weight
       kFitXdlOne = 1,      // split-precision kernels, one fp16 block per hidden layer (2..8-bit layers, or fp16 weights)
       kFitXdlTwo = 2 };    // ... two blocks per hidden layer (a store with fp32 or 16-bit hidden layers)
__host__ __device__ inline uint32_t fp32_model_bytes(uint32_t cls, uint32_t tile_rows_wide, uint32_t L) {
    const uint32_t wp = 16u * cls, tm = (cls == 2 || cls == 4) ? tile_rows_wide : 16u, g = 64u / tm;
    const uint32_t mt = wp / tm, mts = mt == 3 ? 4u : mt, ksteps = wp / g;
    const uint32_t first = 64u * mts, hidden = ksteps * 64u * mts;
    return 4u * (first + (L - 1) * wp + (L - 2) * hidden + 4u * wp + 4u);
}
__host__ __device__ inline uint32_t xdl_model_bytes(int cls, int n_layers, int n_int, int n_raw);
__host__ __device__ inline uint32_t resident_bytes(uint32_t form, uint32_t cls, uint32_t L, uint32_t tile_rows_wide) {
    const uint32_t b = form == kFitFp32 ? fp32_model_bytes(cls, tile_rows_wide, L)
                                        : xdl_model_bytes((int)cls, (int)L, form == kFitXdlOne ? (int)L - 2 : 0,
                                                          form == kFitXdlTwo ? (int)L - 2 : 0);
    return (b + 15u) & ~15u;
}
__host__ __device__ inline bool resident_fits(uint32_t form, uint32_t cls, uint32_t L, uint32_t rec_bytes, uint32_t tile_rows_wide,
                                              uint32_t budget) {
    return (uint64_t)resident_bytes(form, cls, L, tile_rows_wide) + rec_bytes <= budget;
}

// ---- decode kernel ---------------------------------------------------------------------------
struct DecodeArgs {
    const uint8_t *blob;
    const int64_t *ids;
    float *out_f32;               // may be NULL
    uint8_t *out_u8;              // may be NULL
    unsigned long long *status;   // sticky count of out-of-range ids
    uint64_t n_models;
    uint32_t HW, W;
    uint32_t wmagic, wshift;      // p / W == umulhi(p, wmagic) >> wshift for p < 2^31; wmagic == 0 means W == 1
    float inv2W, inv2H;           // 1/(2W), 1/(2H)
    float lo, span;               // coordinate = lo + span * (2k+1)/(2n)
    float pre;                    // w0 / (2 pi)
    uint32_t chunks;              // workgroups per slot
    uint32_t tiles_per_chunk;     // 64-pixel tiles per workgroup
    uint32_t lds_bytes;           // dynamic LDS of this launch; a resident model's packed record is staged at its end
    uint32_t cls;                 // width class this launch serves (padded width / 16); 0 = every class
    uint32_t stream_mode;         // 0: every model of the store is decoded from a resident expanded copy;
                                  // 1: this launch skips the models too deep for that; 2: this launch decodes only those,
                                  //    streaming their layers through LDS in groups
    uint32_t fit_form;            // how a model's resident size is reckoned (resident_fits)
    uint32_t tile_rows_wide;      // MFMA tile rows of the fp32 kernels at padded widths 32 and 64
    uint32_t lds_budget;          // LDS a workgroup may use (160 KB unless the store was opened with less)
    uint32_t no_clamp;
    uint32_t handle_bad;          // this launch zero-fills and counts out-of-range ids
    float neg1;                   // -1.0f, passed as data (keeps a subtraction in mixed-precision fma form)
    const float *affine;          // per-slot 2x3 map of the sampling grid, or NULL
    float ns[3], nb[3];           // per-channel scale / shift applied after the clamp when normalize != 0
    uint32_t normalize;
    const uint32_t *order;        // workgroups take the slots in this order (heaviest model first), or NULL = 0, 1, 2, ...
    uint32_t vec_store;           // H * W is a multiple of 4, the fp32 output 16-byte and the uint8 output 4-byte aligned:
                                  // a lane's consecutive pixels go out as one vector
};

// sin(2 pi r): the hardware sine takes its argument in revolutions and reduces the range
// itself (valid for |r| <= 256; pre-activations here are a few revolutions).  Measured
// max-abs error against fp64 on [-8, 8]: 1.25e-7, and an explicit fract first makes it
// worse (2.6e-7), so none is applied.
__device__ __forceinline__ float sin_rev(float r) {
    return __builtin_amdgcn_sinf(r);
}

// What one workgroup has to do: a range of 64-pixel tiles of one batch slot, and the slot's model.
struct Work {
    uint32_t slot, tile0, tile1;
    size_t plane0;               // element offset of the slot's first output plane
    IndexEntry e;
    uint32_t cls;                // width class of the model
};

// ---- slots ordered by the cost of their models, heaviest first: workgroups are started in grid order, so the long
// ones then start early and the grid's tail is made of short ones.  One workgroup: histogram of a cost key
// (layers x a per-width-class weight) in LDS, prefix from the heaviest key down, scatter.  The order inside a key
// is whatever the atomics give: it does not matter, every slot is decoded by the same code wherever it runs.
constexpr int kOrderKeys = 256;
__device__ __forceinline__ uint32_t order_key(const uint8_t *blob, uint64_t n_models, int64_t id) {
    if (id < 0 || (uint64_t)id >= n_models) return 0u;                       // zero-filled: the cheapest
    const IndexEntry e = *(const IndexEntry *)(blob + sizeof(StoreHeader) + (size_t)id * sizeof(IndexEntry));
    const uint32_t cls = e.width == 0 ? 1u : (e.width + 15u) >> 4;
    const uint32_t per_layer = cls == 1 ? 3u : (cls == 2 ? 6u : (cls == 3 ? 10u : 13u));     // measured cost of a sine layer per width class
    const uint32_t key = per_layer * e.n_layers;
    return key < (uint32_t)kOrderKeys ? key : (uint32_t)kOrderKeys - 1u;
}
__global__ __launch_bounds__(1024) void order_slots_kernel(const uint8_t *blob, uint64_t n_models, const int64_t *ids, uint32_t n,
                                                           uint32_t *order) {
    __shared__ uint32_t cursor[kOrderKeys];
    const uint32_t tid = threadIdx.x;
    if (tid < (uint32_t)kOrderKeys) cursor[tid] = 0u;
    __syncthreads();
    // four slots per thread and round, so that their id and index reads are in flight together
    for (uint32_t s0 = tid; s0 < n; s0 += 4096u) {
        uint32_t key[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) key[u] = s0 + 1024u * u < n ? order_key(blob, n_models, ids[s0 + 1024u * u]) : 0u;
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (s0 + 1024u * u < n) atomicAdd(&cursor[key[u]], 1u);
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t at = 0;
        for (int k = kOrderKeys - 1; k >= 0; --k) {
            const uint32_t c = cursor[k];
            cursor[k] = at;
            at += c;
        }
    }
    __syncthreads();
    for (uint32_t s0 = tid; s0 < n; s0 += 4096u) {
        uint32_t key[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) key[u] = s0 + 1024u * u < n ? order_key(blob, n_models, ids[s0 + 1024u * u]) : 0u;
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (s0 + 1024u * u < n) order[atomicAdd(&cursor[key[u]], 1u)] = s0 + 1024u * u;
    }
}

// ---- gather: workgroup -> (slot, tile range); slot -> id -> index entry (Sec. III-B batch select).
// Returns false when the workgroup has nothing to decode: empty tile range, or an out-of-range id
// (then the launch that handles bad ids has zero-filled the range and counted it), or a model of
// another class, or of the other kind (resident / streamed), than this launch serves.
__device__ __forceinline__ bool decode_prologue(const DecodeArgs &a, Work &w) {
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const uint32_t turn = blockIdx.x / a.chunks;
    const uint32_t chunk = blockIdx.x - turn * a.chunks;
    w.slot = a.order ? a.order[turn] : turn;
    w.tile0 = chunk * a.tiles_per_chunk;
    const uint32_t ntiles_img = (a.HW + 63) >> 6;
    if (w.tile0 >= ntiles_img) return false;
    w.tile1 = min(w.tile0 + a.tiles_per_chunk, ntiles_img);
    w.plane0 = (size_t)w.slot * 3 * a.HW;
    const int64_t id = a.ids[w.slot];
    if (id < 0 || (uint64_t)id >= a.n_models) {
        if (!a.handle_bad) return false;
        const uint32_t p0 = w.tile0 << 6, p1 = min(w.tile1 << 6, a.HW);
        for (int c = 0; c < 3; ++c)
            for (uint32_t p = p0 + tid; p < p1; p += nthreads) {
                if (a.out_f32) a.out_f32[w.plane0 + (size_t)c * a.HW + p] = 0.0f;
                if (a.out_u8) a.out_u8[w.plane0 + (size_t)c * a.HW + p] = 0;
            }
        if (chunk == 0 && tid == 0) atomicAdd(a.status, 1ull);
        return false;
    }
    w.e = *(const IndexEntry *)(a.blob + sizeof(StoreHeader) + (size_t)id * sizeof(IndexEntry));
    w.cls = w.e.width == 0 ? 1u : (w.e.width + 15u) >> 4;
    if (a.cls != 0 && w.cls != a.cls) return false;
    if (a.stream_mode) {
        const bool fits = resident_fits(a.fit_form, w.cls, w.e.n_layers, w.e.nbytes, a.tile_rows_wide, a.lds_budget);
        if (fits != (a.stream_mode == 1u)) return false;
    }
    return true;
}

// ---- the layers of the fp32 kernel, on one wavefront's 64-pixel tile ------------------------------------
// Activations live in Bv[pixel tile][k-step] between layers: the accumulator registers of one layer are the B
// operands of the next.  The weight pointers are per lane (lane * MTS added by the caller), bias tiles per group.
template <int TM, int WP> struct Fp32Tile {
    typedef Layout<TM, WP> LY;
    typedef Tile<TM> T;
    typedef typename T::acc_t acc_t;
    static constexpr int G = LY::G, RV = LY::RV, MT = LY::MT, MTS = LY::MTS, KSTEPS = LY::KSTEPS;
    static constexpr int NT = G;               // pixel tiles per wavefront: NT * TM = 64 pixels

    // coordinates of this lane's pixel in each of its NT tiles; lane group 0 feeds x, 1 feeds y
    static __device__ __forceinline__ void coords(const DecodeArgs &a, const float (&af)[6], uint32_t tile, int lane, float (&bx)[NT]) {
        const int g = lane / TM;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            uint32_t p = (tile << 6) + nt * TM + (lane % TM);
            p = min(p, a.HW - 1);
            const uint32_t row = a.wmagic ? (__umulhi(p, a.wmagic) >> a.wshift) : p, col = p - row * a.W;
            const float x = fmaf(a.span, (float)(2 * col + 1) * a.inv2W, a.lo);
            const float y = fmaf(a.span, (float)(2 * row + 1) * a.inv2H, a.lo);
            const float xa = fmaf(af[0], x, fmaf(af[1], y, af[2])), ya = fmaf(af[3], x, fmaf(af[4], y, af[5]));
            bx[nt] = g == 0 ? xa : (g == 1 ? ya : 0.0f);
        }
    }
    // first layer 2 -> width: one k-step, bias as the C operand, then the sine
    static __device__ __forceinline__ void first(float (&Bv)[NT][KSTEPS], const float *wfirst, const float *bt, const float (&bx)[NT]) {
        acc_t D[NT][MT];
        float a0[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) a0[mt] = wfirst[mt];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            acc_t c;
#pragma unroll
            for (int v = 0; v < RV; ++v) c[v] = bt[mt * G * RV + v];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) D[nt][mt] = T::mfma(a0[mt], bx[nt], c);
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int v = 0; v < RV; ++v) Bv[nt][mt * RV + v] = sin_rev(D[nt][mt][v]);
    }
    // hidden layer width -> width
    static __device__ __forceinline__ void hidden(float (&Bv)[NT][KSTEPS], const float *wl, const float *bt) {
        acc_t D[NT][MT];
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            float av[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) av[mt] = wl[s * 64 * MTS + mt];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                if (s == 0) {
                    acc_t c;
#pragma unroll
                    for (int v = 0; v < RV; ++v) c[v] = bt[mt * G * RV + v];
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) D[nt][mt] = T::mfma(av[mt], Bv[nt][0], c);
                } else {
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) D[nt][mt] = T::mfma(av[mt], Bv[nt][s], D[nt][mt]);
                }
            }
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int v = 0; v < RV; ++v) Bv[nt][mt * RV + v] = sin_rev(D[nt][mt][v]);
    }
    // output layer width -> 3 on the vector ALU (each lane sums over the rows it owns, then the G lane groups are
    // added together), clamp, optional normalisation, NCHW store: lane <-> pixel tile * 64 + lane
    static __device__ __forceinline__ void output(const DecodeArgs &a, const float (&Bv)[NT][KSTEPS], const float *wout, float ob0,
                                                  float ob1, float ob2, uint32_t tile, int lane, size_t plane0) {
        const int g = lane / TM;
        float o[NT][3];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) o[nt][0] = o[nt][1] = o[nt][2] = 0.0f;
#pragma unroll
        for (int r = 0; r < KSTEPS; ++r) {
            const f32x4 w4 = *(const f32x4 *)(wout + r * 4);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                o[nt][0] = fmaf(w4[0], Bv[nt][r], o[nt][0]);
                o[nt][1] = fmaf(w4[1], Bv[nt][r], o[nt][1]);
                o[nt][2] = fmaf(w4[2], Bv[nt][r], o[nt][2]);
            }
        }
#pragma unroll
        for (int d = TM; d < 64; d <<= 1)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int c = 0; c < 3; ++c) o[nt][c] += __shfl_xor(o[nt][c], d, 64);
        float r0 = o[0][0], r1 = o[0][1], r2 = o[0][2];
#pragma unroll
        for (int nt = 1; nt < NT; ++nt)
            if (g == nt) { r0 = o[nt][0]; r1 = o[nt][1]; r2 = o[nt][2]; }
        r0 += ob0; r1 += ob1; r2 += ob2;
        if (!a.no_clamp) {
            r0 = fminf(fmaxf(r0, 0.0f), 1.0f);
            r1 = fminf(fmaxf(r1, 0.0f), 1.0f);
            r2 = fminf(fmaxf(r2, 0.0f), 1.0f);
        }
        if (a.normalize) {
            r0 = fmaf(r0, a.ns[0], a.nb[0]);
            r1 = fmaf(r1, a.ns[1], a.nb[1]);
            r2 = fmaf(r2, a.ns[2], a.nb[2]);
        }
        const uint32_t p = (tile << 6) + lane;
        if (p < a.HW) {
            if (a.out_f32) {
                float *dst = a.out_f32 + plane0 + p;
                dst[0] = r0; dst[a.HW] = r1; dst[2 * (size_t)a.HW] = r2;
            }
            if (a.out_u8) {
                uint8_t *dst = a.out_u8 + plane0 + p;
                dst[0] = (uint8_t)rintf(255.0f * r0);
                dst[a.HW] = (uint8_t)rintf(255.0f * r1);
                dst[2 * (size_t)a.HW] = (uint8_t)rintf(255.0f * r2);
            }
        }
    }
};

// Resident form: the whole model is expanded once per workgroup and every tile runs through all layers.
template <int TM, int WP>
__device__ __forceinline__ void decode_body(const DecodeArgs &a, const Work &w, float *lds) {
    typedef Layout<TM, WP> LY;
    typedef Fp32Tile<TM, WP> FT;
    constexpr int RV = LY::RV, MTS = LY::MTS, KSTEPS = LY::KSTEPS, NT = FT::NT;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const uint32_t slot = w.slot, tile0 = w.tile0, tile1 = w.tile1;
    const size_t plane0 = w.plane0;
    const IndexEntry e = w.e;
    const int L = e.n_layers;

    // ---- stage the packed record at the end of the workgroup's LDS, expand it at the start
    uint32_t *stage = (uint32_t *)((char *)lds + (a.lds_bytes - e.nbytes));
    {
        const uint4 *src = (const uint4 *)(a.blob + e.off);
        uint4 *dst = (uint4 *)stage;
        for (uint32_t q = tid; q < (e.nbytes >> 4); q += nthreads) dst[q] = src[q];
    }
    expand_model<TM, WP>(lds, stage, L, a.pre, tid, nthreads);   // zero-fill barrier orders the staging too
    // Tiles are handed out through a counter in LDS (the first word of the staging area, dead by
    // now): wavefronts sharing a SIMD do not progress at the same rate.
    uint32_t *next_tile = stage;
    if (tid == 0) *next_tile = tile0 + (nthreads >> 6);
    __syncthreads();

    const int lane = tid & 63, wave = tid >> 6;
    const int g = lane / TM;
    const float *wfirst = lds + LY::off_first() + lane * MTS;
    const float *wout = lds + LY::off_out(L) + g * KSTEPS * 4;
    const float ob0 = lds[LY::off_outb(L) + 0], ob1 = lds[LY::off_outb(L) + 1], ob2 = lds[LY::off_outb(L) + 2];
    float af[6] = {1.0f, 0.0f, 0.0f, 0.0f, 1.0f, 0.0f};      // augmentation: this slot's map of the sampling grid
    if (a.affine)
        for (int q = 0; q < 6; ++q) af[q] = a.affine[(size_t)slot * 6 + q];

    for (uint32_t tile = tile0 + wave; tile < tile1;) {
        float Bv[NT][KSTEPS];
        float bx[NT];
        FT::coords(a, af, tile, lane, bx);
        FT::first(Bv, wfirst, lds + LY::off_bias(0) + g * RV, bx);
        for (int l = 1; l < L - 1; ++l)
            FT::hidden(Bv, lds + LY::off_hidden(L, l) + lane * MTS, lds + LY::off_bias(l) + g * RV);
        FT::output(a, Bv, wout, ob0, ob1, ob2, tile, lane, plane0);
        uint32_t nt_ = 0;
        if (lane == 0) nt_ = atomicAdd(next_tile, 1u);
        tile = __builtin_amdgcn_readfirstlane(nt_);
    }
}

// One layer into a slot of the streamed layout: the layer's weights in the resident layout's order at the slot's
// start, its bias tile HIDDEN floats in (the first and the output layer use less of the slot).
template <int TM, int WP>
__device__ __forceinline__ void expand_slot(float *wb, const uint32_t *rec, int L, int l, float pre, int lane, ExpandShare &sh) {
    typedef Layout<TM, WP> LY;
    const LayerRec r = *(const LayerRec *)(rec + l * (sizeof(LayerRec) / 4));
    float *bb = wb + LY::HIDDEN;
    if (l == L - 1)
        expand_layer(rec, r, lane, sh, [=](int o, int i, float v, int) { wb[LY::idx_out(o, i)] = v; },
                     [=](int o, float v) { bb[o] = v; });
    else if (l == 0)
        expand_layer(rec, r, lane, sh, [=](int o, int i, float v, int) { wb[LY::idx_first(o, i)] = v * pre; },
                     [=](int o, float v) { bb[LY::idx_bias(o)] = v * pre; });
    else
        expand_layer(rec, r, lane, sh, [=](int o, int i, float v, int) { wb[LY::idx_hidden(o, i)] = v * pre; },
                     [=](int o, float v) { bb[LY::idx_bias(o)] = v * pre; });
}

// Streamed form, for a model whose expanded weights do not fit LDS: the layers go through LDS in groups of as many
// as fit.  Every wavefront holds one tile's activations in registers; for each group the workgroup expands the
// group's layers straight from the packed record in global memory, then every wavefront takes its tile through
// them.  A slot is one layer's weights followed by its bias tile (the first and the output layer use less of it).
template <int TM, int WP>
__device__ __forceinline__ void decode_stream_body(const DecodeArgs &a, const Work &w, float *lds) {
    typedef Layout<TM, WP> LY;
    typedef Fp32Tile<TM, WP> FT;
    constexpr int RV = LY::RV, MTS = LY::MTS, KSTEPS = LY::KSTEPS, NT = FT::NT;
    constexpr int SLOT = LY::HIDDEN + WP;
    static_assert(LY::FIRST <= LY::HIDDEN && LY::OUTW + 4 <= SLOT, "slot size");
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = nthreads >> 6;
    const int g = lane / TM;
    const IndexEntry e = w.e;
    const int L = e.n_layers;
    const int K = (int)((a.lds_bytes >> 2) / (uint32_t)SLOT);        // layers per group; the host launches with room for one at least
    const uint32_t *rec = (const uint32_t *)(a.blob + e.off);
    const float pre = a.pre;
    float af[6] = {1.0f, 0.0f, 0.0f, 0.0f, 1.0f, 0.0f};
    if (a.affine)
        for (int q = 0; q < 6; ++q) af[q] = a.affine[(size_t)w.slot * 6 + q];

    for (uint32_t t0 = w.tile0; t0 < w.tile1; t0 += (uint32_t)nwaves) {
        const uint32_t tile = t0 + (uint32_t)wave;
        const bool active = tile < w.tile1;                            // the same for a whole wavefront
        float Bv[NT][KSTEPS];
        for (int l0 = 0; l0 < L; l0 += K) {
            const int l1 = l0 + K < L ? l0 + K : L;
            __syncthreads();                                           // every wavefront is done with the previous group
            for (int q = tid; q < (l1 - l0) * SLOT; q += nthreads) lds[q] = 0.0f;
            __syncthreads();
            ExpandShare sh = expand_share(rec, l0, l1, wave, nwaves);
            for (int l = l0; l < l1; ++l) expand_slot<TM, WP>(lds + (l - l0) * SLOT, rec, L, l, pre, lane, sh);
            __syncthreads();
            if (!active) continue;
            for (int l = l0; l < l1; ++l) {
                const float *wb = lds + (l - l0) * SLOT, *bb = wb + LY::HIDDEN;
                if (l == 0) {
                    float bx[NT];
                    FT::coords(a, af, tile, lane, bx);
                    FT::first(Bv, wb + lane * MTS, bb + g * RV, bx);
                } else if (l < L - 1) {
                    FT::hidden(Bv, wb + lane * MTS, bb + g * RV);
                } else {
                    FT::output(a, Bv, wb + g * KSTEPS * 4, bb[0], bb[1], bb[2], tile, lane, w.plane0);
                }
            }
        }
    }
}

// One width class per launch (a.cls != 0), or every class in one launch (a.cls == 0; TMW = MFMA
// tile rows for padded widths 32 and 64): a ragged batch then runs as one grid instead of one
// partly filled grid per class.
template <int TM, int WP, int NTHREADS>
__global__ __launch_bounds__(NTHREADS) void decode_kernel(const DecodeArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    Work w;
    if (!decode_prologue(a, w)) return;
    decode_body<TM, WP>(a, w, lds);
}

template <int TMW, int NTHREADS>
__global__ __launch_bounds__(NTHREADS) void decode_any_kernel(const DecodeArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    Work w;
    if (!decode_prologue(a, w)) return;
    switch (w.cls) {
        case 1: decode_body<16, 16>(a, w, lds); break;
        case 2: decode_body<TMW, 32>(a, w, lds); break;
        case 3: decode_body<16, 48>(a, w, lds); break;
        default: decode_body<TMW, 64>(a, w, lds); break;
    }
}

// The streamed form, one width class per launch, one wavefront per SIMD (the activations stay in registers
// across the expansion of the next group of layers).
constexpr int kStreamThreads = 256;
template <int TM, int WP>
__global__ __launch_bounds__(kStreamThreads) void decode_stream_kernel(const DecodeArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    Work w;
    if (!decode_prologue(a, w)) return;
    decode_stream_body<TM, WP>(a, w, lds);
}

// ---- debug export of the expand stage -----------------------------------------------------
// One layer, straight from the packed record in global memory into one slot (any depth fits), read back out of
// the layout the decode kernels use.
template <int TM, int WP>
__global__ __launch_bounds__(256) void dequant_debug_kernel(const uint8_t *blob, int64_t id, int layer, float *out, float *bias_out) {
    typedef Layout<TM, WP> LY;
    constexpr int SLOT = LY::HIDDEN + WP;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = nthreads >> 6;
    const IndexEntry e = *(const IndexEntry *)(blob + sizeof(StoreHeader) + (size_t)id * sizeof(IndexEntry));
    const int L = e.n_layers;
    const uint32_t *rec = (const uint32_t *)(blob + e.off);
    for (int q = tid; q < SLOT; q += nthreads) lds[q] = 0.0f;
    __syncthreads();
    ExpandShare sh = expand_share(rec, layer, layer + 1, wave, nwaves);
    expand_slot<TM, WP>(lds, rec, L, layer, 1.0f, lane, sh);
    __syncthreads();
    const LayerRec r = *(const LayerRec *)(rec + layer * (sizeof(LayerRec) / 4));
    const int n_in = r.n_in, cnt = r.n_in * r.n_out;
    for (int k = tid; k < cnt; k += nthreads) {
        const int o = k / n_in, i = k - o * n_in;
        float v;
        if (layer == L - 1) v = lds[LY::idx_out(o, i)];
        else if (layer == 0) v = lds[LY::idx_first(o, i)];
        else v = lds[LY::idx_hidden(o, i)];
        out[k] = v;
    }
    if (bias_out)
        for (int o = tid; o < r.n_out; o += nthreads)
            bias_out[o] = (layer == L - 1) ? lds[LY::HIDDEN + o] : lds[LY::HIDDEN + LY::idx_bias(o)];
}

}  // namespace rinr

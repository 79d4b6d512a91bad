// GPU side of the C ABI: store handle, launch logic for the decode kernels.
#include "../../include/rinr.h"
#include "rinr_kernels.hip.h"
#include "rinr_xdl.hip.h"
#include "rinr_validate.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

using namespace rinr;

namespace {

thread_local int g_last_hip = 0;
inline bool hip_fail(hipError_t e) {
    if (e == hipSuccess) return false;
    g_last_hip = (int)e;
    return true;
}
#define RINR_HIP(call) do { if (hip_fail(call)) return RINR_E_HIP; } while (0)

constexpr uint32_t kLdsLimit = 160 * 1024;   // LDS per workgroup on gfx950
constexpr int kThreads = 768;                // launch bound of the decode kernels: 12 wavefronts, 3 per SIMD, <= 168 VGPRs

// tuning knobs (see rinr_tune)
int g_tile_rows_wide = 32;      // MFMA tile for classes 2 and 4: 16 (16x16x4) or 32 (32x32x2)
int g_blocks_per_cu = 0;        // 0 = modelled split; else a fixed grid target in workgroups per CU
int g_threads = 0;              // 0 = choose by image size, else a multiple of 64 up to kThreads
int g_force_fp32 = 0;           // 1 = always use the fp32 MFMA kernel
int g_any_min_tiles = 64;       // stores that mix width classes: images of fewer 64-pixel tiles are decoded class by class

typedef void (*decode_fn)(const DecodeArgs);
typedef void (*debug_fn)(const uint8_t *, int64_t, int, uint32_t, float *, float *);

struct ClassImpl {
    decode_fn decode;      // fp32 MFMA kernel
    decode_fn decode_xdl[7];  // split-precision fp16 MFMA kernel, per kind of hidden layers (kHiddenAllInt, AllRaw, Mixed); + 3: fp16 activations; 6: all fp16
    debug_fn debug;
    int (*total)(int L);   // expanded floats for L layers (fp32 kernel)
};

template <int TM, int WP> int total_of(int L) { return Layout<TM, WP>::total(L); }
template <int TM, int WP> ClassImpl make_impl() {
    return ClassImpl{decode_kernel<TM, WP, kThreads>,
                     {decode_xdl_kernel<WP / 16, kThreads, kHiddenAllInt>, decode_xdl_kernel<WP / 16, kThreads, kHiddenAllRaw>,
                      decode_xdl_kernel<WP / 16, kThreads, kHiddenMixed>, decode_xdl_kernel<WP / 16, kThreads, kHiddenAllInt | kAct16>,
                      decode_xdl_kernel<WP / 16, kThreads, kHiddenAllRaw | kAct16>, decode_xdl_kernel<WP / 16, kThreads, kHiddenMixed | kAct16>,
                      decode_xdl_kernel<WP / 16, kThreads, kAct16 | kWeight16>},
                     dequant_debug_kernel<TM, WP>,
                     total_of<TM, WP>};
}

const void *xdl_any_fn(int kind, bool act16 = false, bool all16 = false) {
    if (all16) return (const void *)decode_xdl_any_kernel<kThreads, kAct16 | kWeight16>;
    if (act16) {
        switch (kind) {
            case kHiddenAllInt: return (const void *)decode_xdl_any_kernel<kThreads, kHiddenAllInt | kAct16>;
            case kHiddenAllRaw: return (const void *)decode_xdl_any_kernel<kThreads, kHiddenAllRaw | kAct16>;
            default: return (const void *)decode_xdl_any_kernel<kThreads, kHiddenMixed | kAct16>;
        }
    }
    switch (kind) {
        case kHiddenAllInt: return (const void *)decode_xdl_any_kernel<kThreads, kHiddenAllInt>;
        case kHiddenAllRaw: return (const void *)decode_xdl_any_kernel<kThreads, kHiddenAllRaw>;
        default: return (const void *)decode_xdl_any_kernel<kThreads, kHiddenMixed>;
    }
}

ClassImpl impl_for(uint32_t cls, int tile_rows_wide) {
    switch (cls) {
        case 1: return make_impl<16, 16>();
        case 2: return tile_rows_wide == 32 ? make_impl<32, 32>() : make_impl<16, 32>();
        case 3: return make_impl<16, 48>();
        default: return tile_rows_wide == 32 ? make_impl<32, 64>() : make_impl<16, 64>();
    }
}

// How many workgroups share one slot's pixels.  Every workgroup pays one expand of the model
// (not overlapped with compute when only one workgroup fits a CU), and a grid that does not
// fill the machine evenly ends in a tail, so both very many small workgroups and few large
// ones cost time.  Pick the split that minimises a simple model of both.
struct Plan { uint32_t chunks, tiles_per_chunk; };
Plan plan_chunks(double n_slots, uint32_t tiles, uint32_t nw, int n_cu, int resident, double tile_us) {
    const double expand_us = 15.0;
    if (n_slots < 1.0) n_slots = 1.0;
    Plan best{1, ((tiles + nw - 1) / nw) * nw};
    double best_t = 1e300;
    if (g_blocks_per_cu > 0) {      // experiment override: fixed target of workgroups per CU
        uint64_t want = (uint64_t)((double)g_blocks_per_cu * n_cu / n_slots + 0.999);
        uint32_t max_chunks = tiles / nw ? tiles / nw : 1;
        uint32_t chunks = (uint32_t)(want < 1 ? 1 : (want > max_chunks ? max_chunks : want));
        uint32_t tpc = (((tiles + chunks - 1) / chunks + nw - 1) / nw) * nw;
        return Plan{(tiles + tpc - 1) / tpc, tpc};
    }
    uint32_t last_tpc = 0;
    for (uint32_t c = 1; c <= tiles; ++c) {
        const uint32_t tpc = (((tiles + c - 1) / c + nw - 1) / nw) * nw;
        if (tpc == last_tpc) { if (tpc <= nw) break; continue; }
        last_tpc = tpc;
        const uint32_t cc = (tiles + tpc - 1) / tpc;
        const double blocks = n_slots * cc;
        double r_eff = blocks / n_cu;
        if (r_eff > resident) r_eff = resident;
        if (r_eff < 1.0) r_eff = 1.0;
        // a workgroup's duration with r_eff of them sharing a CU's four SIMDs; the expand hides behind
        // the other resident workgroups when there are any
        const double block_us = tpc * r_eff / 4.0 * tile_us + (r_eff > 1.5 ? expand_us / r_eff : expand_us);
        const double par = n_cu * r_eff;
        // all workgroups in flight at once: one duration; otherwise the work spread over the machine
        // plus, on average, half a workgroup of tail
        const double t = blocks <= par ? block_us : blocks * block_us / par + 0.5 * block_us;
        if (t < best_t * 0.95) { best_t = t; best = Plan{cc, tpc}; }     // finer splits must pay for their extra expands clearly
        if (tpc <= nw) break;
    }
    return best;
}

}  // namespace

struct rinr_store {
    const uint8_t *blob;
    size_t bytes;
    StoreSummary sum;
    unsigned long long *status;
    int device;
    int n_cu;
    int tile_rows_wide;                       // fixed at open so decode and debug agree
    uint32_t stage_off[kMaxClass + 1];        // floats
    uint32_t lds_bytes[kMaxClass + 1];
    std::vector<IndexEntry> index;            // host copy of the index (debug export, diagnostics)
    double class_tile_us[kMaxClass + 1];      // modelled time of one 64-pixel tile on one SIMD
    double class_tile_us_xdl[kMaxClass + 1];
    bool xdl_ok;                              // every weight fits fp16 range after pre-scaling, and the models fit LDS
    int hidden_kind;                          // kHiddenAllInt / AllRaw / Mixed over all hidden layers of all models
    bool even_cost;                           // every model has the same width class and depth: slot order does not matter
    bool fp32_ok;                             // the fp32 kernels' expanded models fit LDS
    uint32_t xdl_stage_off[kMaxClass + 1];    // floats
    uint32_t xdl_lds_bytes[kMaxClass + 1];
    // launch plan of the last (n, H*W, threads, knob) combination, reused while they repeat
    mutable int64_t plan_hw;
    mutable int32_t plan_n, plan_threads, plan_knob;
    mutable Plan plan[kMaxClass + 1];
    mutable int32_t last_info[4];
};

extern "C" int rinr_tune(int knob, int value) {
    switch (knob) {
        case 0: if (value != 16 && value != 32) return RINR_E_ARG; g_tile_rows_wide = value; return RINR_OK;
        case 1: if (value < 0 || value > 1024) return RINR_E_ARG; g_blocks_per_cu = value; return RINR_OK;
        case 2: if (value != 0 && (value % 64 || value < 64 || value > kThreads)) return RINR_E_ARG; g_threads = value; return RINR_OK;
        case 3: if (value != 0 && value != 1) return RINR_E_ARG; g_force_fp32 = value; return RINR_OK;
        case 4: if (value < 0) return RINR_E_ARG; g_any_min_tiles = value; return RINR_OK;
        default: return RINR_E_ARG;
    }
}

extern "C" int rinr_last_hip_error(void) { return g_last_hip; }

extern "C" int rinr_store_open(const void *device_blob, const void *host_blob, size_t bytes, rinr_store **store) {
    if (!device_blob || !store) return RINR_E_NULL;
    *store = nullptr;
    if ((uintptr_t)device_blob & 15) return RINR_E_ALIGN;
    if (bytes < sizeof(StoreHeader)) return RINR_E_FORMAT;
    std::vector<uint8_t> copy;
    if (!host_blob) {
        copy.resize(bytes);
        RINR_HIP(hipMemcpy(copy.data(), device_blob, bytes, hipMemcpyDeviceToHost));
        host_blob = copy.data();
    }
    StoreSummary sum;
    if (int rc = validate_blob(host_blob, bytes, &sum)) return rc;
    rinr_store *s = new (std::nothrow) rinr_store();
    if (!s) return RINR_E_SIZE;
    s->blob = (const uint8_t *)device_blob;
    s->bytes = bytes;
    s->sum = sum;
    s->tile_rows_wide = g_tile_rows_wide;
    s->index.resize((size_t)sum.header.n_models);
    if (sum.header.n_models)
        std::memcpy(s->index.data(), (const uint8_t *)host_blob + sizeof(StoreHeader),
                    (size_t)sum.header.n_models * sizeof(IndexEntry));
    std::memset(s->last_info, 0, sizeof s->last_info);
    s->plan_hw = -1; s->plan_n = -1; s->plan_threads = -1; s->plan_knob = -1;
    s->even_cost = true;
    {   // mean matrix work per pixel of each class -> time of a 64-pixel tile on one SIMD's MFMA pipe
        double macs[kMaxClass + 1] = {0, 0, 0, 0, 0};
        for (const IndexEntry &e : s->index) {
            const uint32_t c = e.width == 0 ? 1u : (e.width + 15u) >> 4;
            const IndexEntry &f = s->index[0];
            if (e.n_layers != f.n_layers || c != (f.width == 0 ? 1u : (f.width + 15u) >> 4)) s->even_cost = false;
            const double wp = 16.0 * c;
            macs[c] += wp * (4.0 + (e.n_layers - 2) * wp);
        }
        for (uint32_t c = 1; c <= kMaxClass; ++c) {
            const double mean = sum.class_count[c] ? macs[c] / (double)sum.class_count[c] : 0.0;
            // 32 MACs per clock per SIMD at 2.4 GHz, ~87 % of it reachable next to the sine work
            s->class_tile_us[c] = 64.0 * mean / (32.0 * 2400.0 * 0.87) + 0.5;
        }
    }
    {   // split-precision kernel: LDS need per class and fp16 range of every operand it would build
        const uint8_t *hb = (const uint8_t *)host_blob;
        const float pre = (float)((double)sum.header.w0 / (2.0 * M_PI));
        uint32_t need[kMaxClass + 1] = {0, 0, 0, 0, 0};
        double acts[kMaxClass + 1] = {0, 0, 0, 0, 0};
        s->xdl_ok = std::fabs(sum.header.coord_lo) < 60000.0f && std::fabs(sum.header.coord_hi) < 60000.0f;   // coordinates travel as fp16 hi+lo
        int64_t tot_int = 0, tot_raw = 0;
        for (const IndexEntry &e : s->index) {
            const uint32_t c = e.width == 0 ? 1u : (e.width + 15u) >> 4;
            int n_int = 0, n_raw = 0;
            for (int l = 0; l < e.n_layers; ++l) {
                LayerRec r;
                std::memcpy(&r, hb + e.off + (size_t)l * sizeof(LayerRec), sizeof r);
                const bool hidden = l > 0 && l < e.n_layers - 1;
                const float k = l < e.n_layers - 1 ? pre : 1.0f;
                if (hidden && xdl_int_layer(r.bits, r.scale * pre)) { ++n_int; continue; }
                if (hidden) ++n_raw;
                float wmax = 0.0f;
                if (r.bits == 0) {
                    const float *w = (const float *)(hb + e.off + r.code_off);
                    for (uint32_t q = 0; q < r.n_kept; ++q) wmax = std::fmax(wmax, std::fabs(w[q]));
                } else {
                    const float span = (float)std::max<int64_t>(r.zp, ((int64_t)1 << r.bits) - 1 - r.zp);
                    wmax = std::fabs(r.scale) * span;
                }
                if (!(wmax * std::fabs(k) < 60000.0f)) s->xdl_ok = false;
            }
            tot_int += n_int;
            tot_raw += n_raw;
            const uint32_t b = xdl_model_bytes((int)c, e.n_layers, n_int, n_raw);
            if (b > need[c]) need[c] = b;
            acts[c] += (e.n_layers - 1) * 16.0 * c;
        }
        s->hidden_kind = tot_raw == 0 ? kHiddenAllInt : (tot_int == 0 ? kHiddenAllRaw : kHiddenMixed);
        for (uint32_t c = 1; c <= kMaxClass; ++c) {
            s->xdl_stage_off[c] = need[c] / 4;
            s->xdl_lds_bytes[c] = need[c] + sum.class_max_bytes[c];
            if (sum.class_count[c] && s->xdl_lds_bytes[c] > kLdsLimit) s->xdl_ok = false;
            // vector-ALU bound: ~20 clocks per activation per lane (sine + hi/lo split), 64 lanes = 64 pixels
            const double mean = sum.class_count[c] ? acts[c] / (double)sum.class_count[c] : 0.0;
            s->class_tile_us_xdl[c] = (mean * 20.0 + 600.0) / 2400.0;
        }
    }
    s->fp32_ok = true;
    for (uint32_t c = 1; c <= kMaxClass; ++c) {
        s->stage_off[c] = s->lds_bytes[c] = 0;
        if (!sum.class_count[c]) continue;
        if (sum.class_max_layers[c] < 2) { delete s; return RINR_E_UNSUPPORTED; }
        const ClassImpl im = impl_for(c, s->tile_rows_wide);
        const uint32_t tot = ((uint32_t)im.total((int)sum.class_max_layers[c]) + 3u) & ~3u;
        const uint64_t need = (uint64_t)tot * 4 + sum.class_max_bytes[c];
        if (need > kLdsLimit) s->fp32_ok = false;      // fp32 weights are twice the size of the split-precision operands
        s->stage_off[c] = tot;
        s->lds_bytes[c] = (uint32_t)need;
        if (hip_fail(hipFuncSetAttribute((const void *)im.decode, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
            hip_fail(hipFuncSetAttribute((const void *)im.decode_xdl[0], hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
            hip_fail(hipFuncSetAttribute((const void *)im.decode_xdl[1], hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
            hip_fail(hipFuncSetAttribute((const void *)im.decode_xdl[2], hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
            hip_fail(hipFuncSetAttribute((const void *)im.decode_xdl[3], hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
            hip_fail(hipFuncSetAttribute((const void *)im.decode_xdl[4], hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
            hip_fail(hipFuncSetAttribute((const void *)im.decode_xdl[5], hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
            hip_fail(hipFuncSetAttribute((const void *)im.decode_xdl[6], hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
            hip_fail(hipFuncSetAttribute((const void *)im.debug, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit))) {
            delete s;
            return RINR_E_HIP;
        }
    }
    if (!s->fp32_ok && !s->xdl_ok) { delete s; return RINR_E_UNSUPPORTED; }     // too deep for LDS in either form
    if (hip_fail(hipFuncSetAttribute(xdl_any_fn(kHiddenAllInt), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
        hip_fail(hipFuncSetAttribute(xdl_any_fn(kHiddenAllRaw), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
        hip_fail(hipFuncSetAttribute(xdl_any_fn(kHiddenMixed), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
        hip_fail(hipFuncSetAttribute(xdl_any_fn(kHiddenAllInt, true), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
        hip_fail(hipFuncSetAttribute(xdl_any_fn(kHiddenAllRaw, true), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
        hip_fail(hipFuncSetAttribute(xdl_any_fn(kHiddenMixed, true), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
        hip_fail(hipFuncSetAttribute(xdl_any_fn(0, true, true), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
        hip_fail(hipFuncSetAttribute((const void *)decode_any_kernel<16, kThreads>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
        hip_fail(hipFuncSetAttribute((const void *)decode_any_kernel<32, kThreads>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit))) {
        delete s;
        return RINR_E_HIP;
    }
    if (hip_fail(hipGetDevice(&s->device))) { delete s; return RINR_E_HIP; }
    hipDeviceProp_t prop;
    if (hip_fail(hipGetDeviceProperties(&prop, s->device))) { delete s; return RINR_E_HIP; }
    s->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    if (hip_fail(hipMalloc((void **)&s->status, sizeof(unsigned long long)))) { delete s; return RINR_E_HIP; }
    if (hip_fail(hipMemset(s->status, 0, sizeof(unsigned long long)))) {
        (void)hipFree(s->status);
        delete s;
        return RINR_E_HIP;
    }
    *store = s;
    return RINR_OK;
}

extern "C" int rinr_store_close(rinr_store *s) {
    if (!s) return RINR_E_NULL;
    int rc = RINR_OK;
    if (s->status && hip_fail(hipFree(s->status))) rc = RINR_E_HIP;
    delete s;
    return rc;
}

extern "C" int rinr_store_info(const rinr_store *s, int64_t *n_models, int32_t *max_width, int32_t *max_layers) {
    if (!s) return RINR_E_NULL;
    if (n_models) *n_models = (int64_t)s->sum.header.n_models;
    if (max_width) *max_width = (int32_t)s->sum.header.max_width;
    if (max_layers) *max_layers = (int32_t)s->sum.header.max_layers;
    return RINR_OK;
}

namespace {
hipError_t order_slots(const rinr_store *s, const int64_t *image_ids, int32_t n, void *workspace, void *stream) {
    hipLaunchKernelGGL(order_slots_kernel, dim3(1), dim3(1024), 0, (hipStream_t)stream, s->blob, (uint64_t)s->sum.header.n_models,
                       image_ids, (uint32_t)n, (uint32_t *)workspace);
    return hipGetLastError();
}
}  // namespace

extern "C" size_t rinr_decode_workspace_bytes(int32_t n) { return n > 0 ? ((size_t)n * 4 + 15) & ~(size_t)15 : 0; }

extern "C" int rinr_decode_batch_ex(const rinr_store *s, const int64_t *image_ids, int32_t n, int32_t H, int32_t W,
                                    void *out, const rinr_decode_opts *opts, void *stream) {
    if (!s || !opts) return RINR_E_NULL;
    if (n < 0 || H <= 0 || W <= 0) return RINR_E_ARG;
    const int dt = opts->out_dtype;
    if (dt != RINR_OUT_F32 && dt != RINR_OUT_U8 && dt != RINR_OUT_F32_AND_U8) return RINR_E_ARG;
    if (opts->flags & ~(RINR_FLAG_NO_CLAMP | RINR_FLAG_FP32_MFMA | RINR_FLAG_NORMALIZE | RINR_FLAG_FP16_ACT | RINR_FLAG_FP16_ALL)) return RINR_E_ARG;
    if ((opts->flags & RINR_FLAG_NORMALIZE) && dt != RINR_OUT_F32) return RINR_E_ARG;
    if (opts->flags & RINR_FLAG_NORMALIZE)
        for (int c = 0; c < 3; ++c)
            if (!std::isfinite(opts->norm_scale[c]) || !std::isfinite(opts->norm_shift[c])) return RINR_E_ARG;
    if ((opts->flags & RINR_FLAG_NO_CLAMP) && dt != RINR_OUT_F32) return RINR_E_ARG;
    const int64_t HW = (int64_t)H * W;
    if (3 * HW >= (int64_t)1 << 32) return RINR_E_SIZE;     // element offsets inside a slot's three planes are 32-bit
    if (n > 0 && HW > INT64_MAX / 3 / n / 4) return RINR_E_SIZE;
    if (n == 0) { std::memset(s->last_info, 0, sizeof s->last_info); return RINR_OK; }
    if (!image_ids || !out) return RINR_E_NULL;
    if (dt == RINR_OUT_F32_AND_U8 && !opts->out_u8) return RINR_E_NULL;
    if (dt != RINR_OUT_U8 && ((uintptr_t)out & 3)) return RINR_E_ALIGN;
    if ((uintptr_t)image_ids & 7) return RINR_E_ALIGN;
    if ((uintptr_t)opts->affine & 3) return RINR_E_ALIGN;
    if ((uintptr_t)opts->workspace & 3) return RINR_E_ALIGN;
    if (opts->workspace && opts->workspace_bytes < rinr_decode_workspace_bytes(n)) return RINR_E_SIZE;

    const StoreHeader &h = s->sum.header;
    DecodeArgs a;
    std::memset(&a, 0, sizeof a);
    a.blob = s->blob;
    a.ids = image_ids;
    a.out_f32 = dt == RINR_OUT_U8 ? nullptr : (float *)out;
    a.out_u8 = dt == RINR_OUT_U8 ? (uint8_t *)out : (dt == RINR_OUT_F32_AND_U8 ? (uint8_t *)opts->out_u8 : nullptr);
    a.status = s->status;
    a.n_models = h.n_models;
    a.HW = (uint32_t)HW;
    a.W = (uint32_t)W;
    {   // exact division of a pixel index (< 2^31) by W as a multiply-high and a shift
        uint32_t l = 0;
        while ((1ull << l) < (uint64_t)W) ++l;
        a.wmagic = l ? (uint32_t)((((uint64_t)1 << (31 + l)) + (uint64_t)W - 1) / (uint64_t)W) : 0u;
        a.wshift = l ? l - 1 : 0u;
    }
    a.inv2W = (float)(1.0 / (2.0 * W));
    a.inv2H = (float)(1.0 / (2.0 * H));
    a.lo = h.coord_lo;
    a.span = h.coord_hi - h.coord_lo;
    a.pre = (float)((double)h.w0 / (2.0 * M_PI));
    a.no_clamp = (opts->flags & RINR_FLAG_NO_CLAMP) ? 1u : 0u;
    a.neg1 = -1.0f;
    a.affine = opts->affine;
    a.normalize = (opts->flags & RINR_FLAG_NORMALIZE) ? 1u : 0u;
    for (int c = 0; c < 3; ++c) {
        a.ns[c] = a.normalize ? opts->norm_scale[c] : 1.0f;
        a.nb[c] = a.normalize ? opts->norm_shift[c] : 0.0f;
    }
    const bool want_fp32 = (opts->flags & RINR_FLAG_FP32_MFMA) || g_force_fp32;
    if (want_fp32 && !s->fp32_ok) return RINR_E_UNSUPPORTED;
    const bool xdl = s->xdl_ok && !want_fp32;
    const bool all16 = xdl && (opts->flags & RINR_FLAG_FP16_ALL);
    const bool act16 = xdl && (opts->flags & (RINR_FLAG_FP16_ACT | RINR_FLAG_FP16_ALL));
    const int xk = all16 ? 6 : s->hidden_kind + (act16 ? 3 : 0);      // index into ClassImpl::decode_xdl

    const uint32_t tiles = (uint32_t)((HW + 63) >> 6);
    const int threads = g_threads ? g_threads : (tiles >= 96 ? 768 : (tiles >= 64 ? 512 : 256));
    const uint32_t nw = (uint32_t)threads / 64;

    int n_classes = 0;
    for (uint32_t c = 1; c <= kMaxClass; ++c) n_classes += s->sum.class_count[c] ? 1 : 0;
    // a store that mixes width classes: one grid whose workgroups run the body of their slot's class, or, for images of
    // few tiles, one launch per class with that class's LDS size (workgroups of other classes return at once)
    // (an empty store also takes the one grid: every id is out of range and its slot is zero-filled)
    const bool one_grid = n_classes == 0 || (n_classes > 1 && (int64_t)tiles >= (int64_t)g_any_min_tiles);
    const int knob = g_blocks_per_cu * 16 + (xdl ? 1 : 0) + (act16 ? 2 : 0) + (all16 ? 4 : 0) + (one_grid ? 8 : 0);
    const bool replan = !(s->plan_hw == HW && s->plan_n == n && s->plan_threads == threads && s->plan_knob == knob);
    for (uint32_t c = 1; c <= kMaxClass; ++c) a.stage_off[c] = xdl ? s->xdl_stage_off[c] : s->stage_off[c];

    // slots of unequal cost are taken heaviest first when the caller gives the scratch for the order
    const bool order = opts->workspace && !s->even_cost;
    if (order) a.order = (const uint32_t *)opts->workspace;
    int launches = 0;
    uint32_t big_lds = 0, total_blocks = 0;
    if (one_grid) {
        // ragged store: one grid over all slots, each workgroup runs the body of its slot's class
        // (an empty store also comes here: every id is out of range and its slot is zero-filled)
        const void *fn = xdl ? xdl_any_fn(s->hidden_kind, act16, all16)
                             : (s->tile_rows_wide == 32 ? (const void *)decode_any_kernel<32, kThreads>
                                                        : (const void *)decode_any_kernel<16, kThreads>);
        uint32_t lds_bytes = 0;
        double tile_us = 0.0;
        for (uint32_t c = 1; c <= kMaxClass; ++c) {
            if (!s->sum.class_count[c]) continue;
            lds_bytes = std::max(lds_bytes, xdl ? s->xdl_lds_bytes[c] : s->lds_bytes[c]);
            tile_us += (xdl ? s->class_tile_us_xdl[c] : s->class_tile_us[c]) * (double)s->sum.class_count[c] /
                       (double)h.n_models;
        }
        if (replan) {
            int resident = 1;
            if (hip_fail(hipOccupancyMaxActiveBlocksPerMultiprocessor(&resident, fn, threads, lds_bytes)) || resident < 1)
                resident = 1;
            s->plan[0] = plan_chunks((double)n, tiles, nw, s->n_cu, resident, tile_us);
        }
        const Plan pl = s->plan[0];
        if ((uint64_t)n * pl.chunks > 0x7FFFFFFFull) return RINR_E_SIZE;
        a.chunks = pl.chunks;
        a.tiles_per_chunk = pl.tiles_per_chunk;
        a.cls = 0;
        a.handle_bad = 1u;
        if (order) RINR_HIP(order_slots(s, image_ids, n, opts->workspace, stream));
        void *kargs[] = {(void *)&a};
        RINR_HIP(hipLaunchKernel(fn, dim3((uint32_t)n * pl.chunks), dim3((uint32_t)threads), kargs, lds_bytes,
                                 (hipStream_t)stream));
        launches = order ? 2 : 1;
        total_blocks = (uint32_t)n * pl.chunks;
        big_lds = lds_bytes;
    } else {
        for (uint32_t c = 1; c <= kMaxClass; ++c) {
            if (!s->sum.class_count[c]) continue;
            const ClassImpl im = impl_for(c, s->tile_rows_wide);
            const uint32_t lds_bytes = xdl ? s->xdl_lds_bytes[c] : s->lds_bytes[c];
            if (replan) {
                int resident = 1;
                if (hip_fail(hipOccupancyMaxActiveBlocksPerMultiprocessor(&resident, (const void *)(xdl ? im.decode_xdl[xk] : im.decode),
                                                                          threads, lds_bytes)) || resident < 1)
                    resident = 1;
                s->plan[c] = plan_chunks((double)n, tiles, nw, s->n_cu, resident, xdl ? s->class_tile_us_xdl[c] : s->class_tile_us[c]);
            }
            const Plan pl = s->plan[c];
            if ((uint64_t)n * pl.chunks > 0x7FFFFFFFull) return RINR_E_SIZE;
            a.chunks = pl.chunks;
            a.tiles_per_chunk = pl.tiles_per_chunk;
            a.cls = c;
            a.handle_bad = launches == 0 ? 1u : 0u;       // the first launch zero-fills and counts the out-of-range ids
            if (order && launches == 0) RINR_HIP(order_slots(s, image_ids, n, opts->workspace, stream));
            hipLaunchKernelGGL(xdl ? im.decode_xdl[xk] : im.decode, dim3((uint32_t)n * pl.chunks), dim3((uint32_t)threads), lds_bytes,
                               (hipStream_t)stream, a);
            RINR_HIP(hipGetLastError());
            launches += (order && launches == 0) ? 2 : 1;
            total_blocks = (uint32_t)n * pl.chunks;
            big_lds = lds_bytes;
        }
    }
    s->plan_hw = HW; s->plan_n = n; s->plan_threads = threads; s->plan_knob = knob;
    s->last_info[0] = launches;
    s->last_info[1] = (int32_t)total_blocks;
    s->last_info[2] = threads;
    s->last_info[3] = (int32_t)big_lds;
    return RINR_OK;
}

extern "C" int rinr_decode_batch(const rinr_store *s, const int64_t *image_ids, int32_t n, int32_t H, int32_t W,
                                 void *out, void *stream) {
    rinr_decode_opts o;
    std::memset(&o, 0, sizeof o);
    o.out_dtype = RINR_OUT_F32;
    return rinr_decode_batch_ex(s, image_ids, n, H, W, out, &o, stream);
}

extern "C" int rinr_store_status(const rinr_store *s, int64_t *bad_id_count, void *stream) {
    if (!s || !bad_id_count) return RINR_E_NULL;
    RINR_HIP(hipStreamSynchronize((hipStream_t)stream));
    unsigned long long v = 0;
    RINR_HIP(hipMemcpy(&v, s->status, sizeof v, hipMemcpyDeviceToHost));
    *bad_id_count = (int64_t)v;
    return RINR_OK;
}

extern "C" int rinr_debug_dequant(const rinr_store *s, int64_t id, int32_t layer, float *device_out, float *bias_out,
                                  void *stream) {
    if (!s || !device_out) return RINR_E_NULL;
    if (id < 0 || (uint64_t)id >= s->sum.header.n_models) return RINR_E_ARG;
    const IndexEntry &e = s->index[(size_t)id];
    if (layer < 0 || layer >= e.n_layers) return RINR_E_ARG;
    const uint32_t cls = e.width == 0 ? 1u : (e.width + 15u) >> 4;
    if (cls > kMaxClass || !s->sum.class_count[cls]) return RINR_E_FORMAT;
    if (!s->fp32_ok) return RINR_E_UNSUPPORTED;      // the export reads the fp32 kernels' layout
    const ClassImpl im = impl_for(cls, s->tile_rows_wide);
    hipLaunchKernelGGL(im.debug, dim3(1), dim3(256), s->lds_bytes[cls], (hipStream_t)stream, s->blob, id, (int)layer,
                       s->stage_off[cls], device_out, bias_out);
    RINR_HIP(hipGetLastError());
    return RINR_OK;
}

extern "C" int rinr_last_launch_info(const rinr_store *s, int32_t info[4]) {
    if (!s || !info) return RINR_E_NULL;
    std::memcpy(info, s->last_info, sizeof s->last_info);
    return RINR_OK;
}

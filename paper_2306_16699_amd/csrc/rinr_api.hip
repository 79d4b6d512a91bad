// GPU side of the C ABI: store handle, launch logic for the decode kernels.
#include "../../include/rinr.h"
#include "rinr_kernels.hip.h"
#include "rinr_xdl.hip.h"
#include "rinr_validate.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
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

constexpr int kThreads = 768;                // launch bound of the resident decode kernels: 12 wavefronts, 3 per SIMD, <= 168 VGPRs
constexpr double kBoundLimit = 9.5e-4;       // a reduced-precision mode is used where its a-priori error bound is at most this

typedef void (*decode_fn)(const DecodeArgs);
typedef void (*debug_fn)(const uint8_t *, int64_t, int, float *, float *);
typedef void (*xdebug_fn)(const uint8_t *, int64_t, int, uint32_t, float *, float *, float *, float *);

// Kernel families a decode can run; also the value of rinr_last_launch_info's info[4].
enum { kFamSplit = 0, kFamFp32 = 1, kFamAct16 = 2, kFamAll16 = 3 };

struct ClassImpl {
    decode_fn decode;         // fp32 MFMA kernel
    decode_fn decode_xdl[7];  // split-precision fp16 MFMA kernel, per kind of hidden layers (kHiddenAllInt, AllRaw, Mixed); + 3: fp16 activations; 6: all fp16
    decode_fn stream;         // fp32 MFMA kernel, layers streamed through LDS
    decode_fn stream_xdl[3];  // split-precision kernel, layers streamed: hi+lo activations, fp16 activations, all fp16
    debug_fn debug;
    xdebug_fn xdebug[2];      // split-precision operand export: as stored / fp16 weights
    uint32_t slot_bytes;      // fp32 kernels: LDS of one layer in the streamed layout
    uint32_t xslot_bytes;     // split-precision kernels: LDS of one layer in the streamed layout
    uint32_t xtable_bytes;
};

template <int TM, int WP> ClassImpl make_impl() {
    constexpr int CLS = WP / 16, XTM = xdl_tile_rows(CLS);
    return ClassImpl{decode_kernel<TM, WP, kThreads>,
                     {decode_xdl_kernel<CLS, kThreads, kHiddenAllInt>, decode_xdl_kernel<CLS, kThreads, kHiddenAllRaw>,
                      decode_xdl_kernel<CLS, kThreads, kHiddenMixed>, decode_xdl_kernel<CLS, kThreads, kHiddenAllInt | kAct16>,
                      decode_xdl_kernel<CLS, kThreads, kHiddenAllRaw | kAct16>, decode_xdl_kernel<CLS, kThreads, kHiddenMixed | kAct16>,
                      decode_xdl_kernel<CLS, kThreads, kAct16 | kWeight16>},
                     decode_stream_kernel<TM, WP>,
                     {decode_xdl_stream_kernel<CLS, 0>, decode_xdl_stream_kernel<CLS, kAct16>, decode_xdl_stream_kernel<CLS, kAct16 | kWeight16>},
                     dequant_debug_kernel<TM, WP>,
                     {xdl_debug_kernel<XTM, WP, false>, xdl_debug_kernel<XTM, WP, true>},
                     (uint32_t)(Layout<TM, WP>::HIDDEN + WP) * 4u,
                     (uint32_t)XSlot<XTM, WP>::BYTES,
                     (uint32_t)XLayout<XTM, WP>::TABLE};
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

bool allow_full_lds(const void *fn) {
    return !hip_fail(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit));
}

// How many workgroups share one slot's pixels.  Every workgroup pays one expand of the model
// (not overlapped with compute when only one workgroup fits a CU), and a grid that does not
// fill the machine evenly ends in a tail, so both very many small workgroups and few large
// ones cost time.  Pick the split that minimises a simple model of both.
struct Plan { uint32_t chunks, tiles_per_chunk; };
Plan plan_chunks(double n_slots, uint32_t tiles, uint32_t nw, int n_cu, int resident, double tile_us, int blocks_per_cu) {
    const double expand_us = 15.0;
    if (n_slots < 1.0) n_slots = 1.0;
    Plan best{1, ((tiles + nw - 1) / nw) * nw};
    double best_t = 1e300;
    if (blocks_per_cu > 0) {      // experiment override: fixed target of workgroups per CU
        uint64_t want = (uint64_t)((double)blocks_per_cu * n_cu / n_slots + 0.999);
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

// Scratch of rinr_decode_batch_noalloc: the heaviest-first slot order, 4 bytes per slot.  Every GPU the library runs
// on holds its own copy of the array at its own address, found once per device (with that device current) when the
// first store is opened on it.  In host code the array's name is only a stand-in for the symbol: kernels and copies
// get the looked-up address.
__device__ __align__(256) uint32_t scratch[RINR_NOALLOC_MAX_SLOTS];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
uint32_t *g_scratch_ptr[kMaxDevices];       // per device; nullptr = not looked up yet

int scratch_for_device(int device, uint32_t **out) {
    if (device < 0 || device >= kMaxDevices) return RINR_E_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        if (hip_fail(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) || !p) return RINR_E_HIP;
        g_scratch_ptr[device] = (uint32_t *)p;
    }
    *out = g_scratch_ptr[device];
    return RINR_OK;
}

// The three ways a model's resident size is reckoned (see resident_fits): fp32 kernels, split-precision kernels
// with the store's own kinds of hidden layer, split-precision kernels with fp16 weights.
enum { kSizeFp32 = 0, kSizeXdl = 1, kSizeXdl16 = 2, kSizes = 3 };

}  // namespace

struct rinr_store {
    const uint8_t *blob;
    size_t bytes;
    StoreSummary sum;
    unsigned long long *status;
    uint32_t *scratch;                        // this device's copy of the static scratch array
    int device;
    int n_cu;
    int tile_rows_wide;                       // fixed at open so decode and debug agree
    uint32_t lds_budget;                      // LDS a workgroup may use
    std::vector<IndexEntry> index;            // host copy of the index (debug export, diagnostics)
    double class_tile_us[kMaxClass + 1];      // modelled time of one 64-pixel tile on one SIMD
    double class_tile_us_xdl[kMaxClass + 1];
    bool xdl_ok;                              // every operand fits fp16 range after pre-scaling
    int hidden_kind;                          // kHiddenAllInt / AllRaw / Mixed over all hidden layers of all models
    bool even_cost;                           // every model has the same width class and depth: slot order does not matter
    uint32_t fit_form[kSizes];                // resident_fits form per way of sizing
    uint32_t res_lds[kSizes][kMaxClass + 1];  // LDS of a resident launch: largest expanded model + its record, over the models that fit
    uint64_t n_res[kSizes][kMaxClass + 1];    // models decoded from a resident copy
    uint64_t n_str[kSizes][kMaxClass + 1];    // models whose layers are streamed
    uint32_t str_layers[kSizes][kMaxClass + 1];   // deepest streamed model
    double bounds[2];                         // a-priori error bounds of the fp16-activation and the all-fp16 mode
    // launch plan of the last (n, H*W, threads, knobs) combination, reused while they repeat
    int64_t plan_hw;
    int32_t plan_n, plan_threads, plan_knob;
    Plan plan[kMaxClass + 1];
    int32_t last_info[6];
};

extern "C" int rinr_last_hip_error(void) { return g_last_hip; }

extern "C" int rinr_store_open_ex(const void *device_blob, const void *host_blob, size_t bytes, const rinr_open_opts *opts,
                                  rinr_store **store) {
    if (!device_blob || !store) return RINR_E_NULL;
    *store = nullptr;
    if ((uintptr_t)device_blob & 15) return RINR_E_ALIGN;
    if (bytes < sizeof(StoreHeader)) return RINR_E_FORMAT;
    int tile_rows = opts && opts->fp32_tile_rows ? opts->fp32_tile_rows : 32;
    if (tile_rows != 16 && tile_rows != 32) return RINR_E_ARG;
    const uint32_t budget = opts && opts->lds_budget ? (uint32_t)opts->lds_budget : kLdsLimit;
    if (budget < 20u * 1024u || budget > kLdsLimit || (budget & 15u)) return RINR_E_ARG;
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
    s->tile_rows_wide = tile_rows;
    s->lds_budget = budget;
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
    {   // split-precision kernels: kinds of hidden layer, fp16 range of every operand they would build
        const uint8_t *hb = (const uint8_t *)host_blob;
        const float pre = (float)((double)sum.header.w0 / (2.0 * M_PI));
        double acts[kMaxClass + 1] = {0, 0, 0, 0, 0};
        s->xdl_ok = std::fabs(sum.header.coord_lo) < 60000.0f && std::fabs(sum.header.coord_hi) < 60000.0f;   // coordinates travel as fp16 hi+lo
        int64_t tot_int = 0, tot_raw = 0;
        for (const IndexEntry &e : s->index) {
            const uint32_t c = e.width == 0 ? 1u : (e.width + 15u) >> 4;
            for (int l = 0; l < e.n_layers; ++l) {
                LayerRec r;
                std::memcpy(&r, hb + e.off + (size_t)l * sizeof(LayerRec), sizeof r);
                const bool hidden = l > 0 && l < e.n_layers - 1;
                const float k = l < e.n_layers - 1 ? pre : 1.0f;
                if (hidden && xdl_int_layer(r.bits, r.scale * pre)) { ++tot_int; continue; }
                if (hidden) ++tot_raw;
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
            acts[c] += (e.n_layers - 1) * 16.0 * c;
        }
        s->hidden_kind = tot_raw == 0 ? kHiddenAllInt : (tot_int == 0 ? kHiddenAllRaw : kHiddenMixed);
        for (uint32_t c = 1; c <= kMaxClass; ++c) {
            // vector-ALU bound: ~20 clocks per activation per lane (sine + hi/lo split), 64 lanes = 64 pixels
            const double mean = sum.class_count[c] ? acts[c] / (double)sum.class_count[c] : 0.0;
            s->class_tile_us_xdl[c] = (mean * 20.0 + 600.0) / 2400.0;
        }
        store_error_bounds(host_blob, sum, s->bounds);
    }
    // which models each kernel family decodes from a resident copy, and the LDS that takes
    s->fit_form[kSizeFp32] = kFitFp32;
    s->fit_form[kSizeXdl] = s->hidden_kind == kHiddenAllInt ? kFitXdlOne : kFitXdlTwo;
    s->fit_form[kSizeXdl16] = kFitXdlOne;
    std::memset(s->res_lds, 0, sizeof s->res_lds);
    std::memset(s->n_res, 0, sizeof s->n_res);
    std::memset(s->n_str, 0, sizeof s->n_str);
    std::memset(s->str_layers, 0, sizeof s->str_layers);
    for (const IndexEntry &e : s->index) {
        const uint32_t c = e.width == 0 ? 1u : (e.width + 15u) >> 4;
        for (int z = 0; z < kSizes; ++z) {
            if (resident_fits(s->fit_form[z], c, e.n_layers, e.nbytes, (uint32_t)tile_rows, budget)) {
                ++s->n_res[z][c];
                s->res_lds[z][c] = std::max(s->res_lds[z][c], resident_bytes(s->fit_form[z], c, e.n_layers, (uint32_t)tile_rows) + e.nbytes);
            } else {
                ++s->n_str[z][c];
                s->str_layers[z][c] = std::max<uint32_t>(s->str_layers[z][c], e.n_layers);
            }
        }
    }
    bool ok = true;
    for (uint32_t c = 1; c <= kMaxClass && ok; ++c) {
        if (!sum.class_count[c]) continue;
        const ClassImpl im = impl_for(c, s->tile_rows_wide);
        ok = allow_full_lds((const void *)im.decode) && allow_full_lds((const void *)im.stream) &&
             allow_full_lds((const void *)im.debug) && allow_full_lds((const void *)im.xdebug[0]) &&
             allow_full_lds((const void *)im.xdebug[1]);
        for (int k = 0; k < 7 && ok; ++k) ok = allow_full_lds((const void *)im.decode_xdl[k]);
        for (int k = 0; k < 3 && ok; ++k) ok = allow_full_lds((const void *)im.stream_xdl[k]);
    }
    ok = ok && allow_full_lds(xdl_any_fn(kHiddenAllInt)) && allow_full_lds(xdl_any_fn(kHiddenAllRaw)) &&
         allow_full_lds(xdl_any_fn(kHiddenMixed)) && allow_full_lds(xdl_any_fn(kHiddenAllInt, true)) &&
         allow_full_lds(xdl_any_fn(kHiddenAllRaw, true)) && allow_full_lds(xdl_any_fn(kHiddenMixed, true)) &&
         allow_full_lds(xdl_any_fn(0, true, true)) && allow_full_lds((const void *)decode_any_kernel<16, kThreads>) &&
         allow_full_lds((const void *)decode_any_kernel<32, kThreads>);
    if (!ok) { delete s; return RINR_E_HIP; }
    if (hip_fail(hipGetDevice(&s->device))) { delete s; return RINR_E_HIP; }
    if (int rc = scratch_for_device(s->device, &s->scratch)) { delete s; return rc; }
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

extern "C" int rinr_store_open(const void *device_blob, const void *host_blob, size_t bytes, rinr_store **store) {
    return rinr_store_open_ex(device_blob, host_blob, bytes, nullptr, store);
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

extern "C" int rinr_store_error_bounds(const rinr_store *s, float bounds[2]) {
    if (!s || !bounds) return RINR_E_NULL;
    bounds[0] = (float)std::min(s->bounds[0], 1e30);
    bounds[1] = (float)std::min(s->bounds[1], 1e30);
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

extern "C" int rinr_decode_batch_ex(rinr_store *s, const int64_t *image_ids, int32_t n, int32_t H, int32_t W,
                                    void *out, const rinr_decode_opts *opts, void *stream) {
    if (!s || !opts) return RINR_E_NULL;
    if (n < 0 || H <= 0 || W <= 0) return RINR_E_ARG;
    const int dt = opts->out_dtype;
    if (dt != RINR_OUT_F32 && dt != RINR_OUT_U8 && dt != RINR_OUT_F32_AND_U8) return RINR_E_ARG;
    if (opts->flags & ~(RINR_FLAG_NO_CLAMP | RINR_FLAG_FP32_MFMA | RINR_FLAG_NORMALIZE | RINR_FLAG_FP16_ACT | RINR_FLAG_FP16_ALL |
                        RINR_FLAG_FP16_UNCHECKED))
        return RINR_E_ARG;
    if ((opts->flags & RINR_FLAG_NORMALIZE) && dt != RINR_OUT_F32) return RINR_E_ARG;
    if (opts->flags & RINR_FLAG_NORMALIZE)
        for (int c = 0; c < 3; ++c)
            if (!std::isfinite(opts->norm_scale[c]) || !std::isfinite(opts->norm_shift[c])) return RINR_E_ARG;
    if ((opts->flags & RINR_FLAG_NO_CLAMP) && dt != RINR_OUT_F32) return RINR_E_ARG;
    if (opts->launch_threads != 0 && (opts->launch_threads % 64 || opts->launch_threads < 64 || opts->launch_threads > kThreads)) return RINR_E_ARG;
    if (opts->launch_blocks_per_cu < 0 || opts->launch_blocks_per_cu > 1024 || opts->one_grid_min_tiles < 0) return RINR_E_ARG;
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
    a.tile_rows_wide = (uint32_t)s->tile_rows_wide;
    a.vec_store = (HW % 4 == 0 && ((uintptr_t)a.out_f32 & 15) == 0 && ((uintptr_t)a.out_u8 & 3) == 0) ? 1u : 0u;
    a.lds_budget = s->lds_budget;
    for (int c = 0; c < 3; ++c) {
        a.ns[c] = a.normalize ? opts->norm_scale[c] : 1.0f;
        a.nb[c] = a.normalize ? opts->norm_shift[c] : 0.0f;
    }
    // which kernels: fp32 MFMA on request (or where an operand exceeds fp16 range), else split precision, in a
    // reduced-precision form where the caller asks for one and the store's error bound allows it
    const bool xdl = s->xdl_ok && !(opts->flags & RINR_FLAG_FP32_MFMA);
    const bool unchecked = (opts->flags & RINR_FLAG_FP16_UNCHECKED) != 0;
    const bool all16 = xdl && (opts->flags & RINR_FLAG_FP16_ALL) && (unchecked || s->bounds[1] <= kBoundLimit);
    const bool act16 = xdl && (opts->flags & (RINR_FLAG_FP16_ACT | RINR_FLAG_FP16_ALL)) &&
                       (all16 || unchecked || s->bounds[0] <= kBoundLimit);
    const int family = !xdl ? kFamFp32 : (all16 ? kFamAll16 : (act16 ? kFamAct16 : kFamSplit));
    const int xk = all16 ? 6 : s->hidden_kind + (act16 ? 3 : 0);      // index into ClassImpl::decode_xdl
    const int z = !xdl ? kSizeFp32 : (all16 ? kSizeXdl16 : kSizeXdl);
    a.fit_form = s->fit_form[z];

    const uint32_t tiles = (uint32_t)((HW + 63) >> 6);
    const int threads = opts->launch_threads ? opts->launch_threads : (tiles >= 96 ? 768 : (tiles >= 64 ? 512 : 256));
    const uint32_t nw = (uint32_t)threads / 64;
    const int64_t any_min_tiles = opts->one_grid_min_tiles ? opts->one_grid_min_tiles : 64;

    int n_classes = 0;
    uint64_t any_streamed = 0, any_resident = 0;
    for (uint32_t c = 1; c <= kMaxClass; ++c) {
        n_classes += s->sum.class_count[c] ? 1 : 0;
        any_streamed += s->n_str[z][c];
        any_resident += s->n_res[z][c];
    }
    // a store that mixes width classes: one grid whose workgroups run the body of their slot's class, or, for images of
    // few tiles, one launch per class with that class's LDS size (workgroups of other classes return at once)
    // (an empty store also takes the one grid: every id is out of range and its slot is zero-filled)
    const bool one_grid = n_classes == 0 || (n_classes > 1 && (int64_t)tiles >= any_min_tiles);
    const int knob = opts->launch_blocks_per_cu * 16 + family + (one_grid ? 8 : 0);
    const bool replan = !(s->plan_hw == HW && s->plan_n == n && s->plan_threads == threads && s->plan_knob == knob);

    // slots of unequal cost are taken heaviest first when the caller gives the scratch for the order
    const bool order = opts->workspace && !s->even_cost;
    if (order) a.order = (const uint32_t *)opts->workspace;
    int launches = 0;
    bool ordered = false;
    uint32_t big_lds = 0, total_blocks = 0;
    auto before_launch = [&]() -> int {          // the first decode launch zero-fills and counts the out-of-range ids
        a.handle_bad = launches == 0 ? 1u : 0u;
        if (order && !ordered) {
            RINR_HIP(order_slots(s, image_ids, n, opts->workspace, stream));
            ordered = true;
            ++launches;
        }
        return RINR_OK;
    };
    // ---- models decoded from a resident expanded copy
    a.stream_mode = any_streamed ? 1u : 0u;
    if (one_grid && (any_resident || n_classes == 0)) {
        const void *fn = xdl ? xdl_any_fn(s->hidden_kind, act16, all16)
                             : (s->tile_rows_wide == 32 ? (const void *)decode_any_kernel<32, kThreads>
                                                        : (const void *)decode_any_kernel<16, kThreads>);
        uint32_t lds_bytes = 16;
        double tile_us = 0.0;
        for (uint32_t c = 1; c <= kMaxClass; ++c) {
            if (!s->sum.class_count[c]) continue;
            lds_bytes = std::max(lds_bytes, s->res_lds[z][c]);
            tile_us += (xdl ? s->class_tile_us_xdl[c] : s->class_tile_us[c]) * (double)s->sum.class_count[c] /
                       (double)h.n_models;
        }
        if (replan) {
            int resident = 1;
            if (hip_fail(hipOccupancyMaxActiveBlocksPerMultiprocessor(&resident, fn, threads, lds_bytes)) || resident < 1)
                resident = 1;
            s->plan[0] = plan_chunks((double)n, tiles, nw, s->n_cu, resident, tile_us, opts->launch_blocks_per_cu);
        }
        const Plan pl = s->plan[0];
        if ((uint64_t)n * pl.chunks > 0x7FFFFFFFull) return RINR_E_SIZE;
        a.chunks = pl.chunks;
        a.tiles_per_chunk = pl.tiles_per_chunk;
        a.cls = 0;
        a.lds_bytes = lds_bytes;
        if (int rc = before_launch()) return rc;
        void *kargs[] = {(void *)&a};
        RINR_HIP(hipLaunchKernel(fn, dim3((uint32_t)n * pl.chunks), dim3((uint32_t)threads), kargs, lds_bytes,
                                 (hipStream_t)stream));
        ++launches;
        total_blocks = (uint32_t)n * pl.chunks;
        big_lds = lds_bytes;
    } else if (!one_grid) {
        for (uint32_t c = 1; c <= kMaxClass; ++c) {
            if (!s->n_res[z][c]) continue;
            const ClassImpl im = impl_for(c, s->tile_rows_wide);
            const uint32_t lds_bytes = s->res_lds[z][c];
            if (replan) {
                int resident = 1;
                if (hip_fail(hipOccupancyMaxActiveBlocksPerMultiprocessor(&resident, (const void *)(xdl ? im.decode_xdl[xk] : im.decode),
                                                                          threads, lds_bytes)) || resident < 1)
                    resident = 1;
                s->plan[c] = plan_chunks((double)n, tiles, nw, s->n_cu, resident, xdl ? s->class_tile_us_xdl[c] : s->class_tile_us[c],
                                         opts->launch_blocks_per_cu);
            }
            const Plan pl = s->plan[c];
            if ((uint64_t)n * pl.chunks > 0x7FFFFFFFull) return RINR_E_SIZE;
            a.chunks = pl.chunks;
            a.tiles_per_chunk = pl.tiles_per_chunk;
            a.cls = c;
            a.lds_bytes = lds_bytes;
            if (int rc = before_launch()) return rc;
            hipLaunchKernelGGL(xdl ? im.decode_xdl[xk] : im.decode, dim3((uint32_t)n * pl.chunks), dim3((uint32_t)threads), lds_bytes,
                               (hipStream_t)stream, a);
            RINR_HIP(hipGetLastError());
            ++launches;
            total_blocks = (uint32_t)n * pl.chunks;
            big_lds = lds_bytes;
        }
    }
    // ---- models too deep for that: one more launch per width class that has any, layers streamed through LDS in groups.
    //      One wavefront per SIMD and one round of tiles per workgroup: every round re-expands the model anyway.
    if (any_streamed) {
        a.stream_mode = 2u;
        const uint32_t nws = (uint32_t)kStreamThreads / 64;
        a.chunks = (tiles + nws - 1) / nws;
        a.tiles_per_chunk = nws;
        if ((uint64_t)n * a.chunks > 0x7FFFFFFFull) return RINR_E_SIZE;
        for (uint32_t c = 1; c <= kMaxClass; ++c) {
            if (!s->n_str[z][c]) continue;
            const ClassImpl im = impl_for(c, s->tile_rows_wide);
            const uint32_t slot = xdl ? im.xslot_bytes : im.slot_bytes, table = xdl ? im.xtable_bytes : 0u;
            const uint32_t k = std::min<uint32_t>(s->str_layers[z][c], (s->lds_budget - table) / slot);
            const uint32_t lds_bytes = table + k * slot;
            a.cls = c;
            a.lds_bytes = lds_bytes;
            if (int rc = before_launch()) return rc;
            hipLaunchKernelGGL(xdl ? im.stream_xdl[all16 ? 2 : (act16 ? 1 : 0)] : im.stream, dim3((uint32_t)n * a.chunks),
                               dim3((uint32_t)kStreamThreads), lds_bytes, (hipStream_t)stream, a);
            RINR_HIP(hipGetLastError());
            ++launches;
            total_blocks = (uint32_t)n * a.chunks;
            big_lds = std::max(big_lds, lds_bytes);
        }
    }
    s->plan_hw = HW; s->plan_n = n; s->plan_threads = threads; s->plan_knob = knob;
    s->last_info[0] = launches;
    s->last_info[1] = (int32_t)total_blocks;
    s->last_info[2] = threads;
    s->last_info[3] = (int32_t)big_lds;
    s->last_info[4] = family;
    s->last_info[5] = any_streamed ? 1 : 0;
    return RINR_OK;
}

extern "C" int rinr_decode_batch_noalloc(rinr_store *s, const int64_t *image_ids, int32_t n, int32_t H, int32_t W,
                                         void *out, const rinr_decode_opts *opts, void *stream) {
    if (!s || !opts) return RINR_E_NULL;
    if (n > RINR_NOALLOC_MAX_SLOTS) return RINR_E_SIZE;
    rinr_decode_opts o = *opts;
    o.workspace = s->scratch;                   // the device address looked up at open, never the array's name
    o.workspace_bytes = sizeof(uint32_t) * (size_t)RINR_NOALLOC_MAX_SLOTS;
    return rinr_decode_batch_ex(s, image_ids, n, H, W, out, &o, stream);
}

extern "C" int rinr_decode_batch(rinr_store *s, const int64_t *image_ids, int32_t n, int32_t H, int32_t W,
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

namespace {
int debug_target(const rinr_store *s, int64_t id, int32_t layer, uint32_t *cls) {
    if (id < 0 || (uint64_t)id >= s->sum.header.n_models) return RINR_E_ARG;
    const IndexEntry &e = s->index[(size_t)id];
    if (layer < 0 || layer >= e.n_layers) return RINR_E_ARG;
    *cls = e.width == 0 ? 1u : (e.width + 15u) >> 4;
    if (*cls > kMaxClass || !s->sum.class_count[*cls]) return RINR_E_FORMAT;
    return RINR_OK;
}
}  // namespace

extern "C" int rinr_debug_dequant(const rinr_store *s, int64_t id, int32_t layer, float *device_out, float *bias_out,
                                  void *stream) {
    if (!s || !device_out) return RINR_E_NULL;
    uint32_t cls = 0;
    if (int rc = debug_target(s, id, layer, &cls)) return rc;
    const ClassImpl im = impl_for(cls, s->tile_rows_wide);
    hipLaunchKernelGGL(im.debug, dim3(1), dim3(256), im.slot_bytes, (hipStream_t)stream, s->blob, id, (int)layer, device_out, bias_out);
    RINR_HIP(hipGetLastError());
    return RINR_OK;
}

extern "C" int rinr_debug_dequant_split(const rinr_store *s, int64_t id, int32_t layer, int32_t fp16_weights, float *hi_out,
                                        float *lo_out, float *bias_out, float *scale_out, void *stream) {
    if (!s || !hi_out || !lo_out) return RINR_E_NULL;
    uint32_t cls = 0;
    if (int rc = debug_target(s, id, layer, &cls)) return rc;
    const ClassImpl im = impl_for(cls, s->tile_rows_wide);
    const uint32_t lds_bytes = im.xtable_bytes + im.xslot_bytes;
    hipLaunchKernelGGL(im.xdebug[fp16_weights ? 1 : 0], dim3(1), dim3(256), lds_bytes, (hipStream_t)stream, s->blob, id, (int)layer,
                       lds_bytes, hi_out, lo_out, bias_out, scale_out);
    RINR_HIP(hipGetLastError());
    return RINR_OK;
}

extern "C" int rinr_last_launch_info(const rinr_store *s, int32_t info[6]) {
    if (!s || !info) return RINR_E_NULL;
    std::memcpy(info, s->last_info, sizeof s->last_info);
    return RINR_OK;
}

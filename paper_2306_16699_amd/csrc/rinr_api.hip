// GPU side of the C ABI: store handle, launch logic for the decode kernels.
#include "../../include/rinr.h"
#include "rinr_kernels.hip.h"
#include "rinr_validate.h"

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
constexpr int kThreads = 512;                // launch bound of the decode kernels

// tuning knobs (see rinr_tune)
int g_tile_rows_wide = 16;      // MFMA tile for classes 2 and 4: 16 (16x16x4) or 32 (32x32x2)
int g_blocks_per_cu = 8;        // grid target, in workgroups per compute unit
int g_threads = 0;              // 0 = choose by image size, else 256 or 512

typedef void (*decode_fn)(const DecodeArgs);
typedef void (*debug_fn)(const uint8_t *, int64_t, int, uint32_t, float *, float *);

struct ClassImpl {
    decode_fn decode;
    debug_fn debug;
    int (*total)(int L);   // expanded floats for L layers
};

template <int TM, int WP> int total_of(int L) { return Layout<TM, WP>::total(L); }
template <int TM, int WP> ClassImpl make_impl() {
    return ClassImpl{decode_kernel<TM, WP, kThreads>, dequant_debug_kernel<TM, WP>, total_of<TM, WP>};
}

ClassImpl impl_for(uint32_t cls, int tile_rows_wide) {
    switch (cls) {
        case 1: return make_impl<16, 16>();
        case 2: return tile_rows_wide == 32 ? make_impl<32, 32>() : make_impl<16, 32>();
        case 3: return make_impl<16, 48>();
        default: return tile_rows_wide == 32 ? make_impl<32, 64>() : make_impl<16, 64>();
    }
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
    mutable int32_t last_info[4];
};

extern "C" int rinr_tune(int knob, int value) {
    switch (knob) {
        case 0: if (value != 16 && value != 32) return RINR_E_ARG; g_tile_rows_wide = value; return RINR_OK;
        case 1: if (value < 1 || value > 1024) return RINR_E_ARG; g_blocks_per_cu = value; return RINR_OK;
        case 2: if (value != 0 && value != 256 && value != 512) return RINR_E_ARG; g_threads = value; return RINR_OK;
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
    for (uint32_t c = 1; c <= kMaxClass; ++c) {
        s->stage_off[c] = s->lds_bytes[c] = 0;
        if (!sum.class_count[c]) continue;
        if (sum.class_max_layers[c] < 2) { delete s; return RINR_E_UNSUPPORTED; }
        const ClassImpl im = impl_for(c, s->tile_rows_wide);
        const uint32_t tot = ((uint32_t)im.total((int)sum.class_max_layers[c]) + 3u) & ~3u;
        const uint64_t need = (uint64_t)tot * 4 + sum.class_max_bytes[c];
        if (need > kLdsLimit) { delete s; return RINR_E_UNSUPPORTED; }
        s->stage_off[c] = tot;
        s->lds_bytes[c] = (uint32_t)need;
        if (hip_fail(hipFuncSetAttribute((const void *)im.decode, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit)) ||
            hip_fail(hipFuncSetAttribute((const void *)im.debug, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit))) {
            delete s;
            return RINR_E_HIP;
        }
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

extern "C" int rinr_decode_batch_ex(const rinr_store *s, const int64_t *image_ids, int32_t n, int32_t H, int32_t W,
                                    void *out, const rinr_decode_opts *opts, void *stream) {
    if (!s || !opts) return RINR_E_NULL;
    if (n < 0 || H <= 0 || W <= 0) return RINR_E_ARG;
    const int dt = opts->out_dtype;
    if (dt != RINR_OUT_F32 && dt != RINR_OUT_U8 && dt != RINR_OUT_F32_AND_U8) return RINR_E_ARG;
    if (opts->flags & ~RINR_FLAG_NO_CLAMP) return RINR_E_ARG;
    if ((opts->flags & RINR_FLAG_NO_CLAMP) && dt != RINR_OUT_F32) return RINR_E_ARG;
    const int64_t HW = (int64_t)H * W;
    if (HW >= (int64_t)1 << 31) return RINR_E_SIZE;
    if (n > 0 && HW > INT64_MAX / 3 / n / 4) return RINR_E_SIZE;
    if (n == 0) { std::memset(s->last_info, 0, sizeof s->last_info); return RINR_OK; }
    if (!image_ids || !out) return RINR_E_NULL;
    if (dt == RINR_OUT_F32_AND_U8 && !opts->out_u8) return RINR_E_NULL;
    if (dt != RINR_OUT_U8 && ((uintptr_t)out & 3)) return RINR_E_ALIGN;
    if ((uintptr_t)image_ids & 7) return RINR_E_ALIGN;

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
    a.inv2W = (float)(1.0 / (2.0 * W));
    a.inv2H = (float)(1.0 / (2.0 * H));
    a.lo = h.coord_lo;
    a.span = h.coord_hi - h.coord_lo;
    a.pre = (float)((double)h.w0 / (2.0 * M_PI));
    a.no_clamp = (opts->flags & RINR_FLAG_NO_CLAMP) ? 1u : 0u;

    const uint32_t tiles = (uint32_t)((HW + 63) >> 6);
    int threads = g_threads ? g_threads : (tiles >= 64 ? 512 : 256);
    const uint32_t nw = (uint32_t)threads / 64;
    // workgroups per slot: aim at g_blocks_per_cu * CUs workgroups in total, but never fewer
    // than one tile per wavefront in a workgroup; tiles per workgroup a multiple of the waves
    uint64_t want = ((uint64_t)g_blocks_per_cu * (uint64_t)s->n_cu + (uint64_t)n - 1) / (uint64_t)n;
    uint32_t max_chunks = tiles / nw ? tiles / nw : 1;
    uint32_t chunks = (uint32_t)(want < 1 ? 1 : (want > max_chunks ? max_chunks : want));
    uint32_t tpc = (tiles + chunks - 1) / chunks;
    tpc = ((tpc + nw - 1) / nw) * nw;
    chunks = (tiles + tpc - 1) / tpc;
    a.chunks = chunks;
    a.tiles_per_chunk = tpc;
    if ((uint64_t)n * chunks > 0x7FFFFFFFull) return RINR_E_SIZE;

    int launches = 0;
    bool first = true;
    uint32_t big_lds = 0;
    for (uint32_t c = 1; c <= kMaxClass; ++c) {
        if (!s->sum.class_count[c]) continue;
        const ClassImpl im = impl_for(c, s->tile_rows_wide);
        a.cls = c;
        a.stage_off = s->stage_off[c];
        a.handle_bad = first ? 1u : 0u;
        first = false;
        hipLaunchKernelGGL(im.decode, dim3((uint32_t)n * chunks), dim3((uint32_t)threads), s->lds_bytes[c],
                           (hipStream_t)stream, a);
        RINR_HIP(hipGetLastError());
        ++launches;
        big_lds = s->lds_bytes[c];
    }
    s->last_info[0] = launches;
    s->last_info[1] = (int32_t)((uint32_t)n * chunks);
    s->last_info[2] = threads;
    s->last_info[3] = (int32_t)big_lds;
    return RINR_OK;
}

extern "C" int rinr_decode_batch(const rinr_store *s, const int64_t *image_ids, int32_t n, int32_t H, int32_t W,
                                 void *out, void *stream) {
    rinr_decode_opts o;
    o.out_dtype = RINR_OUT_F32;
    o.flags = 0;
    o.out_u8 = nullptr;
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

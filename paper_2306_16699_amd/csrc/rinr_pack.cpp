// Host side of the C ABI: validation, packing, unpacking, error strings.
// No GPU calls in this file.
#include "../../include/rinr.h"
#include "rinr_format.h"
#include "rinr_validate.h"

#include <cmath>
#include <cstring>
#include <vector>

using namespace rinr;

namespace {

bool bits_ok(int32_t b) { return b == 0 || (b >= 2 && b <= 8) || b == 16; }

inline bool kept(const rinr_layer_desc &l, int64_t k) {
    return !l.mask || ((l.mask[k >> 3] >> (k & 7)) & 1);
}

int check_opts(const rinr_store_opts *o) {
    if (!o) return RINR_OK;
    if (!std::isfinite(o->w0) || !std::isfinite(o->coord_lo) || !std::isfinite(o->coord_hi)) return RINR_E_ARG;
    if (o->coord_hi == o->coord_lo) return RINR_E_ARG;
    return RINR_OK;
}

// Validates one model; returns its record size in *rec_bytes.
int check_model(const rinr_model_desc &m, uint64_t *rec_bytes, uint32_t *width) {
    if (m.n_layers < 2 || m.n_layers > RINR_MAX_LAYERS || !m.layers) return RINR_E_MODEL;
    uint64_t bytes = (uint64_t)m.n_layers * sizeof(LayerRec);
    uint32_t wmax = 0;
    for (int l = 0; l < m.n_layers; ++l) {
        const rinr_layer_desc &d = m.layers[l];
        if (d.in < 1 || d.out < 1 || d.in > RINR_MAX_WIDTH || d.out > RINR_MAX_WIDTH) return RINR_E_MODEL;
        if (l == 0 && d.in != 2) return RINR_E_MODEL;
        if (l == m.n_layers - 1 && d.out != 3) return RINR_E_MODEL;
        if (l > 0 && d.in != m.layers[l - 1].out) return RINR_E_MODEL;
        if (!bits_ok(d.bits) || !d.weights || !d.bias) return RINR_E_MODEL;
        if (l < m.n_layers - 1 && (uint32_t)d.out > wmax) wmax = (uint32_t)d.out;
        const int64_t cnt = (int64_t)d.in * d.out;
        if (d.bits != 0) {
            if (!std::isfinite(d.scale)) return RINR_E_MODEL;
            if (d.zp < 0 || d.zp >= (1 << d.bits)) return RINR_E_MODEL;
        }
        uint64_t n_kept = 0;
        for (int64_t k = 0; k < cnt; ++k) {
            if (!kept(d, k)) continue;
            ++n_kept;
            if (d.bits == 0) {
                if (!std::isfinite(((const float *)d.weights)[k])) return RINR_E_MODEL;
            } else if (d.bits <= 8) {
                if (((const uint8_t *)d.weights)[k] >= (1u << d.bits)) return RINR_E_MODEL;
            }  // 16-bit codes cannot exceed their range
        }
        for (int o = 0; o < d.out; ++o)
            if (!std::isfinite(d.bias[o])) return RINR_E_MODEL;
        if (d.mask) bytes += 4 * mask_words((uint64_t)cnt);
        bytes += 4 * code_words(n_kept, (uint32_t)d.bits);
        bytes += 4 * (uint64_t)d.out;
    }
    *rec_bytes = (bytes + 15) & ~(uint64_t)15;
    *width = wmax;
    return RINR_OK;
}

void put_code(uint32_t *stream, uint64_t r, uint32_t cb, uint32_t code) {
    const uint64_t bit = r * cb;
    const uint64_t w = bit >> 5;
    const uint32_t sh = (uint32_t)(bit & 31);
    stream[w] |= code << sh;
    if (sh + cb > 32) stream[w + 1] |= code >> (32 - sh);
}

uint32_t get_code(const uint32_t *stream, uint64_t r, uint32_t cb) {
    const uint64_t bit = r * cb;
    const uint64_t w = bit >> 5;
    const uint32_t sh = (uint32_t)(bit & 31);
    const uint64_t two = (uint64_t)stream[w] | ((uint64_t)stream[w + 1] << 32);
    const uint64_t m = cb == 32 ? 0xFFFFFFFFull : ((1ull << cb) - 1);
    return (uint32_t)((two >> sh) & m);
}

}  // namespace

extern "C" int rinr_pack_size(const rinr_model_desc *models, int64_t n_models, const rinr_store_opts *opts,
                              size_t *bytes) {
    if (!bytes || (n_models > 0 && !models)) return RINR_E_NULL;
    if (n_models < 0) return RINR_E_ARG;
    if (int rc = check_opts(opts)) return rc;
    uint64_t total = sizeof(StoreHeader) + (uint64_t)n_models * sizeof(IndexEntry);
    total = (total + 15) & ~(uint64_t)15;
    for (int64_t i = 0; i < n_models; ++i) {
        uint64_t rb; uint32_t w;
        if (int rc = check_model(models[i], &rb, &w)) return rc;
        total += rb;
    }
    *bytes = (size_t)total;
    return RINR_OK;
}

extern "C" int rinr_pack(const rinr_model_desc *models, int64_t n_models, const rinr_store_opts *opts,
                         void *host_blob, size_t bytes) {
    if (!host_blob) return RINR_E_NULL;
    size_t need = 0;
    if (int rc = rinr_pack_size(models, n_models, opts, &need)) return rc;
    if (bytes < need) return RINR_E_SIZE;
    uint8_t *blob = (uint8_t *)host_blob;
    std::memset(blob, 0, need);
    StoreHeader h;
    std::memset(&h, 0, sizeof h);
    std::memcpy(h.magic, kMagic, 8);
    h.version = kVersion;
    h.header_bytes = sizeof(StoreHeader);
    h.n_models = (uint64_t)n_models;
    h.index_off = sizeof(StoreHeader);
    h.total_bytes = need;
    h.w0 = opts ? opts->w0 : 30.0f;
    h.coord_lo = opts ? opts->coord_lo : -1.0f;
    h.coord_hi = opts ? opts->coord_hi : 1.0f;
    uint64_t off = (sizeof(StoreHeader) + (uint64_t)n_models * sizeof(IndexEntry) + 15) & ~(uint64_t)15;
    for (int64_t i = 0; i < n_models; ++i) {
        const rinr_model_desc &m = models[i];
        uint64_t rb; uint32_t width;
        check_model(m, &rb, &width);
        IndexEntry e;
        e.off = off; e.nbytes = (uint32_t)rb; e.n_layers = (uint16_t)m.n_layers; e.width = (uint16_t)width;
        std::memcpy(blob + sizeof(StoreHeader) + (size_t)i * sizeof(IndexEntry), &e, sizeof e);
        uint8_t *rec = blob + off;
        uint32_t cur = (uint32_t)(m.n_layers * sizeof(LayerRec));
        for (int l = 0; l < m.n_layers; ++l) {
            const rinr_layer_desc &d = m.layers[l];
            const int64_t cnt = (int64_t)d.in * d.out;
            LayerRec r;
            std::memset(&r, 0, sizeof r);
            r.n_in = (uint16_t)d.in; r.n_out = (uint16_t)d.out;
            r.bits = (uint8_t)d.bits; r.has_mask = d.mask ? 1 : 0;
            r.scale = d.bits ? d.scale : 0.0f; r.zp = d.bits ? d.zp : 0;
            if (d.mask) {
                r.mask_off = cur;
                uint32_t *mw = (uint32_t *)(rec + cur);
                for (int64_t k = 0; k < cnt; ++k)
                    if (kept(d, k)) mw[k >> 5] |= 1u << (k & 31);
                cur += 4 * (uint32_t)mask_words((uint64_t)cnt);
            }
            r.code_off = cur;
            uint32_t *cs = (uint32_t *)(rec + cur);
            const uint32_t cb = code_bits((uint32_t)d.bits);
            uint64_t nk = 0;
            for (int64_t k = 0; k < cnt; ++k) {
                if (!kept(d, k)) continue;
                uint32_t code;
                if (d.bits == 0) std::memcpy(&code, (const float *)d.weights + k, 4);
                else if (d.bits <= 8) code = ((const uint8_t *)d.weights)[k];
                else code = ((const uint16_t *)d.weights)[k];
                put_code(cs, nk++, cb, code);
            }
            r.n_kept = (uint32_t)nk;
            cur += 4 * (uint32_t)code_words(nk, (uint32_t)d.bits);
            r.bias_off = cur;
            std::memcpy(rec + cur, d.bias, 4 * (size_t)d.out);
            cur += 4 * (uint32_t)d.out;
            std::memcpy(rec + (size_t)l * sizeof(LayerRec), &r, sizeof r);
        }
        if (width > h.max_width) h.max_width = width;
        if ((uint32_t)m.n_layers > h.max_layers) h.max_layers = (uint32_t)m.n_layers;
        if (rb > h.max_model_bytes) h.max_model_bytes = (uint32_t)rb;
        off += rb;
    }
    std::memcpy(blob, &h, sizeof h);
    return RINR_OK;
}

// Full structural validation of a host copy of a blob.  Shared with rinr_store_open.
int rinr::validate_blob(const void *host_blob, size_t bytes, StoreSummary *sum) {
    if (!host_blob) return RINR_E_NULL;
    if (bytes < sizeof(StoreHeader)) return RINR_E_FORMAT;
    const uint8_t *blob = (const uint8_t *)host_blob;
    StoreHeader h;
    std::memcpy(&h, blob, sizeof h);
    if (std::memcmp(h.magic, kMagic, 8) != 0 || h.version != kVersion) return RINR_E_FORMAT;
    if (h.header_bytes != sizeof(StoreHeader) || h.index_off != sizeof(StoreHeader)) return RINR_E_FORMAT;
    if (h.total_bytes > bytes || h.total_bytes < sizeof(StoreHeader)) return RINR_E_FORMAT;
    if (h.n_models > (h.total_bytes - sizeof(StoreHeader)) / sizeof(IndexEntry)) return RINR_E_FORMAT;
    if (!std::isfinite(h.w0) || !std::isfinite(h.coord_lo) || !std::isfinite(h.coord_hi)) return RINR_E_FORMAT;
    const uint64_t data0 = (sizeof(StoreHeader) + h.n_models * sizeof(IndexEntry) + 15) & ~(uint64_t)15;
    StoreSummary s;
    std::memset(&s, 0, sizeof s);
    s.header = h;
    for (uint64_t i = 0; i < h.n_models; ++i) {
        IndexEntry e;
        std::memcpy(&e, blob + sizeof(StoreHeader) + i * sizeof(IndexEntry), sizeof e);
        if ((e.off & 15) || (e.nbytes & 15) || e.off < data0 || e.off > h.total_bytes ||
            e.nbytes > h.total_bytes - e.off)
            return RINR_E_FORMAT;
        if (e.n_layers < 2 || e.n_layers > RINR_MAX_LAYERS) return RINR_E_FORMAT;
        if ((uint64_t)e.n_layers * sizeof(LayerRec) > e.nbytes) return RINR_E_FORMAT;
        if (e.nbytes > h.max_model_bytes || e.n_layers > h.max_layers || e.width > h.max_width) return RINR_E_FORMAT;
        const uint8_t *rec = blob + e.off;
        uint32_t wmax = 0;
        uint16_t prev_out = 2;
        for (int l = 0; l < e.n_layers; ++l) {
            LayerRec r;
            std::memcpy(&r, rec + (size_t)l * sizeof(LayerRec), sizeof r);
            if (r.n_in < 1 || r.n_out < 1 || r.n_in > RINR_MAX_WIDTH || r.n_out > RINR_MAX_WIDTH) return RINR_E_FORMAT;
            if (r.n_in != prev_out) return RINR_E_FORMAT;
            prev_out = r.n_out;
            if (!bits_ok(r.bits) || r.has_mask > 1) return RINR_E_FORMAT;
            if (r.bits && (r.zp < 0 || r.zp >= (1 << r.bits) || !std::isfinite(r.scale))) return RINR_E_FORMAT;
            const uint64_t cnt = (uint64_t)r.n_in * r.n_out;
            if (r.n_kept > cnt || (!r.has_mask && r.n_kept != cnt)) return RINR_E_FORMAT;
            auto in_rec = [&](uint32_t off, uint64_t words) {
                return (off & 3) == 0 && off >= e.n_layers * sizeof(LayerRec) && off <= e.nbytes &&
                       words * 4 <= e.nbytes - off;
            };
            if (r.has_mask) {
                if (!in_rec(r.mask_off, mask_words(cnt))) return RINR_E_FORMAT;
                const uint32_t *mw = (const uint32_t *)(rec + r.mask_off);
                uint64_t pc = 0;
                for (uint64_t w = 0; w < mask_words(cnt); ++w) pc += (uint64_t)__builtin_popcount(mw[w]);
                if (pc != r.n_kept) return RINR_E_FORMAT;
                if (cnt & 31) {
                    if (mw[mask_words(cnt) - 1] >> (cnt & 31)) return RINR_E_FORMAT;   // bits past the end
                }
            }
            if (!in_rec(r.code_off, code_words(r.n_kept, r.bits))) return RINR_E_FORMAT;
            if (!in_rec(r.bias_off, r.n_out)) return RINR_E_FORMAT;
            if (l < e.n_layers - 1 && r.n_out > wmax) wmax = r.n_out;
        }
        if (prev_out != 3 || wmax != e.width) return RINR_E_FORMAT;
        // class census: padded width in units of 16
        const uint32_t cls = wmax == 0 ? 1 : (wmax + 15) / 16;
        if (cls > kMaxClass) return RINR_E_UNSUPPORTED;
        s.class_count[cls]++;
        if (e.nbytes > s.class_max_bytes[cls]) s.class_max_bytes[cls] = e.nbytes;
        if (e.n_layers > s.class_max_layers[cls]) s.class_max_layers[cls] = e.n_layers;
    }
    if (sum) *sum = s;
    return RINR_OK;
}

extern "C" int rinr_unpack_layer(const void *host_blob, size_t bytes, int64_t model, int32_t layer,
                                 uint16_t *codes_out, float *f32_out, uint8_t *keep_out, float *bias_out,
                                 int32_t meta_out[5], float *scale_out) {
    if (int rc = validate_blob(host_blob, bytes, nullptr)) return rc;
    const uint8_t *blob = (const uint8_t *)host_blob;
    StoreHeader h;
    std::memcpy(&h, blob, sizeof h);
    if (model < 0 || (uint64_t)model >= h.n_models) return RINR_E_ARG;
    IndexEntry e;
    std::memcpy(&e, blob + sizeof(StoreHeader) + (size_t)model * sizeof(IndexEntry), sizeof e);
    if (layer < 0 || layer >= e.n_layers) return RINR_E_ARG;
    const uint8_t *rec = blob + e.off;
    LayerRec r;
    std::memcpy(&r, rec + (size_t)layer * sizeof(LayerRec), sizeof r);
    const int64_t cnt = (int64_t)r.n_in * r.n_out;
    const uint32_t *mw = r.has_mask ? (const uint32_t *)(rec + r.mask_off) : nullptr;
    const uint32_t *cs = (const uint32_t *)(rec + r.code_off);
    const uint32_t cb = code_bits(r.bits);
    uint64_t rank = 0;
    for (int64_t k = 0; k < cnt; ++k) {
        const bool kp = !mw || ((mw[k >> 5] >> (k & 31)) & 1);
        uint32_t code = 0;
        float f = 0.0f;
        if (kp) {
            code = get_code(cs, rank++, cb);
            if (r.bits == 0) std::memcpy(&f, &code, 4);
            else f = r.scale * (float)((int32_t)code - r.zp);
        }
        if (keep_out) keep_out[k] = kp ? 1 : 0;
        if (codes_out && r.bits) codes_out[k] = (uint16_t)code;
        if (f32_out) f32_out[k] = f;
    }
    if (bias_out) std::memcpy(bias_out, rec + r.bias_off, 4 * (size_t)r.n_out);
    if (meta_out) {
        meta_out[0] = r.n_in; meta_out[1] = r.n_out; meta_out[2] = r.bits; meta_out[3] = r.zp;
        meta_out[4] = (int32_t)r.n_kept;
    }
    if (scale_out) *scale_out = r.scale;
    return RINR_OK;
}

extern "C" const char *rinr_strerror(int code) {
    switch (code) {
        case RINR_OK: return "ok";
        case RINR_E_NULL: return "a required pointer is NULL";
        case RINR_E_ARG: return "argument out of range";
        case RINR_E_MODEL: return "invalid model description";
        case RINR_E_SIZE: return "buffer too small or size overflow";
        case RINR_E_FORMAT: return "corrupt store blob";
        case RINR_E_UNSUPPORTED: return "model wider or deeper than the decode kernels support";
        case RINR_E_ALIGN: return "misaligned device pointer";
        case RINR_E_HIP: return "HIP runtime error";
        default: return "unknown rinr error";
    }
}

extern "C" const char *rinr_version(void) { return "rinr 0.1 (gfx950)"; }

// A-priori error bounds of the reduced-precision decode modes, computed on the host from a store's own
// weights when it is opened.  No GPU calls in this file.
//
// The reduced-precision kernels round every hidden activation once to fp16 (RINR_FLAG_FP16_ACT) and the
// hidden layers' pre-scaled weights as well (RINR_FLAG_FP16_ALL).  With u = 2^-12 the largest rounding
// error of a value in [-1, 1], |sin'| <= 1 and R_l the largest absolute row sum of layer l's weights,
// the error d_l of the activations after sine layer l obeys
//     d_0 = u + e,      d_l <= w0 R_l (d_{l-1} + t) + s_l + u + e,      |error of the output| <= R_out d_last + e
// with t = 2^-11 the relative rounding of an fp16 weight (0 when the weights stay exact), s_l = 2 pi n_in 2^-25
// the absolute rounding of weights that fall into fp16's subnormal range, and e a small allowance for what
// the full-precision path itself loses per layer (hardware sine, fp32 accumulation).  The bound is a worst
// case over all inputs in the unit box and all signs; it grows with depth like the product of the layers'
// gains w0 R_l, so it certifies shallow or low-gain models (the paper's small-image shape, Sec. VI-A) and
// declines deep ones, whose measured error is orders of magnitude below it.
#include "rinr_validate.h"

#include <cmath>
#include <cstring>

namespace rinr {

namespace {

inline uint32_t popcount_range(const uint32_t *mw, uint32_t start, uint32_t len) {
    uint32_t pc = 0;
    uint32_t k = start;
    const uint32_t end = start + len;
    while (k < end) {
        const uint32_t w = k >> 5, lo = k & 31;
        const uint32_t take = (32 - lo) < (end - k) ? (32 - lo) : (end - k);
        const uint32_t m = take == 32 ? 0xFFFFFFFFu : (((1u << take) - 1u) << lo);
        pc += (uint32_t)__builtin_popcount(mw[w] & m);
        k += take;
    }
    return pc;
}

// Largest absolute row sum of one layer.  Raw fp32 layers: exact.  Coded layers: kept entries of the row times
// the largest magnitude a code can dequantise to (an upper bound that needs no walk over the code stream).
double max_row_sum(const uint8_t *rec, const LayerRec &r) {
    const uint32_t *mw = r.has_mask ? (const uint32_t *)(rec + r.mask_off) : nullptr;
    double best = 0.0;
    if (r.bits == 0) {
        const uint32_t *cs = (const uint32_t *)(rec + r.code_off);
        uint32_t rank = 0;
        for (uint32_t o = 0; o < r.n_out; ++o) {
            double sum = 0.0;
            for (uint32_t i = 0; i < r.n_in; ++i) {
                const uint32_t k = o * r.n_in + i;
                if (mw && !((mw[k >> 5] >> (k & 31)) & 1u)) continue;
                float f;
                std::memcpy(&f, cs + rank++, 4);
                sum += std::fabs((double)f);
            }
            if (sum > best) best = sum;
        }
        return best;
    }
    const double span = (double)(r.zp > ((1 << r.bits) - 1 - r.zp) ? r.zp : ((1 << r.bits) - 1 - r.zp));
    const double wmax = std::fabs((double)r.scale) * span;
    for (uint32_t o = 0; o < r.n_out; ++o) {
        const uint32_t kept = mw ? popcount_range(mw, o * r.n_in, r.n_in) : r.n_in;
        const double sum = kept * wmax;
        if (sum > best) best = sum;
    }
    return best;
}

}  // namespace

// bounds[0]: one fp16 value per hidden activation; bounds[1]: fp16 hidden weights as well.  Maximum over the models.
void store_error_bounds(const void *host_blob, const StoreSummary &sum, double bounds[2]) {
    const uint8_t *blob = (const uint8_t *)host_blob;
    const double w0 = std::fabs((double)sum.header.w0);
    const double u = std::ldexp(1.0, -12), tw = std::ldexp(1.0, -11), e = 2e-6;
    bounds[0] = bounds[1] = 0.0;
    for (uint64_t m = 0; m < sum.header.n_models; ++m) {
        IndexEntry en;
        std::memcpy(&en, blob + sizeof(StoreHeader) + m * sizeof(IndexEntry), sizeof en);
        const uint8_t *rec = blob + en.off;
        double d[2] = {u + e, u + e};
        for (int l = 1; l < en.n_layers; ++l) {
            LayerRec r;
            std::memcpy(&r, rec + (size_t)l * sizeof(LayerRec), sizeof r);
            const double R = max_row_sum(rec, r);
            if (l == en.n_layers - 1) {
                d[0] = R * d[0] + e;
                d[1] = R * d[1] + e;
            } else {
                d[0] = w0 * R * d[0] + u + e;
                d[1] = w0 * R * (d[1] + tw) + 2.0 * M_PI * r.n_in * std::ldexp(1.0, -25) + u + e;
            }
            if (!(d[0] < 1e30)) d[0] = 1e30;
            if (!(d[1] < 1e30)) d[1] = 1e30;
        }
        if (d[0] > bounds[0]) bounds[0] = d[0];
        if (d[1] > bounds[1]) bounds[1] = d[1];
    }
}

}  // namespace rinr

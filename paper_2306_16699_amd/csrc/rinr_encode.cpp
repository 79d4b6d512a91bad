// Host side of the encode path: pruning-ratio schedules, magnitude masks, per-layer quantiser.
#include "../../include/rinr_fit.h"

#include <algorithm>
#include <cmath>
#include <limits>
#include <new>
#include <numeric>
#include <vector>

// Sec. IV-A, Eq. 2-4: a linear piece between two plateaus, constants as printed.
extern "C" double rinr_prune_ratio(int32_t schedule, double psnr) {
    struct Piece { double lo_db, hi_db, below, slope, intercept, above; };
    static const Piece eq2 = {30.0, 35.0, 0.0, 0.05, -1.5, 0.25};      // Eq. 2
    static const Piece eq34 = {35.0, 40.0, 0.2, 0.04, -1.2, 0.4};      // Eq. 3 and Eq. 4 print the same pieces
    if (schedule < 0 || schedule > 2) return std::numeric_limits<double>::quiet_NaN();
    const Piece &p = schedule == 0 ? eq2 : eq34;
    if (std::isnan(psnr)) return psnr;
    if (psnr < p.lo_db) return p.below;
    if (psnr > p.hi_db) return p.above;
    return p.slope * psnr + p.intercept;
}

// Sec. IV-A: unstructured pruning by magnitude.
extern "C" int rinr_l1_mask(const float *w, int64_t n, double ratio, const uint8_t *keep_in, uint8_t *keep_out) {
    if (n < 0 || !(ratio >= 0.0 && ratio <= 1.0)) return RINR_E_ARG;
    if (n == 0) return RINR_OK;
    if (!w || !keep_out) return RINR_E_NULL;
    try {
        std::vector<int64_t> order((size_t)n);
        std::iota(order.begin(), order.end(), (int64_t)0);
        auto mag = [&](int64_t i) { return (keep_in && !keep_in[i]) ? 0.0f : std::fabs(w[i]); };
        std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) { return mag(a) < mag(b); });
        const int64_t n_prune = (int64_t)std::nearbyint(ratio * (double)n);
        for (int64_t k = 0; k < n; ++k) keep_out[order[(size_t)k]] = k < n_prune ? 0 : 1;
        if (keep_in)
            for (int64_t i = 0; i < n; ++i)
                if (!keep_in[i]) keep_out[i] = 0;
    } catch (const std::bad_alloc &) {
        return RINR_E_SIZE;
    }
    return RINR_OK;
}

// Sec. IV-B: per-layer affine codes.
extern "C" int rinr_quantize_layer(const float *w, const uint8_t *keep, int64_t n, int32_t bits, float *scale, int32_t *zp,
                                   uint16_t *codes) {
    if (n < 0 || !((bits >= 2 && bits <= 8) || bits == 16)) return RINR_E_ARG;
    if (!scale || !zp || (n > 0 && (!w || !codes))) return RINR_E_NULL;
    const double qmax = (double)((1u << bits) - 1u);
    double mn = 0.0, mx = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        if (keep && !keep[i]) continue;
        if (!std::isfinite(w[i])) return RINR_E_ARG;
        mn = std::min(mn, (double)w[i]);
        mx = std::max(mx, (double)w[i]);
    }
    double s = (double)(float)((mx - mn) / qmax);
    if (!(s > 0.0)) s = 1.0;
    const double z = std::min(qmax, std::max(0.0, std::nearbyint(-mn / s)));
    *scale = (float)s;
    *zp = (int32_t)z;
    for (int64_t i = 0; i < n; ++i) {
        double q = z;
        if (!keep || keep[i]) q = std::min(qmax, std::max(0.0, std::nearbyint((double)w[i] / s) + z));
        codes[i] = (uint16_t)q;
    }
    return RINR_OK;
}

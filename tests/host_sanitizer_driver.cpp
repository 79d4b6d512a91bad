// Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only, no GPU call anywhere).
// Built and run by tests/test_host_sanitized.py:
//   g++ -fsanitize=address,undefined -fno-sanitize-recover=undefined  this file
//       + csrc/rinr_pack.cpp csrc/rinr_bounds.cpp csrc/rinr_encode.cpp  (the library's host side)
//       + oracle/inr_oracle.c oracle/fit_oracle.c                       (the checkers)
// 1. pack -> validate -> unpack round trip on random models in exactly-sized heap buffers
//    (a read or write one byte outside is an ASan report);
// 2. seeded mutation fuzz of the blob (byte flips, truncations, edits of header / index / layer-record
//    fields to boundary values): validate_blob must answer RINR_OK or an error code, and whatever it
//    accepts must unpack and size its error bounds without leaving the buffer;
// 3. the encode side's host functions and both oracles on small inputs, edge cases included.
// Exit status 0 and the line "sanitizer driver: ok" mean no report and no failed check.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../include/rinr.h"
#include "../include/rinr_fit.h"
#include "../paper_2306_16699_amd/csrc/rinr_validate.h"
extern "C" {
#include "../oracle/fit_oracle.h"
#include "../oracle/inr_oracle.h"
}

namespace {

uint64_t g_state = 0x1234ABCDull;
uint64_t rnd() {                       // splitmix64
    uint64_t z = (g_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
uint32_t below(uint32_t n) { return n ? (uint32_t)(rnd() % n) : 0u; }
double unit() { return (double)(rnd() >> 11) / 9007199254740992.0; }

#define CHECK(cond) do { if (!(cond)) { std::fprintf(stderr, "check failed: %s (line %d)\n", #cond, __LINE__); std::exit(1); } } while (0)

struct HostLayer {
    int in, out, bits, zp;
    float scale;
    std::vector<float> wf;
    std::vector<uint8_t> w8;
    std::vector<uint16_t> w16;
    std::vector<uint8_t> keep;       // one per weight
    std::vector<uint8_t> mask;       // packed bits, empty = dense
    std::vector<float> bias;
};
struct HostModel { std::vector<HostLayer> layers; };

HostModel random_model() {
    static const int kBits[] = {0, 2, 3, 4, 5, 6, 7, 8, 16};
    HostModel m;
    const int n_layers = 2 + (int)below(RINR_MAX_LAYERS - 1);
    std::vector<int> dims(n_layers + 1);
    dims[0] = 2;
    dims[n_layers] = 3;
    for (int l = 1; l < n_layers; ++l) dims[l] = 1 + (int)below(below(4) == 0 ? RINR_MAX_WIDTH : 12);
    m.layers.resize(n_layers);
    for (int l = 0; l < n_layers; ++l) {
        HostLayer &h = m.layers[l];
        h.in = dims[l];
        h.out = dims[l + 1];
        h.bits = kBits[below(9)];
        h.zp = h.bits ? (int)below(1u << h.bits) : 0;
        h.scale = (float)(1e-4 + 1e-2 * unit());
        const int cnt = h.in * h.out;
        h.keep.assign(cnt, 1);
        const int kind = (int)below(4);              // dense, sparse, empty, full mask
        if (kind) {
            for (int k = 0; k < cnt; ++k) h.keep[k] = kind == 1 ? (unit() < 0.4) : (kind == 2 ? 0 : 1);
            h.mask.assign((size_t)(cnt + 7) / 8, 0);
            for (int k = 0; k < cnt; ++k)
                if (h.keep[k]) h.mask[k >> 3] |= (uint8_t)(1u << (k & 7));
        }
        if (h.bits == 0) { h.wf.resize(cnt); for (auto &v : h.wf) v = (float)(unit() - 0.5); }
        else if (h.bits <= 8) { h.w8.resize(cnt); for (auto &v : h.w8) v = (uint8_t)below(1u << h.bits); }
        else { h.w16.resize(cnt); for (auto &v : h.w16) v = (uint16_t)below(1u << 16); }
        h.bias.resize(h.out);
        for (auto &v : h.bias) v = (float)(0.2 * unit() - 0.1);
    }
    return m;
}

struct Described {
    std::vector<rinr_layer_desc> layers;
    std::vector<rinr_model_desc> models;
};
void describe(const std::vector<HostModel> &ms, Described &d) {
    size_t total = 0;
    for (const auto &m : ms) total += m.layers.size();
    d.layers.resize(total);
    d.models.resize(ms.size());
    size_t k = 0;
    for (size_t j = 0; j < ms.size(); ++j) {
        d.models[j].n_layers = (int32_t)ms[j].layers.size();
        d.models[j].layers = d.layers.data() + k;
        for (const HostLayer &h : ms[j].layers) {
            rinr_layer_desc &r = d.layers[k++];
            r.in = h.in; r.out = h.out; r.bits = h.bits; r.scale = h.scale; r.zp = h.zp;
            r.weights = h.bits == 0 ? (const void *)h.wf.data() : (h.bits <= 8 ? (const void *)h.w8.data() : (const void *)h.w16.data());
            r.mask = h.mask.empty() ? nullptr : h.mask.data();
            r.bias = h.bias.data();
        }
    }
}

// Everything a consumer of an accepted blob reads: every layer unpacked, the error bounds sized.
void consume(const uint8_t *blob, size_t bytes, const rinr::StoreSummary &sum) {
    for (uint64_t m = 0; m < sum.header.n_models; ++m) {
        rinr::IndexEntry e;
        std::memcpy(&e, blob + sizeof(rinr::StoreHeader) + m * sizeof(rinr::IndexEntry), sizeof e);
        for (int l = 0; l < e.n_layers; ++l) {
            int32_t meta[5];
            float scale;
            CHECK(rinr_unpack_layer(blob, bytes, (int64_t)m, l, nullptr, nullptr, nullptr, nullptr, meta, &scale) == RINR_OK);
            const size_t cnt = (size_t)meta[0] * meta[1];
            std::vector<uint16_t> codes(cnt);
            std::vector<float> f(cnt), b((size_t)meta[1]);
            std::vector<uint8_t> keep(cnt);
            CHECK(rinr_unpack_layer(blob, bytes, (int64_t)m, l, codes.data(), f.data(), keep.data(), b.data(), meta, &scale) == RINR_OK);
        }
    }
    double bounds[2];
    rinr::store_error_bounds(blob, sum, bounds);
    CHECK(bounds[0] >= 0.0 && bounds[1] >= bounds[0]);
}

void round_trip_and_fuzz(int n_stores, int n_mutations) {
    for (int s = 0; s < n_stores; ++s) {
        std::vector<HostModel> ms(1 + below(5));
        for (auto &m : ms) m = random_model();
        Described d;
        describe(ms, d);
        rinr_store_opts o = {30.0f, -1.0f, 1.0f};
        size_t bytes = 0;
        CHECK(rinr_pack_size(d.models.data(), (int64_t)ms.size(), &o, &bytes) == RINR_OK);
        uint8_t *blob = (uint8_t *)std::malloc(bytes);          // exactly sized: ASan guards both ends
        CHECK(blob);
        CHECK(rinr_pack(d.models.data(), (int64_t)ms.size(), &o, blob, bytes) == RINR_OK);
        CHECK(rinr_pack(d.models.data(), (int64_t)ms.size(), &o, blob, bytes - 1) == RINR_E_SIZE);
        rinr::StoreSummary sum;
        CHECK(rinr::validate_blob(blob, bytes, &sum) == RINR_OK);
        CHECK(sum.header.n_models == ms.size());
        consume(blob, bytes, sum);
        for (size_t j = 0; j < ms.size(); ++j)                  // the round trip itself
            for (size_t l = 0; l < ms[j].layers.size(); ++l) {
                const HostLayer &h = ms[j].layers[l];
                const size_t cnt = (size_t)h.in * h.out;
                std::vector<uint16_t> codes(cnt);
                std::vector<float> f(cnt), b((size_t)h.out);
                std::vector<uint8_t> keep(cnt);
                int32_t meta[5];
                float scale;
                CHECK(rinr_unpack_layer(blob, bytes, (int64_t)j, (int32_t)l, codes.data(), f.data(), keep.data(), b.data(), meta, &scale) == RINR_OK);
                CHECK(meta[0] == h.in && meta[1] == h.out && meta[2] == h.bits);
                CHECK(std::memcmp(b.data(), h.bias.data(), 4 * (size_t)h.out) == 0);
                for (size_t k = 0; k < cnt; ++k) {
                    CHECK(keep[k] == h.keep[k]);
                    if (!h.keep[k]) { CHECK(f[k] == 0.0f); continue; }
                    if (h.bits == 0) CHECK(std::memcmp(&f[k], &h.wf[k], 4) == 0);
                    else CHECK(codes[k] == (h.bits <= 8 ? (uint16_t)h.w8[k] : h.w16[k]));
                }
            }
        // mutations: each on a fresh exactly-sized copy
        int accepted = 0;
        for (int q = 0; q < n_mutations; ++q) {
            size_t nb = bytes;
            const int kind = (int)below(5);
            if (kind == 0) nb = below((uint32_t)bytes + 1);                     // truncation (also to nothing)
            uint8_t *mut = (uint8_t *)std::malloc(nb ? nb : 1);
            CHECK(mut);
            std::memcpy(mut, blob, nb);
            if (kind == 1 && nb) {                                             // a few byte flips anywhere
                for (int r = 1 + (int)below(4); r > 0; --r) mut[below((uint32_t)nb)] ^= (uint8_t)(1u << below(8));
            } else if (kind >= 2 && nb >= 64) {                                // a 16/32/64-bit field of the header, the index or the first records
                const size_t span = kind == 2 ? 64 : (kind == 3 ? 64 + 16 * ms.size() : nb);
                const size_t lim = span < nb ? span : nb;
                static const uint64_t kEdge[] = {0, 1, 2, 3, 15, 16, 17, 63, 64, 65, 255, 256, 0x7FFF, 0x8000, 0xFFFF, 0x10000,
                                                 0x7FFFFFFFull, 0x80000000ull, 0xFFFFFFFFull, 0xFFFFFFFFFFFFFFFFull};
                const uint64_t v = below(3) ? kEdge[below(20)] : rnd();
                const size_t width = (size_t)2 << below(3);                   // 2, 4 or 8 bytes
                if (lim >= width) {
                    const size_t at = (below((uint32_t)(lim - width + 1)) / 2) * 2;
                    std::memcpy(mut + at, &v, width);
                }
            }
            rinr::StoreSummary ms2;
            const int rc = rinr::validate_blob(nb ? mut : nullptr, nb, &ms2);
            CHECK(rc == RINR_OK || (rc < 0 && rc >= RINR_E_HIP));
            if (rc == RINR_OK) { consume(mut, nb, ms2); ++accepted; }
            std::free(mut);
        }
        (void)accepted;
        std::free(blob);
    }
}

void rejected_descriptions() {
    HostModel m = random_model();
    std::vector<HostModel> ms(1, m);
    Described d;
    describe(ms, d);
    size_t bytes = 0;
    CHECK(rinr_pack_size(d.models.data(), 1, nullptr, &bytes) == RINR_OK);
    CHECK(rinr_pack_size(nullptr, 1, nullptr, &bytes) == RINR_E_NULL);
    CHECK(rinr_pack_size(d.models.data(), -1, nullptr, &bytes) == RINR_E_ARG);
    rinr_layer_desc saved = d.layers[0];
    d.layers[0].in = 3;
    CHECK(rinr_pack_size(d.models.data(), 1, nullptr, &bytes) == RINR_E_MODEL);
    d.layers[0] = saved;
    d.layers[0].bits = 9;
    CHECK(rinr_pack_size(d.models.data(), 1, nullptr, &bytes) == RINR_E_MODEL);
    d.layers[0] = saved;
    d.layers[0].bias = nullptr;
    CHECK(rinr_pack_size(d.models.data(), 1, nullptr, &bytes) == RINR_E_MODEL);
    d.layers[0] = saved;
    rinr_store_opts bad = {30.0f, 1.0f, 1.0f};
    CHECK(rinr_pack_size(d.models.data(), 1, &bad, &bytes) == RINR_E_ARG);
    CHECK(rinr_pack_size(nullptr, 0, nullptr, &bytes) == RINR_OK && bytes == 64);      // an empty store is a header
}

void encode_side() {
    for (int sch = 0; sch <= 2; ++sch)
        for (double p = 20.0; p <= 50.0; p += 0.37) CHECK(std::fabs(rinr_prune_ratio(sch, p) - fit_prune_ratio(sch, p)) <= 1e-12);
    CHECK(std::isnan(rinr_prune_ratio(-1, 33.0)) && std::isnan(rinr_prune_ratio(3, 33.0)) && std::isnan(rinr_prune_ratio(0, NAN)));
    for (int rep = 0; rep < 200; ++rep) {
        const int n = (int)below(300);
        std::vector<float> w((size_t)n);
        std::vector<double> wd((size_t)n);
        std::vector<uint8_t> kin((size_t)n), k1((size_t)n + 1, 7), k2((size_t)n + 1, 7);
        for (int i = 0; i < n; ++i) {
            w[i] = below(7) == 0 ? 0.0f : (float)(unit() - 0.5);
            if (below(9) == 0 && i) w[i] = w[i - 1];                           // ties
            wd[i] = w[i];
            kin[i] = unit() < 0.8;
        }
        const double ratio = below(5) == 0 ? (double)below(2) : unit();
        const bool with_in = below(2);
        CHECK(rinr_l1_mask(w.data(), n, ratio, with_in ? kin.data() : nullptr, k1.data()) == RINR_OK);
        fit_l1_mask(wd.data(), n, ratio, with_in ? kin.data() : nullptr, k2.data());
        CHECK(std::memcmp(k1.data(), k2.data(), (size_t)n) == 0 && k1[(size_t)n] == 7);
        static const int kB[] = {2, 3, 4, 5, 6, 7, 8, 16};
        const int bits = kB[below(8)];
        std::vector<uint16_t> c1((size_t)n + 1, 0xABCD), c2((size_t)n + 1, 0xABCD);
        float s1; double s2; int32_t z1, z2;
        CHECK(rinr_quantize_layer(w.data(), with_in ? kin.data() : nullptr, n, bits, &s1, &z1, c1.data()) == RINR_OK);
        fit_quantize(wd.data(), with_in ? kin.data() : nullptr, n, bits, &s2, &z2, c2.data());
        CHECK((double)s1 == s2 && z1 == z2 && std::memcmp(c1.data(), c2.data(), 2 * (size_t)n) == 0 && c1[(size_t)n] == 0xABCD);
    }
    CHECK(rinr_l1_mask(nullptr, 5, 0.5, nullptr, nullptr) == RINR_E_NULL);
    CHECK(rinr_l1_mask(nullptr, -1, 0.5, nullptr, nullptr) == RINR_E_ARG);
    float nanw[2] = {NAN, 1.0f}; float s; int32_t z; uint16_t c[2];
    CHECK(rinr_quantize_layer(nanw, nullptr, 2, 8, &s, &z, c) == RINR_E_ARG);
    CHECK(rinr_quantize_layer(nanw, nullptr, 2, 9, &s, &z, c) == RINR_E_ARG);
}

void oracles() {
    // decode oracle on a model of every layer kind, exactly-sized outputs
    std::vector<HostModel> ms(3);
    for (auto &m : ms) m = random_model();
    std::vector<std::vector<orc_layer>> ol(ms.size());
    std::vector<std::vector<std::vector<uint16_t>>> codes(ms.size());
    std::vector<orc_model> om(ms.size());
    for (size_t j = 0; j < ms.size(); ++j) {
        codes[j].resize(ms[j].layers.size());
        for (size_t l = 0; l < ms[j].layers.size(); ++l) {
            const HostLayer &h = ms[j].layers[l];
            orc_layer o;
            o.n_in = h.in; o.n_out = h.out; o.bits = h.bits; o.zp = h.zp; o.scale = h.scale;
            o.w_f32 = h.bits == 0 ? h.wf.data() : nullptr;
            if (h.bits) {
                codes[j][l].resize((size_t)h.in * h.out);
                for (size_t k = 0; k < codes[j][l].size(); ++k) codes[j][l][k] = h.bits <= 8 ? h.w8[k] : h.w16[k];
            }
            o.codes = h.bits ? codes[j][l].data() : nullptr;
            o.keep = h.mask.empty() ? nullptr : h.keep.data();
            o.bias = h.bias.data();
            ol[j].push_back(o);
        }
        om[j].n_layers = (int32_t)ol[j].size();
        om[j].layers = ol[j].data();
    }
    const int64_t ids[4] = {2, 0, 1, 2};
    const int H = 5, W = 7;
    std::vector<double> out((size_t)4 * 3 * H * W);
    std::vector<uint8_t> out8((size_t)4 * 3 * H * W);
    CHECK(orc_decode(om.data(), 3, ids, 4, H, W, 30.0, -1.0, 1.0, 1, out.data(), out8.data(), 2) == 0);
    for (double v : out) CHECK(v >= 0.0 && v <= 1.0);
    std::vector<double> aff(4 * 6, 0.3), norm(6, 1.5);
    CHECK(orc_decode_aug(om.data(), 3, ids, 4, H, W, 30.0, 0.0, 1.0, 0, aff.data(), norm.data(), out.data(), 1) == 0);
    const int64_t bad[1] = {3};
    CHECK(orc_decode(om.data(), 3, bad, 1, H, W, 30.0, -1.0, 1.0, 1, out.data(), nullptr, 1) != 0);
    // fit oracle: loss, gradient, one Adam step, PSNR
    const int32_t widths[5] = {2, 6, 9, 4, 3};
    const int32_t L = 4;                           // linear layers: widths has L + 1 entries
    const int64_t np_ = fit_n_params(widths, L);
    std::vector<double> p((size_t)np_), g((size_t)np_), m1((size_t)np_, 0.0), v1((size_t)np_, 0.0), tgt((size_t)3 * H * W), fw((size_t)3 * H * W);
    std::vector<uint8_t> keep((size_t)np_);
    for (auto &x : p) x = 0.2 * (unit() - 0.5);
    for (auto &x : tgt) x = unit();
    for (auto &x : keep) x = unit() < 0.7;
    double loss = 0.0;
    fit_loss_grad(widths, L, 30.0, -1.0, 1.0, H, W, p.data(), keep.data(), tgt.data(), 1.0 / (3 * H * W), &loss, g.data());
    CHECK(std::isfinite(loss) && loss >= 0.0);
    fit_loss_grad(widths, L, 30.0, -1.0, 1.0, H, W, p.data(), nullptr, tgt.data(), 1.0, &loss, g.data());
    fit_forward(widths, L, 30.0, -1.0, 1.0, H, W, p.data(), keep.data(), fw.data());
    fit_adam_step(p.data(), m1.data(), v1.data(), g.data(), keep.data(), np_, 1, fit_cosine_lr(5e-4, 0, 10), 0.9, 0.999, 1e-8);
    CHECK(std::isfinite(fit_psnr(fw.data(), tgt.data(), (int64_t)fw.size())));
}

}  // namespace

int main(int argc, char **argv) {
    const int n_stores = argc > 1 ? std::atoi(argv[1]) : 40;
    const int n_mut = argc > 2 ? std::atoi(argv[2]) : 400;
    rejected_descriptions();
    round_trip_and_fuzz(n_stores, n_mut);
    encode_side();
    oracles();
    std::printf("sanitizer driver: ok (%d stores x %d mutations)\n", n_stores, n_mut);
    return 0;
}

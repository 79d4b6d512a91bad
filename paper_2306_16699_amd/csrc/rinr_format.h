// Packed store layout ("weight format" of the dataset, paper Sec. III-B) shared by the
// host packer and the device kernels.  Little-endian, position independent.
//
//   [StoreHeader 64 B][IndexEntry x n_models][model records, each 16-B aligned]
//
// A model record is
//   [LayerRec x n_layers][payload areas, each 4-B aligned]  padded to 16 B
// and each layer's payload is: mask words (only if has_mask), code stream words, biases.
//   mask   : ceil(in*out/32) u32, bit (k & 31) of word (k >> 5) for flat index k = o*in + i
//   codes  : the kept weights only, ascending k; code r occupies stream bits
//            [r*cb, (r+1)*cb), LSB first, cb = bits (32 for raw fp32); the stream is
//            ceil(n_kept*cb/32) + 1 words long so a two-word window read never leaves it
//   bias   : out fp32
#pragma once
#include <stdint.h>

namespace rinr {

constexpr uint32_t kVersion = 1;
constexpr char kMagic[8] = {'R', 'I', 'N', 'R', 'S', 'T', 'O', '1'};

struct StoreHeader {            // 64 bytes
    char magic[8];
    uint32_t version;
    uint32_t header_bytes;
    uint64_t n_models;
    uint64_t index_off;
    uint64_t total_bytes;
    float w0, coord_lo, coord_hi;
    uint32_t max_width;         // widest hidden (sine) layer over all models
    uint32_t max_layers;        // most linear layers
    uint32_t max_model_bytes;   // largest model record
};
static_assert(sizeof(StoreHeader) == 64, "header layout");

struct IndexEntry {             // 16 bytes
    uint64_t off;               // record offset from blob start, multiple of 16
    uint32_t nbytes;            // record size, multiple of 16
    uint16_t n_layers;
    uint16_t width;             // widest hidden layer of this model (0 if n_layers == 1)
};
static_assert(sizeof(IndexEntry) == 16, "index layout");

struct LayerRec {               // 32 bytes; offsets are bytes from the record start
    uint16_t n_in, n_out;
    uint8_t bits;               // 0 raw fp32, 2..8, 16
    uint8_t has_mask;
    uint16_t reserved0;
    float scale;
    int32_t zp;
    uint32_t n_kept;
    uint32_t mask_off;          // 0 if !has_mask
    uint32_t code_off;
    uint32_t bias_off;
};
static_assert(sizeof(LayerRec) == 32, "layer record layout");

inline uint32_t code_bits(uint32_t bits) { return bits == 0 ? 32u : bits; }
inline uint64_t mask_words(uint64_t cnt) { return (cnt + 31) / 32; }
inline uint64_t code_words(uint64_t n_kept, uint32_t bits) { return (n_kept * code_bits(bits) + 31) / 32 + 1; }

}  // namespace rinr

// Host-side blob validation result, shared by the packer and rinr_store_open.
#pragma once
#include <stddef.h>
#include "rinr_format.h"

namespace rinr {

// Models are grouped into width classes: class c holds models whose widest hidden layer
// pads to 16*c (c = 1..4).  The decode launches one kernel instantiation per class.
constexpr uint32_t kMaxClass = 4;

struct StoreSummary {
    StoreHeader header;
    uint64_t class_count[kMaxClass + 1];
    uint32_t class_max_bytes[kMaxClass + 1];   // largest record in the class
    uint32_t class_max_layers[kMaxClass + 1];
};

int validate_blob(const void *host_blob, size_t bytes, StoreSummary *sum);

// Worst-case output error of the reduced-precision decode modes over a validated blob (maximum over its models):
// bounds[0] for one fp16 value per hidden activation, bounds[1] with fp16 hidden weights as well.
void store_error_bounds(const void *host_blob, const StoreSummary &sum, double bounds[2]);

}  // namespace rinr

// Process-wide tuning table: (nranks, floor(log2 bytes)) -> (algorithm, chunk).
// The C ABI in bcast.h is the interface; this header only shares the entry type.
#pragma once

#include <stddef.h>

#include "bcast.h"

namespace bcast {

struct TuneEntry {
    int algo;
    size_t chunk_bytes;
    double usec;
};

int log2_bucket(size_t bytes);  // floor(log2(bytes)), 0 for bytes <= 1

}  // namespace bcast

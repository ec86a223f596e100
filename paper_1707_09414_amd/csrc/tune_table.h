// Process-wide tuning table: (nranks, floor(log2 bytes)) -> (algorithm, chunk).
// The C ABI in bcast.h is the interface; this header only shares the entry type.
#pragma once

#include <stddef.h>

#include "bcast.h"

namespace bcast {

struct TuneEntry {
    int algo;             // fastest algorithm for the bucket
    size_t chunk_bytes;   // its chunk size (chain only)
    double usec;          // its measured time
    size_t chain_chunk;   // best chunk size for the chain, whoever won (0 = unknown)
    double chain_usec;    // the chain's time at that chunk size
};

int log2_bucket(size_t bytes);  // floor(log2(bytes)), 0 for bytes <= 1

}  // namespace bcast

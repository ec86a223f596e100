// Process-wide tuning table: (nranks, floor(log2 bytes)) -> bcast_tune_entry_t.
// The C ABI in bcast.h is the interface; this header only shares helpers.
#pragma once

#include <stddef.h>

#include "bcast.h"

namespace bcast {

int log2_bucket(size_t bytes);  // floor(log2(bytes)), 0 for bytes <= 1

}  // namespace bcast

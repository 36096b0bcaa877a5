// Internal declarations shared by the host-side translation units of libhs.
#pragma once

#include <stdint.h>

#include "hs.h"

namespace hs {

// printf-style; stores the message returned by hs_last_error() for the calling thread.
void set_error(const char* fmt, ...) __attribute__((format(printf, 1, 2)));

// Admission predicate of the spatial partitions (paper Section IV-A, "Admission Control").
hs_status admission_check(const uint32_t* claimed, const uint32_t* req_a, const uint32_t* req_b,
                          int n_words, int device_cus);

}  // namespace hs

// Internal declarations shared by the host-side translation units of libhs.
#pragma once

#include <stdint.h>

#include "hs.h"

namespace hs {

// printf-style; stores the message returned by hs_last_error() for the calling thread.
void set_error(const char* fmt, ...) __attribute__((format(printf, 1, 2)));

// XCDs (dies with an L2 of their own, 32 CUs each) of a device with that many CUs.
int xcd_count(int device_cus);

// Admission predicate of the spatial partitions (paper Section IV-A, "Admission Control"):
// HS_E_OVERSUBSCRIBED for an empty mask, a CU the device does not have or a CU claimed by
// another application; HS_E_INVAL for bad arguments or a mask without a CU on every XCD.
hs_status admission_check(const uint32_t* claimed, const uint32_t* req_a, const uint32_t* req_b,
                          int n_words, int device_cus);

}  // namespace hs

// What the per-stream front (hs_mux) must know of the application it drives.
int hs_internal_app_batch(const hs_app* app);      // streams per submit
int hs_internal_app_grouped(const hs_app* app);    // 1 while a member of a group


// Internal hooks of so_static.hip for the rest of the library.
#pragma once

#include <hip/hip_runtime.h>

namespace so {

// Resolve, for `device` (which must be current), the device address of the static scratch
// array of so_grad_stats_static.  Called from so_create, so that the first allocation-free
// call on a device finds the address already known.
hipError_t static_setup(int device);

// Message of the last failed so_grad_stats_static call on this thread ("" if none).
const char* static_last_error();

}  // namespace so

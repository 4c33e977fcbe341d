// Host-side helpers shared by the library's source files (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>

namespace mh {

// Records the text of a failed HIP call for minhash_last_hip_error() (per host thread)
// and returns MINHASH_ERR_HIP.
int report_hip_error(hipError_t e, const char* what);

// MINHASH_OK, or the recorded failure of one of the launches since the last hipGetLastError().
int launches_ok();

}  // namespace mh

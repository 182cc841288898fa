// Error plumbing shared by the HIP translation units of the library.
#pragma once
#include <hip/hip_runtime.h>

namespace bs {

// Detail of the last failure on this thread, for bs_last_error().
extern thread_local char g_last_error[256];

// Records `what` and the HIP error string, clears HIP's sticky error, returns BS_ENOMEM or BS_EHIP.
int fail_hip(hipError_t e, const char *what);

}  // namespace bs

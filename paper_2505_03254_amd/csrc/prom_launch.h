// Host-side launch bookkeeping shared by the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include "prom.h"

namespace prom {

// Last HIP error seen by this library on the calling thread (hipSuccess if none).
hipError_t &last_hip_error();

// The HIP "last error" slot is per thread and shared with every other user of the runtime
// in the process, so it is cleared before a launch and read right after it.
inline void clear_hip_error() { (void)hipGetLastError(); }
inline int check_launch()
{
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess) return PROM_OK;
    last_hip_error() = e;
    return PROM_EHIP;
}

// Shape checks of the single-layer entry points without pointers (PROM_OK, PROM_EINVAL or
// PROM_EUNSUPPORTED), for entry points that chain several layers and must refuse before their
// first launch what a later layer would refuse.
int pw_shape_check(int n, int h, int w, int cin, int cout);
int dw_shape_check(int n, int h, int w, int c, int stride);

}  // namespace prom

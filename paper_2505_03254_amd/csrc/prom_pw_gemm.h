// The pointwise kernel for wide layers (k loop outermost over a 128-channel x 256-pixel workgroup
// tile; prom_pw_gemm.hip), selected by pw_prepare (prom_pw.hip).
#pragma once
#include "prom_pw_stream.h"

namespace prom {

size_t pw_gemm_lds_bytes();
PwKernelFn pw_gemm_select(bool prelu);

}  // namespace prom

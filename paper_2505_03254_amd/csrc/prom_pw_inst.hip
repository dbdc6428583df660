// Instantiates the streaming pointwise kernel for one NT (tiles per wavefront), given as
// -DPROM_PW_NT=<n> on the command line, so that the variants compile in parallel.
#include "prom_pw_stream.h"

#ifndef PROM_PW_NT
#error "compile with -DPROM_PW_NT=<1..10>"
#endif

namespace prom {

template <int NT, int PT, int XMODE>
static PwKernelFn pick(bool ks1, bool fullw)
{
    if (ks1) return fullw ? &pw_stream_kernel<NT, PT, XMODE, true, true> : &pw_stream_kernel<NT, PT, XMODE, true, false>;
    return fullw ? &pw_stream_kernel<NT, PT, XMODE, false, true> : &pw_stream_kernel<NT, PT, XMODE, false, false>;
}

template <int NT, int PT>
static PwKernelFn pick_x(int xmode, bool ks1, bool fullw)
{
    return xmode == 16 ? pick<NT, PT, 16>(ks1, fullw) : pick<NT, PT, 8>(ks1, fullw);
}

template <> PwKernelFn pw_stream_select<PROM_PW_NT>(int pt, int xmode, bool ks1, bool fullw)
{
    constexpr int NT = PROM_PW_NT;
    if (pt == 1) return pick_x<NT, 1>(xmode, ks1, fullw);
    if constexpr (NT <= 6) {
        if (pt == 2) return pick_x<NT, 2>(xmode, ks1, fullw);
    }
    if constexpr (NT <= 2) {
        if (pt == 4) return pick_x<NT, 4>(xmode, ks1, fullw);
    }
    return nullptr;
}

}  // namespace prom

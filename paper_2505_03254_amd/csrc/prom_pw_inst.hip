// Instantiates the streaming pointwise kernel for one NT (tiles per wavefront), given as
// -DPROM_PW_NT=<n> on the command line, so that the variants compile in parallel.
#include "prom_pw_stream.h"

#ifndef PROM_PW_NT
#error "compile with -DPROM_PW_NT=<1..10>"
#endif

namespace prom {

template <int NT, int PT, int XMODE, int EPI>
static PwKernelFn pick(bool ks1, bool fullw)
{
    if (ks1)
        return fullw ? &pw_stream_kernel<NT, PT, XMODE, true, true, EPI> : &pw_stream_kernel<NT, PT, XMODE, true, false, EPI>;
    return fullw ? &pw_stream_kernel<NT, PT, XMODE, false, true, EPI> : &pw_stream_kernel<NT, PT, XMODE, false, false, EPI>;
}

template <int NT, int PT>
static PwKernelFn pick_x(int xmode, bool ks1, bool fullw, bool prelu)
{
    if (prelu) return xmode == 16 ? pick<NT, PT, 16, kEpiPrelu>(ks1, fullw) : pick<NT, PT, 8, kEpiPrelu>(ks1, fullw);
    return xmode == 16 ? pick<NT, PT, 16, kEpiPlain>(ks1, fullw) : pick<NT, PT, 8, kEpiPlain>(ks1, fullw);
}

template <> PwKernelFn pw_stream_select<PROM_PW_NT>(int pt, int xmode, bool ks1, bool fullw, bool prelu)
{
    constexpr int NT = PROM_PW_NT;
    if (pt == 1) return pick_x<NT, 1>(xmode, ks1, fullw, prelu);
    if constexpr (NT <= 6) {
        if (pt == 2) return pick_x<NT, 2>(xmode, ks1, fullw, prelu);
    }
    if constexpr (NT <= 2) {
        if (pt == 4) return pick_x<NT, 4>(xmode, ks1, fullw, prelu);
    }
    return nullptr;
}

}  // namespace prom

// Instantiations of the row-cooperative pointwise kernel (see prom_pw_rows.h).
#include "prom_pw_rows.h"

namespace prom {

template <int NT> static PwKernelFn rows_pick(bool ks1, int xmode)
{
    if (xmode == 16) return ks1 ? &pw_rows_kernel<NT, true, 16> : &pw_rows_kernel<NT, false, 16>;
    return ks1 ? &pw_rows_kernel<NT, true, 8> : &pw_rows_kernel<NT, false, 8>;
}

PwKernelFn pw_rows_select(int nt, bool ks1, int xmode)
{
    switch (nt) {
    case 1: return rows_pick<1>(ks1, xmode);
    case 2: return rows_pick<2>(ks1, xmode);
    case 3: return rows_pick<3>(ks1, xmode);
    case 4: return rows_pick<4>(ks1, xmode);
    case 5: return rows_pick<5>(ks1, xmode);
    case 6: return rows_pick<6>(ks1, xmode);
    default: return nullptr;
    }
}

}  // namespace prom

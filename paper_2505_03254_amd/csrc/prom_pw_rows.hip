// Instantiations of the row-cooperative pointwise kernel (see prom_pw_rows.h).
#include "prom_pw_rows.h"

namespace prom {

template <int NT> static PwKernelFn rows_pick(bool ks1)
{
    return ks1 ? &pw_rows_kernel<NT, true> : &pw_rows_kernel<NT, false>;
}

PwKernelFn pw_rows_select(int nt, bool ks1)
{
    switch (nt) {
    case 1: return rows_pick<1>(ks1);
    case 2: return rows_pick<2>(ks1);
    case 3: return rows_pick<3>(ks1);
    case 4: return rows_pick<4>(ks1);
    case 5: return rows_pick<5>(ks1);
    case 6: return rows_pick<6>(ks1);
    default: return nullptr;
    }
}

}  // namespace prom

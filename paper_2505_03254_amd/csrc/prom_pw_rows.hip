// Instantiations of the row-cooperative pointwise kernel (see prom_pw_rows.h).
#include "prom_pw_rows.h"

namespace prom {

template <int NT, int EPI> static PwKernelFn rows_pick_e(bool ks1, int xmode)
{
    if (xmode == 16) return ks1 ? &pw_rows_kernel<NT, true, 16, EPI> : &pw_rows_kernel<NT, false, 16, EPI>;
    return ks1 ? &pw_rows_kernel<NT, true, 8, EPI> : &pw_rows_kernel<NT, false, 8, EPI>;
}

PwKernelFn pw_rows_select(int nt, bool ks1, int xmode, bool prelu)
{
    switch (nt) {
    case 1: return prelu ? rows_pick_e<1, kEpiPrelu>(ks1, xmode) : rows_pick_e<1, kEpiPlain>(ks1, xmode);
    case 2: return prelu ? rows_pick_e<2, kEpiPrelu>(ks1, xmode) : rows_pick_e<2, kEpiPlain>(ks1, xmode);
    case 3: return prelu ? rows_pick_e<3, kEpiPrelu>(ks1, xmode) : rows_pick_e<3, kEpiPlain>(ks1, xmode);
    case 4: return prelu ? rows_pick_e<4, kEpiPrelu>(ks1, xmode) : rows_pick_e<4, kEpiPlain>(ks1, xmode);
    case 5: return prelu ? rows_pick_e<5, kEpiPrelu>(ks1, xmode) : rows_pick_e<5, kEpiPlain>(ks1, xmode);
    case 6: return prelu ? rows_pick_e<6, kEpiPrelu>(ks1, xmode) : rows_pick_e<6, kEpiPlain>(ks1, xmode);
    default: return nullptr;
    }
}

}  // namespace prom

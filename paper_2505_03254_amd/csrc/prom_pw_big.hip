// Several LARGE independent pointwise layers in one launch, each with the kernel body of the plan
// the library picks for it alone.  A large layer alone costs 6-8 us of ramp-up and drain on top of
// its streaming time; in one launch only the first and the last layer pay them.  The bodies are
// those of the plans of the large layers at the head of MobileNetV2 (high resolution, few
// channels); a layer with another plan is launched on its own.
#include "prom_pw_rows.h"

namespace prom {

// body ids
enum { kBodyS1x4 = 0, kBodyS6x1 = 1, kBodyR3x8 = 2, kBodyS2x2 = 3, kBodyS2x4 = 4, kBodyR3 = 5, kBodyR6 = 6 };

int pw_big_body_id(int nt, int pt, int xmode, bool ks1, bool fullw, int row_waves)
{
    if (row_waves) {
        if (!ks1) return -1;
        if (nt == 3 && xmode == 8) return kBodyR3x8;
        if (nt == 3 && xmode == 16) return kBodyR3;
        if (nt == 6 && xmode == 16) return kBodyR6;
        return -1;
    }
    if (xmode != 16) return -1;
    if (nt == 1 && pt == 4 && ks1 && fullw) return kBodyS1x4;
    if (nt == 6 && pt == 1 && ks1 && fullw) return kBodyS6x1;
    if (nt == 2 && pt == 2 && !ks1 && !fullw) return kBodyS2x2;
    if (nt == 2 && pt == 4 && !ks1 && !fullw) return kBodyS2x4;
    return -1;
}

size_t pw_big_body_lds(int body, const PwArgs &a)
{
    switch (body) {
    case kBodyS1x4: return lds_bytes_fast(1, a.KS);
    case kBodyS6x1: return lds_bytes_fast(6, a.KS);
    case kBodyS2x2:
    case kBodyS2x4: return lds_bytes_fast(2, a.KS);
    case kBodyR3x8:
    case kBodyR3: return lds_bytes_rows(3, a.cw, a.KS);
    default: return lds_bytes_rows(6, a.cw, a.KS);
    }
}

// One member's work with the epilogue kind E (plain or PReLU) fixed at compile time.
template <int E>
__device__ __forceinline__ void pw_big_member(int body, const PwArgs &a, const int lid, unsigned char *lds_raw)
{
    switch (body) {
    case kBodyS1x4: pw_stream_body<1, 4, 16, true, true, ring_depth<4>(), E>(a, lid, lds_raw); break;
    case kBodyS6x1: pw_stream_body<6, 1, 16, true, true, ring_depth<1>(), E>(a, lid, lds_raw); break;
    case kBodyS2x2: pw_stream_body<2, 2, 16, false, false, ring_depth<2>(), E>(a, lid, lds_raw); break;
    case kBodyS2x4: pw_stream_body<2, 4, 16, false, false, ring_depth<4>(), E>(a, lid, lds_raw); break;
    case kBodyR3x8: pw_rows_body<3, true, 8, 4, E>(a, lid, lds_raw); break;
    case kBodyR3: pw_rows_body<3, true, 16, 4, E>(a, lid, lds_raw); break;
    default: pw_rows_body<6, true, 16, 4, E>(a, lid, lds_raw); break;
    }
}

// EPI: kEpiPlain if no member is a PReLU layer, else kEpiBoth: each member then runs through a
// copy of the bodies compiled for its kind alone (a body that carries both epilogues needs more
// registers than either, and the six-tile bodies would spill).
template <int EPI>
__global__ __launch_bounds__(256, 2) void pw_bigbatch_kernel(const PwBatchArgs b)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int bid = blockIdx.x;
    int i = 0;
    while (i + 1 < b.count && bid >= b.start[i + 1]) ++i;
    const int lid = logical_block_id(bid - b.start[i], b.start[i + 1] - b.start[i]);
    const PwArgs &a = b.layer[i];
    if constexpr (EPI != kEpiPlain) {
        if (a.mult_neg) {
            pw_big_member<kEpiPrelu>(b.body[i], a, lid, lds_raw);
            return;
        }
    }
    pw_big_member<kEpiPlain>(b.body[i], a, lid, lds_raw);
}

// any_prelu: a member of the launch is a PReLU layer.
PwBatchFn pw_bigbatch_fn(bool any_prelu)
{
    return any_prelu ? &pw_bigbatch_kernel<kEpiBoth> : &pw_bigbatch_kernel<kEpiPlain>;
}

}  // namespace prom

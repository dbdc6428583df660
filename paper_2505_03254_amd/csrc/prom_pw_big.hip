// Several LARGE independent pointwise layers in one launch, each with the kernel body of the plan
// the library picks for it alone.  A large layer alone costs 6-8 us of ramp-up and drain on top of
// its streaming time; in one launch only the first and the last layer pay them.  The bodies are
// those of the plans of the large layers at the head of MobileNetV2 (high resolution, few
// channels); a layer with another plan is launched on its own.
#include "prom_pw_rows.h"
#include "prom_pw_expand.h"

namespace prom {

// body ids
enum { kBodyS1x4 = 0, kBodyS6x1 = 1, kBodyR3x8 = 2, kBodyS2x2 = 3, kBodyS2x4 = 4, kBodyR3 = 5, kBodyR6 = 6, kBodyE3x8 = 7 };
constexpr int kExpandRowsG = 4;  // pixel tiles per unit of the full-row body

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

// A layer planned for the row-cooperative body with 8-byte loads (one k step, rows of 48-channel
// pieces: 24 -> 144) runs faster in the body where one wavefront assembles whole rows by itself
// (7 -> about 11 GB/s per workgroup inside the shared launch; the same exchange for the six-tile
// streaming body of 16 -> 96 was measured and is slower).  That body has no residual path.
// Returns the body to run and re-plans `a` for it; *units_per_wg_round is the number of pixel
// units a workgroup takes per round, or 0 if the plan is unchanged.
int pw_big_replan(int body, PwArgs &a, int *units_per_wg_round)
{
    *units_per_wg_round = 0;
    if (body == kBodyR3x8 && !a.residual && a.KS == 1 && a.Nc % 48 == 0 &&
        lds_bytes_expand_rows(a.Nc / 48, 3, kExpandRowsG, a.Nc) <= 56 * 1024) {
        a.cw = 0;
        a.n_chunks = 1;
        a.units = (a.M + 16 * kExpandRowsG - 1) / (16 * kExpandRowsG);
        *units_per_wg_round = 4;
        return kBodyE3x8;
    }
    return body;
}

// Time a workgroup of the body spends per pixel while the chip is full (ns; from the per-workgroup
// timeline of the MobileNetV2 head at batch 128: 32->16, 16->96, 96/144->24, 24->144), or 0 for a
// body that was not measured.  The launch sizes its workgroups by it so that they take about equally long.
double pw_big_body_ns_per_pixel(int body)
{
    switch (body) {
    case kBodyS1x4: return 3.1;
    case kBodyS6x1: return 9.0;
    case kBodyS2x2: return 12.0;
    case kBodyE3x8: return 18.0;
    default: return 0.0;
    }
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
    case kBodyE3x8: return lds_bytes_expand_rows(a.Nc / 48, 3, kExpandRowsG, a.Nc);
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
    case kBodyE3x8: pw_expand_rows_body<kExpandRowsG, 3, 8, E == kEpiPrelu>(a, lid, lds_raw); break;
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
    const int lid = logical_block_id(bid - b.start[i], b.start[i + 1] - b.start[i], i);
    const PwArgs a = b.layer[i];  // a copy: a reference into the by-value argument can force all of it into scratch memory
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

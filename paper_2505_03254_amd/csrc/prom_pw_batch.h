// Bodies of the shared launch of small layers (prom_pw_conv_sequence): which kernel body a member
// runs, by the plan the host made for it.  Shared by pw_batch_kernel (the launch of small layers)
// and pw_bigbatch_kernel, which takes the smallest, latency-bound members behind its large ones.
#pragma once
#include "prom_pw_rows.h"
#include "prom_pw_expand.h"
#include "prom_pw_wreg.h"

namespace prom {

// ============================================================================================
// Several independent layers in one launch: workgroups [start[i], start[i+1]) (both multiples
// of 8) run layer i with the plan NT = 4, PT = 1 and 16-byte activation loads.  The launch,
// prologue and write-back latencies of one layer overlap with the streaming of the others.
constexpr int kBatchNT = 4;
#ifndef PROM_BATCH_DEPTH
#define PROM_BATCH_DEPTH 4
#endif
constexpr int kBatchDepth = PROM_BATCH_DEPTH;  // activation load groups in flight per wavefront
// Tiles per wavefront of a batch member: kBatchNT, or half of it for a layer with many k
// steps, whose decoded fragments would otherwise set the LDS size (and with it the number of
// resident workgroups) of the whole launch.
constexpr int kBatchNTDeep = 3;
constexpr int kBatchDeepKS = 10;
// The narrower body also takes the PReLU layers whose last chunk is ragged: the PReLU epilogue
// with per-lane channel conditions at 4 tiles is the one combination above 168 registers, which
// would cost every member of the launch its third wavefront per SIMD.
__host__ __device__ constexpr int batch_nt(int ks, bool prelu_ragged)
{
    return ks >= kBatchDeepKS || prelu_ragged ? kBatchNTDeep : kBatchNT;
}
__host__ __device__ inline int batch_nt(const PwArgs &a)
{
    return batch_nt(a.KS, a.mult_neg != nullptr && a.Nc % (16 * kBatchNT) != 0);
}
// Pixel tiles per unit of pw_expand_body by number of k steps (registers: 4 per tile and k step).
constexpr int kExpandG1 = 4, kExpandG2 = 3, kExpandG3 = 2, kExpandG5 = 1;
__host__ __device__ constexpr int expand_g(int ks)
{
    return ks == 1 ? kExpandG1 : ks == 2 ? kExpandG2 : ks == 3 ? kExpandG3 : kExpandG5;
}
constexpr int kExpandLds = 52 * 1024;  // three workgroups per CU
constexpr int kExpandRowsG1 = 2;       // pixel tiles per unit of the full-row form (one k step)

// One member's work with the epilogue kind E (plain or PReLU) fixed at compile time.
template <int E>
__device__ __forceinline__ void pw_batch_member(const PwArgs &a, const int lid, unsigned char *lds_raw)
{
    // FULLW bodies (every chunk 16*NT channels wide) have no per-lane conditions in the epilogue;
    // with one k step there is no branch around the epilogue either, so the waits on the prefetch
    // ring are exact (a store in a conditional epilogue makes them conservative)
    if (batch_nt(a) == kBatchNTDeep) {
        if (a.Nc % (16 * kBatchNTDeep) == 0)
            pw_stream_body<kBatchNTDeep, 1, 16, false, true, kBatchDepth, E>(a, lid, lds_raw);
        else
            pw_stream_body<kBatchNTDeep, 1, 16, false, false, kBatchDepth, E>(a, lid, lds_raw);
    } else if (a.Nc % (16 * kBatchNT) == 0) {
        if (a.KS == 1)
            pw_stream_body<kBatchNT, 1, 16, true, true, kBatchDepth, E>(a, lid, lds_raw);
        else
            pw_stream_body<kBatchNT, 1, 16, false, true, kBatchDepth, E>(a, lid, lds_raw);
    } else {
        if constexpr (E == kEpiPlain)  // (a PReLU layer with a ragged last chunk has the narrow body)
            pw_stream_body<kBatchNT, 1, 16, false, false, kBatchDepth, E>(a, lid, lds_raw);
    }
}

template <bool PRELU>
__device__ __forceinline__ void pw_expand_member(const PwArgs &a, const int lid, unsigned char *lds_raw)
{
    if (a.KS == 1)
        pw_expand_body<1, kExpandG1, PRELU>(a, lid, lds_raw);
    else if (a.KS == 2)
        pw_expand_body<2, kExpandG2, PRELU>(a, lid, lds_raw);
    else if (a.KS == 3)
        pw_expand_body<3, kExpandG3, PRELU>(a, lid, lds_raw);
    else
        pw_expand_body<5, kExpandG5, PRELU>(a, lid, lds_raw);
}

// Bodies of pw_wreg_body (weights in registers) a batch member can be planned for: body id ->
// (k steps, tiles per wavefront, pixel tiles fetched ahead).
enum { kWreg6x1 = 1, kWreg6x2 = 2, kWreg9x2 = 3, kWreg9x3 = 4, kWreg15x3 = 5 };

template <int E>
__device__ __forceinline__ void pw_wreg_member(int body, const PwArgs &a, const int lid, unsigned char *lds_raw)
{
    switch (body) {
    case kWreg6x1: pw_wreg_body<6, 1, 3, true, E>(a, lid, lds_raw); break;
    case kWreg6x2: pw_wreg_body<6, 2, 3, true, E>(a, lid, lds_raw); break;
    case kWreg9x2: pw_wreg_body<9, 2, 2, false, E>(a, lid, lds_raw); break;
    case kWreg9x3: pw_wreg_body<9, 3, 2, false, E>(a, lid, lds_raw); break;
    default: pw_wreg_body<15, 3, 1, false, E>(a, lid, lds_raw); break;
    }
}


// One member of the launch of small layers, epilogue kind E (plain or PReLU) fixed at compile time.
// a.cw <= -10: the host planned the layer for the body that keeps the weights in registers (never
// a PReLU layer); a.cw == -1: the full-row form of the body that keeps the activations of a pixel
// group in registers while it walks over the output channels; a.cw > 0: that body; 0: streaming.
template <int E>
__device__ __forceinline__ void pw_small_member(const PwArgs &a, const int lid, unsigned char *lds_raw)
{
    if (a.cw <= -10) {
        pw_wreg_member<kEpiPlain>(-10 - a.cw, a, lid, lds_raw);
    } else if (a.cw < 0) {
        pw_expand_rows_body<kExpandRowsG1, 4, 16, E == kEpiPrelu>(a, lid, lds_raw);
    } else if (a.cw) {
        pw_expand_member<E == kEpiPrelu>(a, lid, lds_raw);
    } else {
        pw_batch_member<E>(a, lid, lds_raw);
    }
}

}  // namespace prom

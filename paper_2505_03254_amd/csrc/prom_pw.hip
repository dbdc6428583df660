// Host side of the ternary pointwise convolution (argument checks, launch planning, the
// C entry points) and the generic any-shape kernel.  The streaming kernel lives in
// prom_pw_stream.h and is instantiated per NT in prom_pw_inst.hip.
#include "prom_pw_batch.h"
#include "prom_pw_gemm.h"
#include "prom_launch.h"

#include <cstdlib>
#include <algorithm>
#include <mutex>
#include <vector>

namespace prom {

// ============================================================================================
// Generic kernel: any shape and alignment, byte-wise activation loads and output stores
// (RAW: int32 accumulators instead of requantised bytes).  Correct, not fast.
// ============================================================================================
template <int NT, bool RAW>
__global__ __launch_bounds__(256) void pw_generic_kernel(const PwArgs a)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int KS = a.KS;
    v4i *frag = reinterpret_cast<v4i *>(lds_raw);
    v4i *lpar = frag + NT * KS * 64;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int j = lane & 15;
    const int g = lane >> 4;

    const int lid = logical_block_id();
    const int chunk = lid % a.n_chunks;
    const int wg = lid / a.n_chunks;
    if (wg >= a.wg_per_chunk) return;
    const int cbase = chunk * NT * 16;
    const int Wv = a.wg_per_chunk * 4;
    const int K = a.K, M = a.M, Nc = a.Nc;

    stage_weights<NT, !RAW>(a, cbase, frag, lpar, !RAW && a.mult_neg != nullptr);

    v4i par[NT][4];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) par[t][r] = RAW ? v4i{0, 0, 0, 0} : lpar[(t * 4 + g) * 4 + r];
    const int lo = in_vgpr(a.lo), hi = in_vgpr(a.hi);
    const int m128 = in_vgpr(-128), p127 = in_vgpr(127);

    for (int u = wg * 4 + wave; u < a.units; u += Wv) {
        const int m = u * 16 + j;
        const bool mvalid = m < M;
        const int8_t *xrow = a.x + (long long)(mvalid ? m : 0) * K;
        v4i acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = v4i{0, 0, 0, 0};
        for (int ks = 0; ks < KS; ++ks) {
            // 16 bytes k = 64*ks + 16*g + e; positions beyond K meet zero weights, so any finite
            // value will do there: clamp the address instead of branching
            v4i b;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                uint32_t v = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int k = 64 * ks + 16 * g + 4 * d + e;
                    v |= (uint32_t)(uint8_t)xrow[k < K ? k : K - 1] << (8 * e);
                }
                b[d] = (int)v;
            }
#pragma unroll
            for (int t = 0; t < NT; ++t)
                acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(frag[(t * KS + ks) * 64 + lane], b, acc[t], 0, 0, 0);
        }
        const long long rowoff = (long long)m * Nc + cbase;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int cl = chan_of<NT>(t, g, r);
                if (mvalid && cbase + cl < Nc) {
                    if constexpr (RAW) {
                        a.acc_out[rowoff + cl] = acc[t][r];
                    } else {
                        int v = a.mult_neg ? requant_prelu_i64(acc[t][r], par[t][r], lo, hi)
                                           : requant_i64<true>(acc[t][r], par[t][r], lo, hi);
                        if (a.residual) v = med3_i32(v + (int)a.residual[rowoff + cl], m128, p127);
                        a.y[rowoff + cl] = (int8_t)v;
                    }
                }
            }
        }
    }
}

// EPI: kEpiPlain if no member is a PReLU layer, else kEpiBoth.  A launch of both kinds runs each
// member through a copy of the bodies compiled for its kind alone (a body that carries both
// epilogues needs more registers than either).
#ifdef PROM_TIMELINE
// Developer build: where single-layer launches record their stamps (see PW_STAMP), and a marker
// kernel that records the clock between launches.
static int32_t *&debug_stamp_buffer()
{
    static int32_t *p = nullptr;
    return p;
}
__global__ void debug_mark_kernel(unsigned long long *buf, int slot) { buf[slot] = wall_clock64(); }

// Developer build (-DPROM_TIMELINE): every workgroup of the shared launch of small layers records
// the constant-rate clock (100 MHz) at its start and end and the member it ran, for a
// per-workgroup timeline of the launch; read back with prom_debug_timeline.
constexpr int kTimelineMax = 32768;
__device__ unsigned long long g_timeline[2 * kTimelineMax];
__device__ int g_timeline_member[kTimelineMax];
struct TimelineScope {
    int bid, member;
    __device__ TimelineScope(int bid_, int member_) : bid(bid_), member(member_)
    {
        if (threadIdx.x == 0 && bid < kTimelineMax) {
            g_timeline[2 * bid] = wall_clock64();
            g_timeline_member[bid] = member;
        }
    }
    __device__ ~TimelineScope()
    {
        __syncthreads();
        if (threadIdx.x == 0 && bid < kTimelineMax) g_timeline[2 * bid + 1] = wall_clock64();
    }
};
#endif

template <int EPI>
__global__ __launch_bounds__(256, 2) void pw_batch_kernel(const PwBatchArgs b)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int bid = blockIdx.x;
    int i = 0;
    while (i + 1 < b.count && bid >= b.start[i + 1]) ++i;
    const int local = bid - b.start[i];
    const int nblk = b.start[i + 1] - b.start[i];
    const PwArgs a = b.layer[i];  // a copy: a reference into the by-value argument can force all of it into scratch memory
    const int lid = logical_block_id(local, nblk, i);
#ifdef PROM_TIMELINE
    TimelineScope timeline_scope(bid, i);
#endif
    if constexpr (EPI != kEpiPlain) {
        if (a.mult_neg) {
            pw_small_member<kEpiPrelu>(a, lid, lds_raw);
            return;
        }
    }
    pw_small_member<kEpiPlain>(a, lid, lds_raw);
}

__global__ __launch_bounds__(256) void copy_kernel(const v4i *__restrict__ src, v4i *__restrict__ dst,
                                                   long long n16)
{
    const long long stride = (long long)gridDim.x * 256;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// ---------------------------------------------------------------------------- host side
constexpr int kMaxCin = 4096;
constexpr int kLdsBudget = 64 * 1024;  // decoded fragments; parameters and staging come on top
constexpr int kLdsMax = 96 * 1024;     // dynamic LDS limit requested per kernel (gfx950: 160 KB per CU)
constexpr int kNumCU = 256;
constexpr long long kStreamBytes = (1LL << 31) - (1LL << 16);  // 32-bit buffer offsets

using KernelFn = PwKernelFn;

// mode 0: requantised output; mode 1: raw accumulators.  fast: streaming kernel applies.
static KernelFn select_kernel(int nt, int pt, int xmode, bool ks1, bool fullw, bool fast, int mode, bool prelu)
{
    if (!fast) {
        const bool raw = mode == 1;
        switch (nt) {
        case 1: return raw ? &pw_generic_kernel<1, true> : &pw_generic_kernel<1, false>;
        case 2: return raw ? &pw_generic_kernel<2, true> : &pw_generic_kernel<2, false>;
        case 3: return raw ? &pw_generic_kernel<3, true> : &pw_generic_kernel<3, false>;
        default: return raw ? &pw_generic_kernel<4, true> : &pw_generic_kernel<4, false>;
        }
    }
    switch (nt) {
    case 1: return pw_stream_select<1>(pt, xmode, ks1, fullw, prelu);
    case 2: return pw_stream_select<2>(pt, xmode, ks1, fullw, prelu);
    case 3: return pw_stream_select<3>(pt, xmode, ks1, fullw, prelu);
    case 4: return pw_stream_select<4>(pt, xmode, ks1, fullw, prelu);
    case 5: return pw_stream_select<5>(pt, xmode, ks1, fullw, prelu);
    case 6: return pw_stream_select<6>(pt, xmode, ks1, fullw, prelu);
    case 7: return pw_stream_select<7>(pt, xmode, ks1, fullw, prelu);
    case 8: return pw_stream_select<8>(pt, xmode, ks1, fullw, prelu);
    case 9: return pw_stream_select<9>(pt, xmode, ks1, fullw, prelu);
    case 10: return pw_stream_select<10>(pt, xmode, ks1, fullw, prelu);
    default: return nullptr;
    }
}

// Workgroups of `fn` that fit on one CU with `lds` bytes of dynamic LDS; also raises the
// kernel's dynamic-LDS limit once.  Cached per (kernel, LDS size); 0 on error.
static int resident_workgroups(KernelFn fn, size_t lds, int threads = 256)
{
    struct Entry { KernelFn fn; size_t lds; int threads; int occ; };
    static std::mutex mu;
    static std::vector<Entry> cache;
    std::lock_guard<std::mutex> lock(mu);
    bool seen_fn = false;
    for (const Entry &e : cache) {
        if (e.fn == fn) {
            seen_fn = true;
            if (e.lds == lds && e.threads == threads) return e.occ;
        }
    }
    if (!seen_fn) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kLdsMax);
        if (e != hipSuccess && lds > 64 * 1024) {
            last_hip_error() = e;
            return 0;
        }
    }
    int occ = 0;
    const hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, reinterpret_cast<const void *>(fn),
                                                                      threads, lds);
    if (e != hipSuccess || occ < 1) {
        last_hip_error() = e;
        (void)hipGetLastError();
        return 0;
    }
    cache.push_back({fn, lds, threads, occ});
    return occ;
}

static bool overlaps(const void *p, size_t pn, const void *q, size_t qn)
{
    const uintptr_t a = (uintptr_t)p, b = (uintptr_t)q;
    return a < b + qn && b < a + pn;
}

static int max_pt_for(int nt) { return nt <= 2 ? 4 : (nt <= 6 ? 2 : 1); }

// Row-cooperative plan for a layer whose row does not fit one wavefront's chunk: CW chunks of NT
// tiles per workgroup that together are the whole row, cout == 16*NT*CW.  (Splitting a wider
// row into several such pieces was measured and is no faster than the plain kernel.)  Prefers
// 4 wavefronts per row (fewer registers each).  Returns false if there is no such split or it
// does not fit the LDS budget.
static bool plan_rows(int cin, int cout, int ks, int *cw_out, int *nt_out)
{
    if (cin % 8 != 0) return false;
    for (int cw = 4; cw >= 2; --cw) {
        if (cout % (16 * cw) != 0) continue;
        const int nt = cout / (16 * cw);
        if (nt < 1 || nt > kRowsMaxNT) continue;
        if ((long long)cw * nt * ks * 1024 > kLdsBudget) continue;
        *cw_out = cw;
        *nt_out = nt;
        return true;
    }
    return false;
}

struct PwLaunch {
    PwArgs a;
    KernelFn fn;
    int nt, pt, xmode, grid;
    int threads;  // workgroup size: 256, or 64*cw*(4/cw) for the row-cooperative kernel
    size_t lds;
    bool fast;
    bool rows;  // row-cooperative kernel (a.cw != 0)
    int big_body;  // body of pw_bigbatch_kernel that runs this plan, or -1
    int mode;
    bool gemm;  // the kernel of wide layers (k loop outermost); never a member of a shared launch
};

// Validate the arguments and fill the launch description.  mode: 0 = requantised int8
// output, 1 = raw int32 accumulators.  shape_only: plan from the shape alone (no pointers,
// no device queries).  Launches nothing.
static int pw_prepare(const int8_t *x, int n, int h, int w, int cin, const void *w_packed, int cout,
                      const prom_requant_t *rq, const int8_t *residual, int8_t *y, int32_t *acc_out,
                      const prom_pw_plan_t *plan, int mode, bool shape_only, PwLaunch &L)
{
    if (n <= 0 || h <= 0 || w <= 0 || cin <= 0 || cout <= 0) return PROM_EINVAL;
    const long long M = (long long)n * h * w;
    if (!shape_only) {
        if (!x || !w_packed) return PROM_EINVAL;
        if (((uintptr_t)w_packed & 3) != 0) return PROM_EINVAL;
        if (mode == 0) {
            if (!rq || !rq->bias || !rq->mult || !rq->shift || !y) return PROM_EINVAL;
            if (rq->act_min < -128 || rq->act_max > 127 || rq->act_min > rq->act_max) return PROM_EINVAL;
        } else {
            if (!acc_out || ((uintptr_t)acc_out & 3) != 0) return PROM_EINVAL;
        }
    }
    if (cin > kMaxCin) return PROM_EUNSUPPORTED;
    if (M >= (1LL << 31) - (1LL << 22)) return PROM_EUNSUPPORTED;
    if (M * (long long)(cin > cout ? cin : cout) >= (1LL << 40)) return PROM_EUNSUPPORTED;
    if (!shape_only) {
        const size_t xbytes = (size_t)M * cin, ybytes = (size_t)M * cout;
        const size_t wbytes = prom_packed_size(cout, cin);
        if (mode == 0) {
            if (overlaps(y, ybytes, x, xbytes) || overlaps(y, ybytes, w_packed, wbytes)) return PROM_EALIAS;
            if (residual && residual != y && overlaps(y, ybytes, residual, ybytes)) return PROM_EALIAS;
        } else {
            if (overlaps(acc_out, ybytes * 4, x, xbytes) || overlaps(acc_out, ybytes * 4, w_packed, wbytes))
                return PROM_EALIAS;
        }
    }

    PwArgs &a = L.a;
    a.x = x;
    a.wq = static_cast<const uint32_t *>(w_packed);
    a.bias = rq ? rq->bias : nullptr;
    a.mult = rq ? rq->mult : nullptr;
    a.mult_neg = rq ? rq->mult_neg : nullptr;
    a.shift = rq ? rq->shift : nullptr;
    a.residual = mode == 0 ? residual : nullptr;
    a.y = y;
    a.acc_out = acc_out;
#ifdef PROM_TIMELINE
    if (mode == 0) a.acc_out = debug_stamp_buffer();
#endif
    a.M = (int)M;
    a.K = cin;
    a.Nc = cout;
    a.KW = (cin + 15) / 16;
    a.KS = (cin + 63) / 64;
    a.lo = rq ? rq->act_min : 0;
    a.hi = rq ? rq->act_max : 0;

    const int n_tiles = (cout + 15) / 16;
    const bool aligned = (((uintptr_t)x | (uintptr_t)y | (uintptr_t)residual) & 3) == 0;
    // The streaming kernel uses unsigned 32-bit byte offsets that saturate at kOobOffset; tensor
    // sizes and per-iteration strides must stay below that value.
    const bool small = (M + 4096) * (long long)(cin > cout ? cin : cout) < kStreamBytes - (1LL << 24);
    bool fast = mode == 0 && aligned && small && (cin % 8 == 0) && (cout % 4 == 0);

    int nt, pt;
    const int nt_lds = kLdsBudget / (a.KS * 1024);  // >= 1 since KS <= 64
    const bool one_chunk_only = cout % 16 != 0;      // more chunks need whole 16-byte pieces per row
    if (fast && one_chunk_only && (n_tiles > kMaxNT || n_tiles > nt_lds)) fast = false;
    if (!fast) {
        if (plan && (plan->tiles_per_wave || plan->pixel_tiles)) return PROM_EINVAL;
        nt = nt_lds < 4 ? nt_lds : 4;
        if (nt > n_tiles) nt = n_tiles;
        pt = 1;
    } else {
        int nt_cap = nt_lds < kMaxNT ? nt_lds : kMaxNT;
        if (plan && plan->tiles_per_wave) {
            if (plan->tiles_per_wave < 1 || plan->tiles_per_wave > nt_cap) return PROM_EINVAL;
            if (one_chunk_only && plan->tiles_per_wave < n_tiles) return PROM_EINVAL;
            nt = plan->tiles_per_wave;
        } else if (one_chunk_only) {
            nt = n_tiles;
        } else {
            if (nt_cap > 9) nt_cap = 9;
            const int chunks = (n_tiles + nt_cap - 1) / nt_cap;
            nt = (n_tiles + chunks - 1) / chunks;
        }
        if (plan && plan->pixel_tiles) {
            pt = plan->pixel_tiles;
            if (!(pt == 1 || pt == 2 || pt == 4) || pt > max_pt_for(nt)) return PROM_EINVAL;
        } else {
            pt = nt <= 2 ? (a.KS == 1 ? 4 : 2) : (nt <= 4 ? 2 : 1);
            while (pt > 1 && M < (long long)64 * pt * kNumCU * 2) pt >>= 1;  // small layers: finer groups
        }
    }
    // A layer that would be split into several chunks takes the row-cooperative kernel when
    // its shape allows (an explicit tile plan keeps the plain streaming kernel).
    a.cw = 0;
    L.rows = false;
    if (plan && plan->row_waves) {
        const int cw = plan->row_waves, rnt = plan->tiles_per_wave;
        if (!fast || cw < 2 || cw > 4 || rnt < 1 || rnt > kRowsMaxNT || plan->pixel_tiles > 1) return PROM_EINVAL;
        if (cout % (16 * rnt * cw) != 0) return PROM_EINVAL;
        if (lds_bytes_rows(rnt, cw, a.KS) > (size_t)kLdsMax) return PROM_EINVAL;
        L.rows = true;
        a.cw = cw;
        nt = rnt;
        pt = 1;
    } else if (fast && !(plan && (plan->tiles_per_wave || plan->pixel_tiles)) && a.KS == 1 &&
               ((n_tiles + nt - 1) / nt > 1 || nt >= 8)) {
        // also instead of one chunk of 8 or more tiles, whose kernel needs so many registers that
        // only one wavefront per SIMD is resident.  Only for layers of one k step (expansions from
        // at most 64 channels): with more input channels the plain kernel with wide chunks is the
        // faster one (56x56 at batch 128: 128 -> 256 39 us against 49, 256 -> 128 33 against 65,
        // 256 -> 256 52 against 84), since the rows a workgroup shares grow with the k steps while
        // the write-back this form coalesces stays the same.
        int cw = 0, rnt = 0;
        if (plan_rows(cin, cout, a.KS, &cw, &rnt)) {
            L.rows = true;
            a.cw = cw;
            nt = rnt;
            pt = 1;
        }
    }
    L.nt = nt;
    L.pt = pt;
    L.fast = fast;
    L.mode = mode;
    L.xmode = !fast ? 1 : (cin % 16 == 0 ? 16 : 8);
    L.threads = L.rows ? rows_threads(a.cw) : 256;
    if (L.rows) {
        L.lds = lds_bytes_rows(nt, a.cw, a.KS);
        L.fn = pw_rows_select(nt, a.KS == 1, L.xmode, a.mult_neg != nullptr);
    } else {
        L.lds = fast ? lds_bytes_fast(nt, a.KS) : lds_bytes_generic(nt, a.KS);
        L.fn = select_kernel(nt, pt, L.xmode, a.KS == 1, cout % (16 * nt) == 0, fast, mode, a.mult_neg != nullptr);
    }
    if (!L.fn) return PROM_EINVAL;
    L.big_body = fast ? pw_big_body_id(nt, pt, L.xmode, a.KS == 1, cout % (16 * nt) == 0, a.cw) : -1;

    a.n_chunks = L.rows ? cout / (16 * nt * a.cw) : (n_tiles + nt - 1) / nt;
    a.units = (int)((M + 16 * pt - 1) / (16 * pt));
    // a workgroup's 4 wavefronts take 4 groups per round (4 / cw groups in the row-cooperative kernel)
    const long long wg_units = L.rows ? (a.units + rows_groups(a.cw) - 1) / rows_groups(a.cw) : (a.units + 3) / 4;
    long long wgs;
    if (plan && plan->workgroups) {
        if (plan->workgroups < 1) return PROM_EINVAL;
        wgs = plan->workgroups;
        if (wgs > wg_units) wgs = wg_units;
    } else {
        // One resident round of workgroups, every wavefront with the same number of groups.
        int occ = 2;
        if (!shape_only) {
            occ = resident_workgroups(L.fn, L.lds, L.threads);
            if (occ < 1) return PROM_EHIP;
        }
        long long target = ((long long)kNumCU * occ) / a.n_chunks;
        if (target < 1) target = 1;
        if (target > wg_units) target = wg_units;
        const long long rounds = (wg_units + target - 1) / target;
        wgs = (wg_units + rounds - 1) / rounds;
    }
    a.wg_per_chunk = (int)wgs;
    const long long total = wgs * a.n_chunks;
    if (total > (1LL << 30)) return PROM_EUNSUPPORTED;
    L.grid = (int)((total + 7) / 8 * 8);

    // Wide layers: the kernel with the k loop outermost.  With a thousand input channels the decoded
    // weights of all k steps fit LDS only for two to four channel tiles per chunk, and every chunk
    // streams the activations again; the tile kernel decodes per k step and does 32 MFMAs per 4
    // activation loads.  Measured (batch 128, one launch per layer, cache-cold, us against the
    // streaming kernel): 14x14 1024 -> 512 33 against 37, 1024 -> 1024 56 against 63; 7x7
    // 1024 -> 2048 31 against 36, 2048 -> 1024 32 against 58.  With 512 and fewer input channels the
    // streaming kernel is the faster one (14x14 512 -> 1024 26 against 43 us, 28x28 512 -> 512 45
    // against 76), so the library takes the tile kernel from 1024 input channels on -- when its
    // tiles fill the chip: a tile takes 6 us plus 0.65 us per k step however few there are, and with
    // less than one tile per compute unit the streaming kernel, which spreads the pixels over more
    // workgroups, is faster (batch 32: 14x14 1024 -> 512, 100 tiles, 13 against 19 us; 7x7
    // 1024 -> 2048, 112 tiles, 13 against 20; 2048 -> 1024, 56 tiles, 19 against 26; 14x14
    // 1024 -> 1024, 200 tiles, 22 against 20).  The two meet at about 180 tiles of 16 k steps and 80
    // tiles of 32: tiles x k steps >= 2800.
    L.gemm = false;
    const int k_outer = plan ? plan->k_outer : 0;
    if (k_outer != 0 && k_outer != 1 && k_outer != -1) return PROM_EINVAL;
    const bool aligned16 = shape_only || ((((uintptr_t)x | (uintptr_t)y | (uintptr_t)residual) & 15) == 0 &&
                                          ((uintptr_t)w_packed & 7) == 0);
    const bool gemm_ok = fast && cin % 64 == 0 && cout % 16 == 0 && aligned16;
    if (k_outer == 1) {
        if (!gemm_ok || plan->tiles_per_wave || plan->pixel_tiles || plan->row_waves || plan->workgroups)
            return PROM_EINVAL;
    }
    const bool explicit_stream = plan && (plan->tiles_per_wave || plan->pixel_tiles || plan->row_waves);
    const long long gemm_tiles = ((M + 255) / 256) * ((cout + 127) / 128);
    const bool gemm_pays = cin >= 1024 && cout >= 256 && gemm_tiles * (cin / 64) >= 2800;
    if (gemm_ok && (k_outer == 1 || (k_outer == 0 && !explicit_stream && gemm_pays))) {
        L.gemm = true;
        L.rows = false;
        a.cw = 0;
        L.nt = 8;
        L.pt = 4;
        L.xmode = 16;
        L.threads = 256;
        L.lds = pw_gemm_lds_bytes();
        L.fn = pw_gemm_select(a.mult_neg != nullptr);
        L.big_body = -1;
        a.n_chunks = (cout + 127) / 128;
        a.units = (int)((M + 63) / 64);
        a.wg_per_chunk = (int)((M + 255) / 256);
        const long long tot = (long long)a.n_chunks * a.wg_per_chunk;
        if (tot > (1LL << 30)) return PROM_EUNSUPPORTED;
        L.grid = (int)((tot + 7) / 8 * 8);
    }
    return PROM_OK;
}

static int pw_launch(const PwLaunch &L, hipStream_t st)
{
    if (L.lds > 64 * 1024 && resident_workgroups(L.fn, L.lds, L.threads) < 1) return PROM_EHIP;
    clear_hip_error();
    PwArgs args = L.a;
    void *kargs[] = {&args};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(L.fn), dim3(L.grid), dim3(L.threads), kargs,
                                         L.lds, st);
    if (e != hipSuccess) {
        last_hip_error() = e;
        (void)hipGetLastError();
        return PROM_EHIP;
    }
    return check_launch();
}

static int pw_dispatch(const int8_t *x, int n, int h, int w, int cin, const void *w_packed, int cout,
                       const prom_requant_t *rq, const int8_t *residual, int8_t *y, int32_t *acc_out,
                       const prom_pw_plan_t *plan, void *stream, int mode)
{
    PwLaunch L;
    const int rc = pw_prepare(x, n, h, w, cin, w_packed, cout, rq, residual, y, acc_out, plan, mode,
                              false, L);
    if (rc != PROM_OK) return rc;
    return pw_launch(L, static_cast<hipStream_t>(stream));
}

}  // namespace prom

extern "C" int prom_pw_conv_ex(const int8_t *x, int n, int h, int w, int cin, const void *w_packed,
                               int cout, const prom_requant_t *rq, const int8_t *residual, int8_t *y,
                               const prom_pw_plan_t *plan, void *stream)
{
    return prom::pw_dispatch(x, n, h, w, cin, w_packed, cout, rq, residual, y, nullptr, plan, stream, 0);
}

extern "C" int prom_pw_conv(const int8_t *x, int n, int h, int w, int cin, const void *w_packed,
                            int cout, const prom_requant_t *rq, const int8_t *residual, int8_t *y,
                            void *stream)
{
    return prom::pw_dispatch(x, n, h, w, cin, w_packed, cout, rq, residual, y, nullptr, nullptr, stream, 0);
}

extern "C" int prom_pw_accum_i32(const int8_t *x, int n, int h, int w, int cin, const void *w_packed,
                                 int cout, int32_t *acc, void *stream)
{
    return prom::pw_dispatch(x, n, h, w, cin, w_packed, cout, nullptr, nullptr, nullptr, acc, nullptr,
                             stream, 1);
}

extern "C" int prom_pw_plan_query(int n, int h, int w, int cin, int cout, prom_pw_plan_t *plan_out,
                                  int *load_bytes_out)
{
    if (!plan_out) return PROM_EINVAL;
    prom::PwLaunch L;
    const int rc = prom::pw_prepare(nullptr, n, h, w, cin, nullptr, cout, nullptr, nullptr, nullptr,
                                    nullptr, nullptr, 0, true, L);
    if (rc != PROM_OK) return rc;
    plan_out->tiles_per_wave = L.nt;
    plan_out->pixel_tiles = L.pt;
    plan_out->workgroups = L.a.wg_per_chunk;
    plan_out->row_waves = L.a.cw;
    plan_out->k_outer = L.gemm ? 1 : 0;
    if (load_bytes_out) *load_bytes_out = L.xmode;
    return PROM_OK;
}

namespace prom {

// A layer can join a batched launch if the streaming kernel takes it with 16-byte loads, every
// chunk row is whole 16-byte pieces, and it is small enough that its own launch would be
// dominated by fixed costs.
constexpr long long kBatchMaxBytes = 32LL << 20;
constexpr long long kBatchBytesPerWg = 256LL << 10;  // bytes the first workgroups of a batch move (later ones less)
constexpr long long kBatchRefWork = 300LL << 20;     // launches with at least this much work take pieces of that size
constexpr long long kBigRefWork = 400LL << 20;       // the same for the launch of large layers

// Factor on the piece size (bytes or time per workgroup) of a shared launch with `work` bytes.
static double launch_scale(long long work, long long ref_work)
{
    // (proportional: with the square or the cube of the ratio the MobileNetV2 sweep at batch 32
    // takes 97 and 116 us instead of 81, at batch 64 125 and 141 instead of 128)
    const double s = (double)work / (double)ref_work;
    return s >= 1.0 ? 1.0 : (s < 0.0625 ? 0.0625 : s);
}

static bool batchable(const PwLaunch &L)
{
    const PwArgs &a = L.a;
    if (!L.fast || L.gemm || L.mode != 0 || a.K % 16 != 0 || a.Nc % 16 != 0) return false;
    if (batch_nt(a) * a.KS * 1024 > kLdsBudget) return false;
    const long long bytes = (long long)a.M * (a.K + a.Nc);
    if (bytes <= kBatchMaxBytes) return true;
    // larger layers too, up to four times that, when the launch of the large layers has no body for
    // their plan: alone in a sequence of independent layers they would stream at their own
    // launch's pace (batch 256: eight layers of MobileNetV2, 2.5 TB/s one by one)
    // Only layers with a small weight matrix: the bodies of the shared launch re-read the
    // activations once per chunk of output channels, which wide layers with many input channels
    // (ResNeXt: 256 -> 512 at 28x28) pay for; those are faster alone.
    const bool has_big_body = L.big_body >= 0 && L.lds <= (size_t)kLdsBudget;
    return !has_big_body && bytes <= 4 * kBatchMaxBytes && (long long)a.K * a.Nc <= 64 * 1024;
}

struct Range { uintptr_t lo, hi; };
static bool hits(const Range &p, const Range &q) { return p.lo < q.hi && q.lo < p.hi; }

// true if running `b` concurrently with `a` could change a result: one writes what the other
// reads or writes
static bool conflicts(const PwArgs &a, const PwArgs &b)
{
    const Range ya{(uintptr_t)a.y, (uintptr_t)a.y + (size_t)a.M * a.Nc};
    const Range yb{(uintptr_t)b.y, (uintptr_t)b.y + (size_t)b.M * b.Nc};
    const Range xa{(uintptr_t)a.x, (uintptr_t)a.x + (size_t)a.M * a.K};
    const Range xb{(uintptr_t)b.x, (uintptr_t)b.x + (size_t)b.M * b.K};
    if (hits(ya, yb) || hits(ya, xb) || hits(yb, xa)) return true;
    if (b.residual && hits(ya, Range{(uintptr_t)b.residual, (uintptr_t)b.residual + (size_t)b.M * b.Nc})) return true;
    if (a.residual && hits(yb, Range{(uintptr_t)a.residual, (uintptr_t)a.residual + (size_t)a.M * a.Nc})) return true;
    // parameters and weights are read-only inputs: a layer writing into another's weights is
    // not something the single-layer entry point allows either, but stay safe
    const Range wa{(uintptr_t)a.wq, (uintptr_t)a.wq + (size_t)a.Nc * a.KW * 4};
    const Range wb{(uintptr_t)b.wq, (uintptr_t)b.wq + (size_t)b.Nc * b.KW * 4};
    if (hits(ya, wb) || hits(yb, wa)) return true;
    // ... nor into another's requantisation parameters
    auto writes_params = [](const Range &y, const PwArgs &p) {
        const int32_t *arrs[4] = {p.bias, p.mult, p.shift, p.mult_neg};
        for (const int32_t *q : arrs)
            if (q && hits(y, Range{(uintptr_t)q, (uintptr_t)q + (size_t)p.Nc * 4})) return true;
        return false;
    };
    return writes_params(ya, b) || writes_params(yb, a);
}

// Sub-chunks (64 output channels) per part if the layer is one for pw_expand_body, else 0:
// 1, 2, 3 or 5 k steps (the bodies that are compiled), whole sub-chunks, no residual, and fewer
// passes over the activations than the streaming body's chunks would make.
static int expand_plan(const PwArgs &m, int *nparts)
{
    if (m.residual || m.Nc % 64 != 0 || (m.KS > 3 && m.KS != 5) || m.K % 16 != 0) return 0;
    const int sc_total = m.Nc / 64;
    int nmax = 1;
    while (nmax < sc_total && lds_bytes_expand(nmax + 1, m.KS) <= (size_t)kExpandLds) ++nmax;
    const int parts = (sc_total + nmax - 1) / nmax;
    const int nt = batch_nt(m);
    const int chunks = (m.Nc / 16 + nt - 1) / nt;
    if (parts >= chunks) return 0;
    *nparts = parts;
    return (sc_total + parts - 1) / parts;
}

// Plan of a batch member for pw_wreg_body (weights in registers, activations through LDS), if its
// shape is one the compiled bodies take (6, 9 or 15 k steps, no PReLU).  Measured on the launch of
// the 28 small MobileNetV2 layers at batch 128 (per-workgroup timeline): 384 -> 96 moves 7.3
// instead of 4.7 GB/s per workgroup, 576 -> 96 6.1 instead of 4.0, 960 -> 160 3.9-4.7 instead of
// 1.7, and the layers that were one chunk anyway (384 -> 64) gain from the coalesced loads.
struct WregPlan { int body, ntw, la, groups; };
static bool wreg_plan(const PwArgs &m, WregPlan *p)
{
    if (m.K % 16 != 0 || m.Nc % 16 != 0 || m.mult_neg) return false;
    const int tiles = m.Nc / 16;
    switch (m.KS) {
    case 6: p->ntw = tiles <= 4 ? 1 : 2; p->la = 3; p->body = tiles <= 4 ? kWreg6x1 : kWreg6x2; break;
    case 9: p->ntw = tiles <= 8 ? 2 : 3; p->la = 2; p->body = tiles <= 8 ? kWreg9x2 : kWreg9x3; break;
    case 15: p->ntw = 3; p->la = 1; p->body = kWreg15x3; break;
    default: return false;
    }
    p->groups = (tiles + 4 * p->ntw - 1) / (4 * p->ntw);
    return true;
}

// A member of the launch of small layers, re-planned for the bodies of pw_small_member: PT = 1,
// plain streaming (measured: the row-cooperative form gains nothing inside a shared launch, where
// fixed costs per workgroup and the balance between layers decide), or one of the bodies for
// expansion layers and deep projections.
struct SmallPlan {
    PwArgs a;
    size_t lds;
    long long work;        // bytes one chunk (part, group) moves
    long long unit_bytes;  // bytes of one unit of a body with large units, else 0
    int la;                // weights-in-registers body: steps per round of its prefetch ring, else 0
};

static void plan_small_shape(const PwLaunch &m, SmallPlan &sp)
{
    PwArgs &a = sp.a;
    a = m.a;
    a.cw = 0;
    sp.unit_bytes = 0;
    sp.la = 0;
    const int n_tiles = (a.Nc + 15) / 16;
    const int nt = batch_nt(a);
    int parts = 0;
    const int nsc = expand_plan(a, &parts);
    const bool full_rows = nsc && parts == 1 && a.KS == 1 &&
                           lds_bytes_expand_rows(nsc, 4, kExpandRowsG1, a.Nc) <= (size_t)kExpandLds;
    WregPlan wp;
    if (wreg_plan(a, &wp)) {
        // weights in registers: a workgroup belongs to one group of 64*ntw channels and walks
        // over 16-pixel tiles, all four wavefronts on the same tile
        a.cw = -10 - wp.body;
        a.n_chunks = wp.groups;
        a.units = (a.M + 15) / 16;
        const int gw = 64 * wp.ntw < a.Nc ? 64 * wp.ntw : a.Nc;
        sp.work = (long long)a.M * (a.K + gw);
        sp.lds = lds_bytes_wreg(a.K, wp.ntw);
        sp.la = wp.la;
    } else if (full_rows) {
        // all output channels in one part and a unit's rows small enough for LDS: whole rows
        a.cw = -1;
        a.n_chunks = 1;
        a.units = (a.M + 16 * kExpandRowsG1 - 1) / (16 * kExpandRowsG1);
        sp.work = (long long)a.M * (a.K + a.Nc);
        sp.lds = lds_bytes_expand_rows(nsc, 4, kExpandRowsG1, a.Nc);
        sp.unit_bytes = 16LL * kExpandRowsG1 * (a.K + a.Nc);
    } else if (nsc) {
        a.cw = nsc;
        a.n_chunks = parts;
        a.units = (a.M + 16 * expand_g(a.KS) - 1) / (16 * expand_g(a.KS));
        sp.work = (long long)a.M * (a.K + 64 * nsc);
        sp.lds = lds_bytes_expand(nsc, a.KS);
        sp.unit_bytes = 16LL * expand_g(a.KS) * (a.K + 64 * nsc);
    } else {
        a.n_chunks = (n_tiles + nt - 1) / nt;
        a.units = (a.M + 15) / 16;
        sp.work = (long long)a.M * (a.K + 16 * nt);
        sp.lds = lds_bytes_fast(nt, a.KS);
    }
}

// Workgroups of a planned member that move about per_wg bytes each; returns its workgroups in the
// launch (a multiple of 8).
static int size_small_member(SmallPlan &sp, long long per_wg)
{
    PwArgs &a = sp.a;
    const bool wreg = a.cw <= -10;
    const long long wg_units = wreg ? a.units : (a.units + 3) / 4;
    long long wgs = (sp.work + per_wg - 1) / per_wg;
    if (wreg) {
        // whole rounds of the prefetch ring: every workgroup the same number of steps
        long long tiles_per_wg = (a.units + wgs - 1) / wgs;
        tiles_per_wg = (tiles_per_wg + sp.la - 1) / sp.la * sp.la;
        wgs = (a.units + tiles_per_wg - 1) / tiles_per_wg;
    } else if (sp.unit_bytes) {
        // units are large here (16*G pixels x all channels of the part): give every wavefront
        // the same whole number of them
        long long upw = (per_wg + 2 * sp.unit_bytes) / (4 * sp.unit_bytes);
        if (upw < 1) upw = 1;
        wgs = (a.units + 4 * upw - 1) / (4 * upw);
    }
    if (wgs < 1) wgs = 1;
    if (wgs > wg_units) wgs = wg_units;
    a.wg_per_chunk = (int)wgs;
    return (int)((wgs * a.n_chunks + 7) / 8 * 8);
}

static int launch_batch(const PwLaunch *const *members, int count, hipStream_t st)
{
    static thread_local PwBatchArgs b;
    static thread_local SmallPlan plans[kMaxBatch];
    b.count = count;
    size_t lds = 0;
    int start = 0;
    // Work of a member = bytes its chunks move (activations are read once per chunk).  The members
    // are independent, so their order in the table is the library's: ascending by work.  The smallest
    // layers are bound by latency (every workgroup pays 2 to 4 us for its weights before it moves
    // 64 to 256 KB); dispatched last they leave the memory system idle while the launch drains,
    // dispatched first their latencies hide behind the streaming layers that follow (the MobileNetV2
    // sweep at batch 128: 213.6 us per step against 221.5 in network order, where the 7x7 layers
    // come last; descending order 222.7).  Workgroups are dispatched in table order: the first ones
    // get large pieces (each workgroup pays one cold round trip for its weights and first loads
    // before it streams), the last ones small pieces so that the chip drains evenly at the end of
    // the launch.
    long long total_work = 0, done_work = 0;
    int order[kMaxBatch];
    for (int i = 0; i < count; ++i) {
        plan_small_shape(*members[i], plans[i]);
        total_work += plans[i].work * plans[i].a.n_chunks;
        order[i] = i;
    }
    std::stable_sort(order, order + count, [&](int p, int q) {
        return plans[p].work * plans[p].a.n_chunks < plans[q].work * plans[q].a.n_chunks;
    });
    // The piece sizes were chosen on a launch of some 400 MB (about 100 us); a launch with less work
    // takes proportionally smaller pieces, or a few long workgroups would be all of it.
    const double scale = launch_scale(total_work, kBatchRefWork);
    const long long first_wg = (long long)(kBatchBytesPerWg * scale);
    for (int k = 0; k < count; ++k) {
        SmallPlan &sp = plans[order[k]];
        const long long per_wg = done_work * 10 < total_work * 7   ? first_wg
                                 : done_work * 10 < total_work * 9 ? first_wg / 2
                                                                   : first_wg / 4;
        done_work += sp.work * sp.a.n_chunks;
        const int nblk = size_small_member(sp, per_wg);
        b.layer[k] = sp.a;
        b.start[k] = start;
        start += nblk;
        if (sp.lds > lds) lds = sp.lds;
    }
    b.start[count] = start;
    bool any_prelu = false;
    for (int i = 0; i < count; ++i) any_prelu |= members[i]->a.mult_neg != nullptr;
    const PwBatchFn fn = any_prelu ? &pw_batch_kernel<kEpiBoth> : &pw_batch_kernel<kEpiPlain>;
    if (resident_workgroups(reinterpret_cast<KernelFn>(fn), lds) < 1) return PROM_EHIP;
    clear_hip_error();
    void *kargs[] = {&b};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(fn), dim3(start), dim3(256), kargs, lds, st);
    if (e != hipSuccess) {
        last_hip_error() = e;
        (void)hipGetLastError();
        return PROM_EHIP;
    }
    return check_launch();
}

// A large layer can join the launch of large layers if pw_bigbatch_kernel carries the body of its plan.
constexpr long long kBigBytesPerWg = 768LL << 10;  // measured best of 128 KB .. 2 MB on the MobileNetV2 head
constexpr double kBigWgMicros = 60.0;              // workgroup time aimed at where the body's speed is known
static bool big_batchable(const PwLaunch &L)
{
    return L.fast && !L.gemm && L.mode == 0 && L.big_body >= 0 && !batchable(L) && L.lds <= (size_t)kLdsBudget;
}

static int launch_big(const PwLaunch *const *members, int count, hipStream_t st)
{
    static thread_local PwBatchArgs b;
    b.count = count;
    size_t lds = 0;
    int start = 0;
    long long total_work = 0, done_work = 0;
    for (int i = 0; i < count; ++i) {
        const PwLaunch &L = *members[i];
        const int width = 16 * L.nt * (L.rows ? L.a.cw : 1);
        total_work += (long long)L.a.M * (L.a.K + width) * L.a.n_chunks;
    }
    // (workgroup sizes below were measured on a launch of 500 MB; less work, smaller pieces)
    const double scale = launch_scale(total_work, kBigRefWork);
    const long long big_wg = (long long)(kBigBytesPerWg * scale);
    const double wg_micros = kBigWgMicros * scale;
    for (int i = 0; i < count; ++i) {
        const PwLaunch &L = *members[i];
        PwArgs a = L.a;  // keeps its own plan (tiles, pixel tiles, chunks); only the grid changes
        const int width = 16 * L.nt * (L.rows ? a.cw : 1);
        const long long work = (long long)a.M * (a.K + width);
        int per_step = L.rows ? rows_groups(a.cw) : 4;
        int replanned = 0;
        const int body = pw_big_replan(L.big_body, a, &replanned);
        if (replanned) per_step = replanned;
        const long long wg_units = (a.units + per_step - 1) / per_step;
        const long long per_wg = done_work * 10 < total_work * 8   ? big_wg
                                 : done_work * 20 < total_work * 19 ? big_wg / 2
                                                                    : big_wg / 4;
        done_work += work * a.n_chunks;
        long long wgs = (work + per_wg - 1) / per_wg;
        // Bodies differ in speed (3 to 18 ns per pixel and workgroup), and workgroups of equal
        // bytes then end the launch with the slow ones still running: where the body's speed is
        // known, size by time instead -- 60 us for the first 70 % of the work, 30 us after it
        // (swept 30-100 us and 60-100 %: 116-118 us against 121-122 for the launch of the six
        // MobileNetV2 head layers).
        // (the figures were taken with 1 to 3 k steps; a deeper layer keeps the byte rule)
        const double ns = a.KS <= 3 ? pw_big_body_ns_per_pixel(body) : 0.0;
        if (ns > 0) {
            const bool early = (done_work - work * a.n_chunks) * 10 < total_work * 7;
            wgs = (long long)((double)a.M * ns / ((early ? wg_micros : wg_micros / 2) * 1000.0) + 0.999);
        }
        if (wgs < 1) wgs = 1;
        if (wgs > wg_units) wgs = wg_units;
        a.wg_per_chunk = (int)wgs;
        const int nblk = (int)((wgs * a.n_chunks + 7) / 8 * 8);
        b.layer[i] = a;
        b.body[i] = (unsigned char)body;
        b.start[i] = start;
        start += nblk;
        const size_t l = pw_big_body_lds(body, a);
        if (l > lds) lds = l;
    }
    b.start[count] = start;
    bool any_prelu = false;
    for (int i = 0; i < count; ++i) any_prelu |= members[i]->a.mult_neg != nullptr;
    const PwBatchFn fn = pw_bigbatch_fn(any_prelu);
    if (resident_workgroups(reinterpret_cast<KernelFn>(fn), lds) < 1) return PROM_EHIP;
    clear_hip_error();
    void *kargs[] = {&b};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(fn), dim3(start), dim3(256), kargs, lds, st);
    if (e != hipSuccess) {
        last_hip_error() = e;
        (void)hipGetLastError();
        return PROM_EHIP;
    }
    return check_launch();
}

}  // namespace prom

#ifdef PROM_TIMELINE
extern "C" int prom_debug_set_stamp_buffer(void *dev_buf)
{
    prom::debug_stamp_buffer() = static_cast<int32_t *>(dev_buf);
    return PROM_OK;
}
extern "C" int prom_debug_mark(void *dev_buf, int slot, void *stream)
{
    hipLaunchKernelGGL(prom::debug_mark_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(stream),
                       static_cast<unsigned long long *>(dev_buf), slot);
    return PROM_OK;
}

// Copies the timeline of the last launch of small layers to the host: t[2*i], t[2*i+1] = start
// and end clock of workgroup i (0 if it never ran), member[i] = its layer.  Synchronises the device.
extern "C" int prom_debug_timeline(unsigned long long *t_host, int *member_host, int n)
{
    if (!t_host || !member_host || n <= 0 || n > prom::kTimelineMax) return PROM_EINVAL;
    if (hipDeviceSynchronize() != hipSuccess) return PROM_EHIP;
    if (hipMemcpyFromSymbol(t_host, HIP_SYMBOL(prom::g_timeline), sizeof(unsigned long long) * 2 * n) != hipSuccess)
        return PROM_EHIP;
    if (hipMemcpyFromSymbol(member_host, HIP_SYMBOL(prom::g_timeline_member), sizeof(int) * n) != hipSuccess)
        return PROM_EHIP;
    static unsigned long long zeros[2 * prom::kTimelineMax];
    if (hipMemcpyToSymbol(HIP_SYMBOL(prom::g_timeline), zeros, sizeof(zeros)) != hipSuccess) return PROM_EHIP;
    return PROM_OK;
}
#endif

int prom::pw_shape_check(int n, int h, int w, int cin, int cout)
{
    PwLaunch L;
    return pw_prepare(nullptr, n, h, w, cin, nullptr, cout, nullptr, nullptr, nullptr, nullptr, nullptr, 0, true, L);
}

extern "C" int prom_pw_batchable(int n, int h, int w, int cin, int cout)
{
    prom::PwLaunch L;
    const int rc = prom::pw_prepare(nullptr, n, h, w, cin, nullptr, cout, nullptr, nullptr, nullptr,
                                    nullptr, nullptr, 0, true, L);
    if (rc != PROM_OK) return rc;
    return prom::batchable(L) ? 1 : 0;
}

extern "C" int prom_pw_batch_class(int n, int h, int w, int cin, int cout)
{
    prom::PwLaunch L;
    const int rc = prom::pw_prepare(nullptr, n, h, w, cin, nullptr, cout, nullptr, nullptr, nullptr,
                                    nullptr, nullptr, 0, true, L);
    if (rc != PROM_OK) return rc;
    return prom::batchable(L) ? 1 : (prom::big_batchable(L) ? 2 : 0);
}

extern "C" int prom_pw_conv_sequence(const prom_pw_layer_t *layers, int count, int *bad_layer, void *stream)
{
    using namespace prom;
    if (!layers || count <= 0) return PROM_EINVAL;
    constexpr int kMaxSeq = 256;
    if (count > kMaxSeq) return PROM_EUNSUPPORTED;
    static thread_local PwLaunch plans[kMaxSeq];
    for (int i = 0; i < count; ++i) {
        const prom_pw_layer_t &l = layers[i];
        const int rc = pw_prepare(l.x, l.n, l.h, l.w, l.cin, l.w_packed, l.cout, &l.rq, l.residual,
                                  l.y, nullptr, nullptr, 0, false, plans[i]);
        if (rc != PROM_OK) {
            if (bad_layer) *bad_layer = i;
            return rc;
        }
    }
    // Results are those of running the layers one after the other.  Layers that do not touch each
    // other's data wait in one of two pending batches -- small layers (pw_batch_kernel) and large
    // layers whose plan pw_bigbatch_kernel carries -- and each batch becomes one launch where its
    // layers run concurrently.  A layer that conflicts with a pending one forces both batches out
    // first; any other layer that fits no batch is launched at once and may overtake them.
    hipStream_t st = static_cast<hipStream_t>(stream);
    // (Small layers wait for up to two launches' worth: a network with more independent small
    // layers than a launch holds is then not cut in sequence order, which would put its last, smallest
    // layers -- one latency chain per workgroup -- in a launch of their own, but dealt out by size, so
    // that each launch has large layers to stream behind its small ones.  RegNetX-400MF's 48 layers
    // at batch 128: two launches of 24 instead of the first 32 and the last 16.)
    constexpr int kMaxPending = 2 * kMaxBatch;
    const PwLaunch *pending[2][kMaxPending];
    int npending[2] = {0, 0};
    int first_pending[2] = {0, 0};
    auto flush_one = [&](int c) -> int {
        int rc = PROM_OK;
        if (npending[c] == 1) {
            rc = pw_launch(*pending[c][0], st);
        } else if (npending[c] > kMaxBatch) {
            std::stable_sort(pending[c], pending[c] + npending[c], [](const PwLaunch *p, const PwLaunch *q) {
                return (long long)p->a.M * (p->a.K + p->a.Nc) < (long long)q->a.M * (q->a.K + q->a.Nc);
            });
            const PwLaunch *half[2][kMaxBatch];
            int nhalf[2] = {0, 0};
            for (int k = 0; k < npending[c]; ++k) half[k & 1][nhalf[k & 1]++] = pending[c][k];
            for (int h = 0; h < 2 && rc == PROM_OK; ++h) rc = launch_batch(half[h], nhalf[h], st);
        } else if (npending[c] > 1) {
            rc = c == 0 ? launch_batch(pending[c], npending[c], st) : launch_big(pending[c], npending[c], st);
        }
        npending[c] = 0;
        if (rc != PROM_OK && bad_layer) *bad_layer = first_pending[c];
        return rc;
    };
    auto flush_all = [&]() -> int {
        // the large layers first: they were written first in the usual order of a network, and the
        // small batch then fills the chip while they drain
        const int rc = flush_one(1);
        if (rc != PROM_OK) return rc;
        return flush_one(0);
    };
    for (int i = 0; i < count; ++i) {
        const int cls = batchable(plans[i]) ? 0 : (big_batchable(plans[i]) ? 1 : -1);
        bool clash = false;
        for (int c = 0; c < 2 && !clash; ++c)
            for (int k = 0; k < npending[c] && !clash; ++k) clash = conflicts(pending[c][k]->a, plans[i].a);
        if (clash) {
            const int rc = flush_all();
            if (rc != PROM_OK) return rc;
        }
        if (cls >= 0) {
            if (npending[cls] == (cls == 0 ? kMaxPending : kMaxBatch)) {
                const int rc = flush_one(cls);
                if (rc != PROM_OK) return rc;
            }
            if (npending[cls] == 0) first_pending[cls] = i;
            pending[cls][npending[cls]++] = &plans[i];
        } else {
            const int rc = pw_launch(plans[i], st);
            if (rc != PROM_OK) {
                if (bad_layer) *bad_layer = i;
                return rc;
            }
        }
    }
    return flush_all();
}

extern "C" int prom_copy_bytes(const void *src, void *dst, size_t nbytes, void *stream)
{
    if (!src || !dst || nbytes == 0 || (nbytes & 15) != 0) return PROM_EINVAL;
    if ((((uintptr_t)src | (uintptr_t)dst) & 15) != 0) return PROM_EINVAL;
    const long long n16 = (long long)(nbytes / 16);
    long long blocks = (n16 + 255) / 256;
    if (blocks > prom::kNumCU * 4) blocks = prom::kNumCU * 4;  // measured best of 1 to 64 workgroups per CU (5.6 against 4.6 TB/s at 16)
    prom::clear_hip_error();
    hipLaunchKernelGGL(prom::copy_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const prom::v4i *>(src),
                       static_cast<prom::v4i *>(dst), n16);
    return prom::check_launch();
}

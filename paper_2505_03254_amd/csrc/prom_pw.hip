// Ternary pointwise 1x1 convolution on gfx950: int8 MFMA over weights decoded from 2-bit
// codes into LDS, activations streamed from HBM straight into the MFMA operand registers,
// exact integer requantisation in the epilogue.
//
// Formulation.  The layer is Y[m][co] = sum_k X[m][k] * W[co][k]  (paper Section 2: a sum of
// input channels; Section 3.1: convolve with the ternary weights, rescale afterwards).  The
// kernel computes the transpose, D = W_tile (16 channels x 64 k) * X_tile^T (64 k x 16 pixels)
// with v_mfma_i32_16x16x64_i8, because then
//   - the B operand of lane l is 16 consecutive k-bytes of pixel (l & 15): one 16-byte global
//     load from the NHWC row, no LDS staging of activations;
//   - the D registers of lane l are 4 consecutive output channels of pixel (l & 15): one
//     packed dword of int8 outputs, and per-lane requantisation parameters.
// A wavefront owns NT 16-channel tiles (a "chunk" of 16*NT output channels) and walks over
// pixel tiles; the 4 wavefronts of a workgroup share the decoded weights of the chunk.
#include "prom.h"
#include "prom_device.h"
#include "prom_launch.h"

namespace prom {

struct PwArgs {
    const int8_t *x;
    const uint32_t *wq;
    const int32_t *bias;
    const int32_t *mult;
    const int32_t *shift;
    const int8_t *residual;
    int8_t *y;
    int32_t *acc_out;
    long long M;      // pixels
    long long units;  // pixel groups of 64*PT pixels (one per workgroup iteration)
    int K, Nc;
    int KW;           // packed 32-bit words per weight row = ceil(K/16)
    int KS;           // 64-wide k steps = ceil(K/64)
    int n_chunks;     // output-channel chunks of 16*NT channels
    int wg_per_chunk;
    int lo_b, hi_b;   // activation window + kQBias
};

// Tiles of a chunk are stored in groups of 4, then 2, then 1 so that a lane's outputs of a
// group are 16, 8 or 4 contiguous bytes and the four lane groups of a pixel write one
// contiguous 64/32/16-byte segment.
template <int NT> __host__ __device__ constexpr int grp_size(int t)
{
    return t < 4 * (NT / 4) ? 4 : (((NT % 4) >= 2 && t < 4 * (NT / 4) + 2) ? 2 : 1);
}
template <int NT> __host__ __device__ constexpr int grp_first(int t)
{
    return t < 4 * (NT / 4) ? (t & ~3)
           : (((NT % 4) >= 2 && t < 4 * (NT / 4) + 2) ? 4 * (NT / 4)
                                                       : 4 * (NT / 4) + ((NT % 4) >= 2 ? 2 : 0));
}
// Channel (relative to the chunk base) held in D row 4*gr + r of tile slot t.
template <int NT> __host__ __device__ constexpr int chan_of(int t, int gr, int r)
{
    return 16 * grp_first<NT>(t) + 4 * grp_size<NT>(t) * gr + 4 * (t - grp_first<NT>(t)) + r;
}

// One lane's 16 k-bytes of pixel m starting at k = koff; zero beyond M or K.
template <int XMODE>
__device__ __forceinline__ v4i load_frag(const int8_t *__restrict__ x, long long m, long long M,
                                         int koff, int K)
{
    v4i f = {0, 0, 0, 0};
    if (m >= M) return f;
    const int8_t *p = x + m * (long long)K + koff;
    if constexpr (XMODE == 16) {
        if (koff < K) f = *reinterpret_cast<const v4i_a4 *>(p);
    } else if constexpr (XMODE == 8) {
        if (koff + 8 <= K) {
            const v2i lo = *reinterpret_cast<const v2i_a4 *>(p);
            f[0] = lo[0];
            f[1] = lo[1];
        }
        if (koff + 16 <= K) {
            const v2i hi = *reinterpret_cast<const v2i_a4 *>(p + 8);
            f[2] = hi[0];
            f[3] = hi[1];
        }
    } else {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t v = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int k = koff + 4 * d + b;
                if (k < K) v |= (uint32_t)(uint8_t)p[4 * d + b] << (8 * b);
            }
            f[d] = (int)v;
        }
    }
    return f;
}

// 16 two-bit codes (layout of prom_pack_ternary) -> 16 int8 weights in MFMA operand order.
__device__ __forceinline__ v4i decode_word(uint32_t word)
{
    v4i f;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        // code c in {0,1,3} -> byte selector 2c in {0,2,6} of the 8-byte table below
        const uint32_t sel = ((word >> (2 * d)) & 0x03030303u) << 1;
        // table bytes: [0]=0x00 (zero), [2]=0x01 (+1), [6]=0xFF (-1)
        f[d] = (int)__builtin_amdgcn_perm(0x00FF0000u, 0x00010000u, sel);
    }
    return f;
}

template <int NT, int PT, int XMODE, bool BYTEWISE, bool RAW>
__global__ __launch_bounds__(256) void pw_kernel(const PwArgs a)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    v4i *frag = reinterpret_cast<v4i *>(lds_raw);  // [NT][KS][64 lanes] decoded A operands

    set_f64_round_down();

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int j = lane & 15;  // pixel within a 16-pixel tile
    const int g = lane >> 4;  // k group on the input side, channel group on the output side

    // Consecutive workgroup ids go round-robin over the 8 XCDs; make logical neighbours
    // (the chunks of one pixel range) land on the same XCD so they share its L2.
    const int nblk = gridDim.x;  // multiple of 8
    const int lid = (blockIdx.x & 7) * (nblk >> 3) + (blockIdx.x >> 3);
    const int chunk = lid % a.n_chunks;
    const int wg = lid / a.n_chunks;
    if (wg >= a.wg_per_chunk) return;
    const int cbase = chunk * NT * 16;
    const int KS = a.KS;

    // ---- decode this chunk's weights into LDS -------------------------------------------
    const int nfrag = NT * KS * 64;
    for (int idx = tid; idx < nfrag; idx += 256) {
        const int l = idx & 63;
        const int tk = idx >> 6;
        const int ks = tk % KS;
        const int t = tk / KS;
        const int i = l & 15;
        const int c = cbase + chan_of<NT>(t, i >> 2, i & 3);
        const int kw = 4 * ks + (l >> 4);
        uint32_t word = 0;
        if (c < a.Nc && kw < a.KW) word = a.wq[(long long)c * a.KW + kw];
        frag[idx] = decode_word(word);
    }

    // ---- per-lane requantisation parameters: 4 channels per tile slot --------------------
    double scale[NT][4];
    v4i biasv[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int c = cbase + chan_of<NT>(t, g, r);
            int b = 0;
            double s = 0.0;
            if (!RAW && c < a.Nc) {
                b = a.bias[c];
                s = make_scale(a.mult[c], a.shift[c]);
            }
            biasv[t][r] = b;
            scale[t][r] = s;
        }
    }
    __syncthreads();

    const long long W = a.wg_per_chunk;
    const int koff0 = 16 * g;
    auto load_b = [&](v4i(&b)[PT], long long u, int ks) {
        const long long mb = (u * 4 + wave) * (16 * PT) + j;
#pragma unroll
        for (int p = 0; p < PT; ++p)
            b[p] = load_frag<XMODE>(a.x, mb + 16 * p, a.M, 64 * ks + koff0, a.K);
    };

    v4i bcur[PT], bnxt[PT];
    long long u = wg;
    if (u < a.units) load_b(bcur, u, 0);

    for (; u < a.units; u += W) {
        v4i acc[PT][NT];
#pragma unroll
        for (int p = 0; p < PT; ++p)
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[p][t] = biasv[t];

        for (int ks = 0; ks < KS; ++ks) {
            if (ks + 1 < KS) {
                load_b(bnxt, u, ks + 1);
            } else if (u + W < a.units) {
                load_b(bnxt, u + W, 0);
            } else {
#pragma unroll
                for (int p = 0; p < PT; ++p) bnxt[p] = v4i{0, 0, 0, 0};
            }
            const v4i *fk = frag + ks * 64 + lane;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const v4i wfrag = fk[t * KS * 64];
#pragma unroll
                for (int p = 0; p < PT; ++p)
                    acc[p][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wfrag, bcur[p], acc[p][t], 0, 0, 0);
            }
#pragma unroll
            for (int p = 0; p < PT; ++p) bcur[p] = bnxt[p];
        }

        // ---- epilogue ---------------------------------------------------------------------
#pragma unroll
        for (int p = 0; p < PT; ++p) {
            const long long m = (u * 4 + wave) * (16 * PT) + 16 * p + j;
            const bool mvalid = m < a.M;
            const long long rowoff = m * (long long)a.Nc;
#pragma unroll
            for (int t0 = 0; t0 < NT; t0 += grp_size<NT>(t0)) {
                constexpr int dummy = 0;
                (void)dummy;
                const int S = grp_size<NT>(t0);
                const int c0 = cbase + chan_of<NT>(t0, g, 0);  // lane's first channel of the group
                if constexpr (RAW) {
#pragma unroll
                    for (int tt = 0; tt < 4; ++tt) {
                        if (tt < S) {
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const int c = c0 + 4 * tt + r;
                                if (mvalid && c < a.Nc) a.acc_out[rowoff + c] = acc[p][t0 + tt][r];
                            }
                        }
                    }
                } else if constexpr (BYTEWISE) {
#pragma unroll
                    for (int tt = 0; tt < 4; ++tt) {
                        if (tt < S) {
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const int c = c0 + 4 * tt + r;
                                if (mvalid && c < a.Nc) {
                                    int v = requant_to_biased(acc[p][t0 + tt][r], scale[t0 + tt][r],
                                                              a.lo_b, a.hi_b);
                                    if (a.residual)
                                        v = min(max(v + (int)a.residual[rowoff + c], kQBias - 128),
                                                kQBias + 127);
                                    a.y[rowoff + c] = (int8_t)(v - kQBias);
                                }
                            }
                        }
                    }
                } else {
                    // Nc % 4 == 0: every dword of 4 channels is entirely inside or outside.
                    uint32_t res[4] = {0, 0, 0, 0};
                    const bool wide = mvalid && (c0 + 4 * S <= a.Nc);
                    if (a.residual) {
                        const int8_t *rp = a.residual + rowoff + c0;
                        if (wide) {
                            if (S == 4) {
                                const v4i v = *reinterpret_cast<const v4i_a4 *>(rp);
                                res[0] = v[0]; res[1] = v[1]; res[2] = v[2]; res[3] = v[3];
                            } else if (S == 2) {
                                const v2i v = *reinterpret_cast<const v2i_a4 *>(rp);
                                res[0] = v[0]; res[1] = v[1];
                            } else {
                                res[0] = *reinterpret_cast<const uint32_t *>(rp);
                            }
                        } else if (mvalid) {
#pragma unroll
                            for (int tt = 0; tt < 4; ++tt)
                                if (tt < S && c0 + 4 * tt + 4 <= a.Nc)
                                    res[tt] = *reinterpret_cast<const uint32_t *>(rp + 4 * tt);
                        }
                    }
                    uint32_t out[4] = {0, 0, 0, 0};
#pragma unroll
                    for (int tt = 0; tt < 4; ++tt) {
                        if (tt < S) {
                            int v[4];
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                v[r] = requant_to_biased(acc[p][t0 + tt][r], scale[t0 + tt][r],
                                                         a.lo_b, a.hi_b);
                            if (a.residual) {
#pragma unroll
                                for (int r = 0; r < 4; ++r)
                                    v[r] = min(max(v[r] + sbyte(res[tt], r), kQBias - 128), kQBias + 127);
                            }
                            out[tt] = pack4_low_bytes(v[0], v[1], v[2], v[3]);
                        }
                    }
                    int8_t *yp = a.y + rowoff + c0;
                    if (wide) {
                        if (S == 4) {
                            *reinterpret_cast<v4i_a4 *>(yp) = v4i{(int)out[0], (int)out[1], (int)out[2], (int)out[3]};
                        } else if (S == 2) {
                            *reinterpret_cast<v2i_a4 *>(yp) = v2i{(int)out[0], (int)out[1]};
                        } else {
                            *reinterpret_cast<uint32_t *>(yp) = out[0];
                        }
                    } else if (mvalid) {
#pragma unroll
                        for (int tt = 0; tt < 4; ++tt)
                            if (tt < S && c0 + 4 * tt + 4 <= a.Nc)
                                *reinterpret_cast<uint32_t *>(yp + 4 * tt) = out[tt];
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------- host side
constexpr int kMaxCin = 4096;
constexpr int kLdsBudget = 64 * 1024;
constexpr int kNumCU = 256;

template <int NT, int PT, int XMODE, bool BYTEWISE, bool RAW>
static int launch_one(const PwArgs &a, int grid, size_t lds, hipStream_t st)
{
    clear_hip_error();
    hipLaunchKernelGGL((pw_kernel<NT, PT, XMODE, BYTEWISE, RAW>), dim3(grid), dim3(256), lds, st, a);
    return check_launch();
}

template <int NT, int XMODE>
static int launch_pt(const PwArgs &a, int pt, int grid, size_t lds, hipStream_t st)
{
    if (pt == 1) return launch_one<NT, 1, XMODE, false, false>(a, grid, lds, st);
    if constexpr (NT <= 6) {
        if (pt == 2) return launch_one<NT, 2, XMODE, false, false>(a, grid, lds, st);
    }
    if constexpr (NT <= 2) {
        if (pt == 4) return launch_one<NT, 4, XMODE, false, false>(a, grid, lds, st);
    }
    return PROM_EINVAL;
}

template <int XMODE>
static int launch_nt(const PwArgs &a, int nt, int pt, int grid, size_t lds, hipStream_t st)
{
    switch (nt) {
    case 1: return launch_pt<1, XMODE>(a, pt, grid, lds, st);
    case 2: return launch_pt<2, XMODE>(a, pt, grid, lds, st);
    case 3: return launch_pt<3, XMODE>(a, pt, grid, lds, st);
    case 4: return launch_pt<4, XMODE>(a, pt, grid, lds, st);
    case 5: return launch_pt<5, XMODE>(a, pt, grid, lds, st);
    case 6: return launch_pt<6, XMODE>(a, pt, grid, lds, st);
    case 7: return launch_pt<7, XMODE>(a, pt, grid, lds, st);
    case 8: return launch_pt<8, XMODE>(a, pt, grid, lds, st);
    case 9: return launch_pt<9, XMODE>(a, pt, grid, lds, st);
    case 10: return launch_pt<10, XMODE>(a, pt, grid, lds, st);
    case 11: return launch_pt<11, XMODE>(a, pt, grid, lds, st);
    case 12: return launch_pt<12, XMODE>(a, pt, grid, lds, st);
    default: return PROM_EINVAL;
    }
}

static bool overlaps(const void *p, size_t pn, const void *q, size_t qn)
{
    const uintptr_t a = (uintptr_t)p, b = (uintptr_t)q;
    return a < b + qn && b < a + pn;
}

static int max_pt_for(int nt) { return nt <= 2 ? 4 : (nt <= 6 ? 2 : 1); }

struct PwLaunch {
    PwArgs a;
    int nt, pt, xmode, grid;
    size_t lds;
    bool fast;
    int mode;
};

// Validate the arguments and fill the launch description.  mode: 0 = requantised int8
// output, 1 = raw int32 accumulators.  Launches nothing.
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
    a.shift = rq ? rq->shift : nullptr;
    a.residual = mode == 0 ? residual : nullptr;
    a.y = y;
    a.acc_out = acc_out;
    a.M = M;
    a.K = cin;
    a.Nc = cout;
    a.KW = (cin + 15) / 16;
    a.KS = (cin + 63) / 64;
    a.lo_b = (rq ? rq->act_min : 0) + kQBias;
    a.hi_b = (rq ? rq->act_max : 0) + kQBias;

    const int n_tiles = (cout + 15) / 16;
    const bool aligned = (((uintptr_t)x | (uintptr_t)y | (uintptr_t)residual) & 3) == 0;
    const bool fast = mode == 0 && aligned && (cin % 8 == 0) && (cout % 4 == 0);

    int nt, pt;
    if (!fast) {
        if (plan && (plan->tiles_per_wave || plan->pixel_tiles)) return PROM_EINVAL;
        nt = 4;
        pt = 1;
        if (nt * a.KS * 1024 > kLdsBudget) nt = kLdsBudget / (a.KS * 1024);
    } else {
        const int nt_lds = kLdsBudget / (a.KS * 1024);  // >= 1 since KS <= 64
        int nt_cap = nt_lds < 12 ? nt_lds : 12;
        if (plan && plan->tiles_per_wave) {
            if (plan->tiles_per_wave < 1 || plan->tiles_per_wave > nt_cap) return PROM_EINVAL;
            nt = plan->tiles_per_wave;
        } else {
            if (nt_cap > 9) nt_cap = 9;
            const int chunks = (n_tiles + nt_cap - 1) / nt_cap;
            nt = (n_tiles + chunks - 1) / chunks;
        }
        if (plan && plan->pixel_tiles) {
            pt = plan->pixel_tiles;
            if (!(pt == 1 || pt == 2 || pt == 4) || pt > max_pt_for(nt)) return PROM_EINVAL;
        } else {
            pt = nt <= 2 ? 4 : (nt <= 4 ? 2 : 1);
            while (pt > 1 && M < (long long)64 * pt * kNumCU) pt >>= 1;  // small layers: more units
        }
    }
    a.n_chunks = (n_tiles + nt - 1) / nt;
    a.units = (M + 64 * pt - 1) / (64 * pt);
    long long wgs;
    if (plan && plan->workgroups) {
        if (plan->workgroups < 1) return PROM_EINVAL;
        wgs = plan->workgroups;
    } else {
        wgs = (kNumCU * 4 + a.n_chunks - 1) / a.n_chunks;
    }
    if (wgs > a.units) wgs = a.units;
    a.wg_per_chunk = (int)wgs;
    const long long total = wgs * a.n_chunks;
    if (total > (1LL << 30)) return PROM_EUNSUPPORTED;
    L.grid = (int)((total + 7) / 8 * 8);
    L.lds = (size_t)nt * a.KS * 1024;
    L.nt = nt;
    L.pt = pt;
    L.fast = fast;
    L.mode = mode;
    L.xmode = !fast ? 1 : (cin % 16 == 0 ? 16 : 8);
    return PROM_OK;
}

static int pw_launch(const PwLaunch &L, hipStream_t st)
{
    const PwArgs &a = L.a;
    if (L.mode == 1) {
        switch (L.nt) {
        case 1: return launch_one<1, 1, 1, true, true>(a, L.grid, L.lds, st);
        case 2: return launch_one<2, 1, 1, true, true>(a, L.grid, L.lds, st);
        case 3: return launch_one<3, 1, 1, true, true>(a, L.grid, L.lds, st);
        default: return launch_one<4, 1, 1, true, true>(a, L.grid, L.lds, st);
        }
    }
    if (!L.fast) {
        switch (L.nt) {
        case 1: return launch_one<1, 1, 1, true, false>(a, L.grid, L.lds, st);
        case 2: return launch_one<2, 1, 1, true, false>(a, L.grid, L.lds, st);
        case 3: return launch_one<3, 1, 1, true, false>(a, L.grid, L.lds, st);
        default: return launch_one<4, 1, 1, true, false>(a, L.grid, L.lds, st);
        }
    }
    if (L.xmode == 16) return launch_nt<16>(a, L.nt, L.pt, L.grid, L.lds, st);
    return launch_nt<8>(a, L.nt, L.pt, L.grid, L.lds, st);
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

__global__ __launch_bounds__(256) void copy_kernel(const v4i *__restrict__ src, v4i *__restrict__ dst,
                                                   long long n16)
{
    const long long stride = (long long)gridDim.x * 256;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
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

extern "C" int prom_pw_plan_query(int n, int h, int w, int cin, int cout, prom_pw_plan_t *plan_out)
{
    if (!plan_out) return PROM_EINVAL;
    prom::PwLaunch L;
    const int rc = prom::pw_prepare(nullptr, n, h, w, cin, nullptr, cout, nullptr, nullptr, nullptr,
                                    nullptr, nullptr, 0, true, L);
    if (rc != PROM_OK) return rc;
    plan_out->tiles_per_wave = L.nt;
    plan_out->pixel_tiles = L.pt;
    plan_out->workgroups = L.a.wg_per_chunk;
    plan_out->reserved = L.xmode;
    return PROM_OK;
}

extern "C" int prom_pw_conv_sequence(const prom_pw_layer_t *layers, int count, int *bad_layer, void *stream)
{
    if (!layers || count <= 0) return PROM_EINVAL;
    constexpr int kMaxSeq = 256;
    if (count > kMaxSeq) return PROM_EUNSUPPORTED;
    static thread_local prom::PwLaunch plans[kMaxSeq];
    for (int i = 0; i < count; ++i) {
        const prom_pw_layer_t &l = layers[i];
        const int rc = prom::pw_prepare(l.x, l.n, l.h, l.w, l.cin, l.w_packed, l.cout, &l.rq, l.residual,
                                        l.y, nullptr, nullptr, 0, false, plans[i]);
        if (rc != PROM_OK) {
            if (bad_layer) *bad_layer = i;
            return rc;
        }
    }
    for (int i = 0; i < count; ++i) {
        const int rc = prom::pw_launch(plans[i], static_cast<hipStream_t>(stream));
        if (rc != PROM_OK) {
            if (bad_layer) *bad_layer = i;
            return rc;
        }
    }
    return PROM_OK;
}

extern "C" int prom_copy_bytes(const void *src, void *dst, size_t nbytes, void *stream)
{
    if (!src || !dst || nbytes == 0 || (nbytes & 15) != 0) return PROM_EINVAL;
    if ((((uintptr_t)src | (uintptr_t)dst) & 15) != 0) return PROM_EINVAL;
    const long long n16 = (long long)(nbytes / 16);
    long long blocks = (n16 + 255) / 256;
    if (blocks > prom::kNumCU * 16) blocks = prom::kNumCU * 16;
    prom::clear_hip_error();
    hipLaunchKernelGGL(prom::copy_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const prom::v4i *>(src),
                       static_cast<prom::v4i *>(dst), n16);
    return prom::check_launch();
}

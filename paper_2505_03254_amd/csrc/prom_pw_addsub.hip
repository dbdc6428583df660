// Design B of the pointwise layer, kept for the A/B measurement: multiplication-free
// accumulation on the vector ALU.  "A ternary weight turns the convolution into a sum of
// input channels" (paper Section 2) taken literally: for every output channel the kernel adds
// up the input bytes whose weight is +1 and those whose weight is -1 and subtracts the two.
//
// Mapping: one lane = one pixel (its cin bytes live in registers), 64 pixels per wavefront,
// output channels looped over; the weights of a channel are the same for all lanes, so they
// are kept as byte masks in LDS and read as broadcasts.  Four input channels are handled per
// pair of instructions: v_and_b32 (select the bytes whose weight has the wanted sign) and
// v_sad_u8 against zero (sum of the four selected bytes).  Inputs are biased to unsigned
// (x ^ 0x80 per byte); the 128*(#plus - #minus) this adds is folded into the channel constant.
// With lane = pixel no cross-lane reduction is needed; splitting cin across lanes instead
// would add a 6-step DPP reduction per output and is slower still.
//
// The epilogue (integer requantisation, LDS-staged coalesced stores) is the one of the MFMA
// kernel, so the two designs differ only in how the accumulators are produced.
#include "prom_pw_stream.h"
#include "prom_launch.h"

namespace prom {

struct AddSubArgs {
    const int8_t *x;
    const uint32_t *wq;
    const int32_t *bias;
    const int32_t *mult;
    const int32_t *shift;
    const int8_t *residual;
    int8_t *y;
    int M, K, Nc, KW;
    int CC;        // output channels per chunk (multiple of 16, or Nc)
    int n_chunks;
    int lo, hi;
};

// KD = dwords of input per pixel kept in registers (cin <= 4*KD).
template <int KD>
__global__ __launch_bounds__(256) void pw_addsub_kernel(const AddSubArgs a)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int K = a.K, Nc = a.Nc, CC = a.CC;
    const int KQ = (K + 3) / 4;                                  // 4-byte k groups
    v2i *masks = reinterpret_cast<v2i *>(lds_raw);               // [CC][KQ] (plus mask, minus mask)
    v4i *lpar = reinterpret_cast<v4i *>(masks + CC * KQ);        // [CC] (C lo, C hi, mult, shift)
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    unsigned char *stage = reinterpret_cast<unsigned char *>(lpar + CC) + wave * (64 * CC);  // [64 px][CC]

    const int chunk = blockIdx.y;
    const int cbase = chunk * CC;
    const int RW = min(CC, Nc - cbase);  // valid channels of this chunk (multiple of 4)

    // ---- masks and parameters of the chunk ---------------------------------------------------
    for (int idx = tid; idx < RW * KQ; idx += 256) {
        const int c = idx / KQ, q = idx - c * KQ;
        const uint32_t word = a.wq[(long long)(cbase + c) * a.KW + (q >> 2)];
        // codes of k = 4q..4q+3 sit at bits 8b + 2d with d = q & 3
        const uint32_t codes = (word >> (2 * (q & 3))) & 0x03030303u;
        const uint32_t nz = codes & 0x01010101u;           // bit 0: weight is not zero
        const uint32_t ng = (codes >> 1) & 0x01010101u;    // bit 1: weight is negative
        const uint32_t neg = ng * 0xFFu, pos = (nz & ~ng) * 0xFFu;
        masks[idx] = v2i{(int)pos, (int)neg};
    }
    for (int c = tid; c < RW; c += 256) {
        int npos = 0, nneg = 0;
        for (int kw = 0; kw < a.KW; ++kw) {
            const uint32_t word = a.wq[(long long)(cbase + c) * a.KW + kw];
            const uint32_t nz = word & 0x55555555u, ng = (word >> 1) & 0x55555555u;
            nneg += __builtin_popcount(ng);
            npos += __builtin_popcount(nz & ~ng);
        }
        const int pm = a.mult[cbase + c], ps = a.shift[cbase + c];
        // sums are taken over x+128: remove 128*(npos - nneg) together with the bias
        const long long b = (long long)a.bias[cbase + c] - 128LL * (npos - nneg);
        const long long C = b * pm + (1LL << (30 + ps));
        lpar[c] = v4i{(int)(uint32_t)C, (int)(C >> 32), pm, ps};
    }
    __syncthreads();

    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a.x), 0, a.M * K, kBufFlags);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, a.M * Nc, kBufFlags);
    const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.residual ? a.residual : a.y), 0, a.M * Nc, kBufFlags);
    const int lo = in_vgpr(a.lo), hi = in_vgpr(a.hi);
    const int m128 = in_vgpr(-128), p127 = in_vgpr(127);

    const int groups = (a.M + 63) / 64;
    const int Wv = gridDim.x * 4;
    for (int gi = blockIdx.x * 4 + wave; gi < groups; gi += Wv) {
        const int m = gi * 64 + lane;
        // the pixel's input row, biased to unsigned bytes; bytes beyond cin meet zero masks
        uint32_t xr[KD];
#pragma unroll
        for (int q = 0; q < KD; ++q) {
            const int off = 4 * q < K ? m * K + 4 * q : kOobOffset;
            xr[q] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rx, off, 0, 0) ^ 0x80808080u;
        }
        for (int c4 = 0; c4 < RW; c4 += 4) {
            int v[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const v2i *mk = masks + (c4 + r) * KQ;
                uint32_t sp = 0, sn = 0;
#pragma unroll
                for (int q = 0; q < KD; ++q) {
                    if (q < KQ) {
                        const v2i mm = mk[q];
                        sp = __builtin_amdgcn_sad_u8(xr[q] & (uint32_t)mm[0], 0u, sp);
                        sn = __builtin_amdgcn_sad_u8(xr[q] & (uint32_t)mm[1], 0u, sn);
                    }
                }
                v[r] = requant_i64<true>((int)sp - (int)sn, lpar[c4 + r], lo, hi);
            }
            if (a.residual) {
                const uint32_t res = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rr, m * Nc + cbase + c4, 0, 0);
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = med3_i32(v[r] + sbyte(res, r), m128, p127);
            }
            *reinterpret_cast<uint32_t *>(stage + lane * RW + c4) = pack4_low_bytes(v[0], v[1], v[2], v[3]);
        }
        // write the staged 64 x RW tile in 16-byte pieces (contiguous when the chunk is the row)
        const int tile_off = gi * 64 * Nc + cbase;
        if (RW == Nc || (RW & 15) == 0) {
            const int pieces = 4 * RW;  // 64*RW/16
            for (int q = lane; q < pieces; q += 64) {
                int go;
                if (RW == Nc) {
                    go = 16 * q;
                } else {
                    const int per_row = RW >> 4, row = q / per_row;
                    go = row * Nc + 16 * (q - row * per_row);
                }
                const v4i v = *reinterpret_cast<const v4i *>(stage + 16 * q);
                // tile offset in the vector offset: see the note at the store of the streaming kernel
                store_b128_guarded(v, ry, go + tile_off);
            }
        } else {
            for (int q = lane; q < 16 * RW; q += 64) {  // dword pieces
                const int row = (4 * q) / RW, col = 4 * q - row * RW;
                __builtin_amdgcn_raw_buffer_store_b32(*reinterpret_cast<const int *>(stage + 4 * q), ry,
                                                      row * Nc + col, tile_off, 0);
            }
        }
    }
}

using AddSubFn = void (*)(const AddSubArgs);

static AddSubFn select_addsub(int kd)
{
    if (kd <= 4) return &pw_addsub_kernel<4>;
    if (kd <= 8) return &pw_addsub_kernel<8>;
    if (kd <= 16) return &pw_addsub_kernel<16>;
    if (kd <= 24) return &pw_addsub_kernel<24>;
    if (kd <= 36) return &pw_addsub_kernel<36>;
    if (kd <= 48) return &pw_addsub_kernel<48>;
    if (kd <= 64) return &pw_addsub_kernel<64>;
    return nullptr;
}

}  // namespace prom

extern "C" int prom_pw_conv_addsub(const int8_t *x, int n, int h, int w, int cin, const void *w_packed,
                                   int cout, const prom_requant_t *rq, const int8_t *residual, int8_t *y,
                                   void *stream)
{
    using namespace prom;
    if (!x || !w_packed || !y || !rq || !rq->bias || !rq->mult || !rq->shift) return PROM_EINVAL;
    if (n <= 0 || h <= 0 || w <= 0 || cin <= 0 || cout <= 0) return PROM_EINVAL;
    if (rq->act_min < -128 || rq->act_max > 127 || rq->act_min > rq->act_max) return PROM_EINVAL;
    const long long M = (long long)n * h * w;
    if ((((uintptr_t)x | (uintptr_t)y | (uintptr_t)residual | (uintptr_t)w_packed) & 3) != 0) return PROM_EINVAL;
    if (cin > 256 || cin % 4 != 0 || cout % 4 != 0) return PROM_EUNSUPPORTED;
    if (rq->mult_neg) return PROM_EUNSUPPORTED;  // the comparison kernel has the plain epilogue only
    if ((M + 64) * (long long)(cin > cout ? cin : cout) >= (1LL << 31) - (1LL << 20)) return PROM_EUNSUPPORTED;
    {
        const uintptr_t ya = (uintptr_t)y, xa = (uintptr_t)x;
        if (ya < xa + (size_t)M * cin && xa < ya + (size_t)M * cout) return PROM_EALIAS;
    }
    AddSubArgs a;
    a.x = x; a.wq = static_cast<const uint32_t *>(w_packed);
    a.bias = rq->bias; a.mult = rq->mult; a.shift = rq->shift;
    a.residual = residual; a.y = y;
    a.M = (int)M; a.K = cin; a.Nc = cout; a.KW = (cin + 15) / 16;
    a.lo = rq->act_min; a.hi = rq->act_max;
    // chunk of output channels: masks 2*cin bytes + 16 parameter bytes + 256 staging bytes each
    const int per_channel = 2 * ((cin + 3) / 4) * 4 + 16 + 4 * 64;
    int cc = (60 * 1024) / per_channel;
    if (cc >= cout) {
        cc = cout;
    } else {
        cc &= ~15;
        if (cc < 16) return PROM_EUNSUPPORTED;
    }
    a.CC = cc;
    a.n_chunks = (cout + cc - 1) / cc;
    const AddSubFn fn = select_addsub((cin + 3) / 4);
    if (!fn) return PROM_EUNSUPPORTED;
    const size_t lds = (size_t)cc * per_channel;
    const long long groups = (M + 63) / 64;
    long long wgs = (groups + 3) / 4;
    if (wgs > 256 * 4) wgs = 256 * 4;
    clear_hip_error();
    AddSubArgs args = a;
    void *kargs[] = {&args};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(fn), dim3((unsigned)wgs, a.n_chunks),
                                         dim3(256), kargs, lds, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        last_hip_error() = e;
        (void)hipGetLastError();
        return PROM_EHIP;
    }
    return check_launch();
}

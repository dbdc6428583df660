// Host-side parts of the C ABI: ternary weight packing and error strings.
// The packed format is documented at prom_pack_ternary in prom.h.
#include "prom.h"
#include "prom_launch.h"

#include <cstring>
#include <vector>

namespace {
inline int words_per_row(int cin) { return (cin + 15) / 16; }
}  // namespace

extern "C" size_t prom_packed_size(int cout, int cin)
{
    if (cout <= 0 || cin <= 0) return 0;
    return (size_t)cout * (size_t)words_per_row(cin) * sizeof(uint32_t);
}

extern "C" int prom_pack_ternary(const int8_t *w_host, int cout, int cin, void *packed_host,
                                 size_t packed_bytes)
{
    if (!w_host || !packed_host || cout <= 0 || cin <= 0) return PROM_EINVAL;
    const size_t need = prom_packed_size(cout, cin);
    if (packed_bytes < need) return PROM_EWORKSPACE;
    const size_t total = (size_t)cout * (size_t)cin;
    for (size_t i = 0; i < total; ++i)
        if (w_host[i] < -1 || w_host[i] > 1) return PROM_EVALUE;
    const int kw = words_per_row(cin);
    unsigned char *out = static_cast<unsigned char *>(packed_host);
    for (int c = 0; c < cout; ++c) {
        const int8_t *row = w_host + (size_t)c * cin;
        for (int j = 0; j < kw; ++j) {
            uint32_t word = 0;
            for (int e = 0; e < 16; ++e) {
                const int k = 16 * j + e;
                if (k >= cin) break;
                const uint32_t code = (uint32_t)(row[k]) & 3u;  // 0->00, 1->01, -1->11
                const int d = e >> 2, b = e & 3;
                word |= code << (8 * b + 2 * d);
            }
            std::memcpy(out + ((size_t)c * kw + j) * 4, &word, 4);
        }
    }
    return PROM_OK;
}

extern "C" int prom_unpack_ternary(const void *packed_host, size_t packed_bytes, int cout, int cin,
                                   int8_t *w_host)
{
    if (!w_host || !packed_host || cout <= 0 || cin <= 0) return PROM_EINVAL;
    if (packed_bytes < prom_packed_size(cout, cin)) return PROM_EWORKSPACE;
    const int kw = words_per_row(cin);
    const unsigned char *in = static_cast<const unsigned char *>(packed_host);
    for (int c = 0; c < cout; ++c) {
        for (int k = 0; k < cin; ++k) {
            uint32_t word;
            std::memcpy(&word, in + ((size_t)c * kw + k / 16) * 4, 4);
            const int e = k & 15, d = e >> 2, b = e & 3;
            const uint32_t code = (word >> (8 * b + 2 * d)) & 3u;
            if (code == 2u) return PROM_EVALUE;
            w_host[(size_t)c * cin + k] = (int8_t)(code == 3u ? -1 : (int)code);
        }
    }
    return PROM_OK;
}

// ---- grouped 3x3 convolution: weights in the operand order of the matrix-core kernels -----------
// Group sizes 32 and 64: [block of 64 channels][tile t: 4][tap s: 9][lane: 64] entries of 16 bytes.
// Lane (i = lane & 15, kg = lane >> 4) of tile t holds, for output channel
// oc = 64*block + 16*(i >> 2) + 4*t + (i & 3) and tap s, the weights that multiply input channels
// 64*block + 16*kg + 0..15: w[s][oc][...] where the input channel belongs to oc's group, zero
// elsewhere.
// Group sizes 4, 8 and 16 (a tile of 16 output channels sees the 16 input channels at the same
// positions, so the taps go into the k dimension): [block][tile t: 4][step s: 3][lane: 64] entries.
// Lane (i, kg) of tile t holds, for output channel oc = 64*block + 16*t + i and tap 4*s + kg, the
// weights on input channels 64*block + 16*t + 0..15, zero outside oc's group and for taps 9..11.
extern "C" size_t prom_gconv_frag_size(int c, int group_size)
{
    if (c <= 0 || c % 4 != 0) return 0;
    if (group_size != 4 && group_size != 8 && group_size != 16 && group_size != 32 && group_size != 64) return 0;
    if (c % group_size != 0) return 0;
    const size_t per_block = group_size <= 16 ? 4 * 3 * 64 * 16 : 4 * 9 * 64 * 16;
    return (size_t)((c + 63) / 64) * per_block;
}

extern "C" int prom_gconv_pack(const int8_t *w_host, int c, int group_size, void *frag_host, size_t frag_bytes)
{
    if (!w_host || !frag_host) return PROM_EINVAL;
    const size_t need = prom_gconv_frag_size(c, group_size);
    if (need == 0) return PROM_EUNSUPPORTED;
    if (frag_bytes < need) return PROM_EWORKSPACE;
    int8_t *out = static_cast<int8_t *>(frag_host);
    std::memset(out, 0, need);
    const int ncb = (c + 63) / 64;
    const bool taps_in_k = group_size <= 16;
    const int steps = taps_in_k ? 3 : 9;
    for (int cb = 0; cb < ncb; ++cb)
        for (int t = 0; t < 4; ++t)
            for (int s = 0; s < steps; ++s)
                for (int lane = 0; lane < 64; ++lane) {
                    const int i = lane & 15, kg = lane >> 4;
                    const int oc = taps_in_k ? 64 * cb + 16 * t + i : 64 * cb + 16 * (i >> 2) + 4 * t + (i & 3);
                    const int tap = taps_in_k ? 4 * s + kg : s;
                    if (oc >= c || tap >= 9) continue;
                    const int gfirst = (oc / group_size) * group_size;
                    int8_t *e = out + ((((size_t)cb * 4 + t) * steps + s) * 64 + lane) * 16;
                    for (int b = 0; b < 16; ++b) {
                        const int ic = 64 * cb + 16 * (taps_in_k ? t : kg) + b;
                        if (ic >= gfirst && ic < gfirst + group_size)
                            e[b] = w_host[((size_t)tap * c + oc) * group_size + (ic - gfirst)];
                    }
                }
    return PROM_OK;
}

hipError_t &prom::last_hip_error()
{
    static thread_local hipError_t e = hipSuccess;
    return e;
}

extern "C" int prom_requant_check(const prom_requant_t *rq, int channels, int cin, int *bad_channel)
{
    if (bad_channel) *bad_channel = -1;
    if (!rq || !rq->bias || !rq->mult || !rq->shift || channels <= 0 || cin < 0) return PROM_EINVAL;
    if (rq->act_min < -128 || rq->act_max > 127 || rq->act_min > rq->act_max) return PROM_EINVAL;
    std::vector<int32_t> b(channels), m(channels), sh(channels);
    const size_t nbytes = (size_t)channels * sizeof(int32_t);
    // hipMemcpy from device memory waits for the work already enqueued on the device
    if (hipMemcpy(b.data(), rq->bias, nbytes, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(m.data(), rq->mult, nbytes, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(sh.data(), rq->shift, nbytes, hipMemcpyDeviceToHost) != hipSuccess) {
        prom::last_hip_error() = hipGetLastError();
        return PROM_EHIP;
    }
    const long long acc_max = 128LL * cin;  // |x| <= 128 and, in a pointwise layer, |w| <= 1
    for (int c = 0; c < channels; ++c) {
        const long long ab = b[c] < 0 ? -(long long)b[c] : (long long)b[c];
        const bool ok = m[c] > 0 && sh[c] >= 0 && sh[c] <= 31 && ab < (1LL << 29) && acc_max + ab < (1LL << 30);
        if (!ok) {
            if (bad_channel) *bad_channel = c;
            return PROM_EINVAL;
        }
    }
    return PROM_OK;
}

extern "C" const char *prom_last_hip_error(void)
{
    return hipGetErrorString(prom::last_hip_error());
}

extern "C" const char *prom_strerror(int code)
{
    switch (code) {
    case PROM_OK: return "success";
    case PROM_EINVAL: return "invalid argument (null pointer, non-positive dimension, bad activation window or stride)";
    case PROM_EUNSUPPORTED: return "shape beyond a compiled limit";
    case PROM_EALIAS: return "output buffer overlaps an input";
    case PROM_EWORKSPACE: return "workspace or output buffer missing or too small";
    case PROM_ESCRATCH: return "the problem needs more scratch memory than the fixed array of this no-allocation entry point holds";
    case PROM_EHIP: return "HIP runtime error at kernel launch";
    case PROM_EVALUE: return "weight value outside {-1,0,+1}";
    default: return "unknown error code";
    }
}

// Device helpers shared by the HIP kernels: exact requantisation and byte packing.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace prom {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
// 4-byte-aligned views for global accesses whose address is only dword aligned
typedef int v4i_a4 __attribute__((ext_vector_type(4), aligned(4)));
typedef int v2i_a4 __attribute__((ext_vector_type(2), aligned(4)));

// Bias applied to the rounded quotient before the float->int truncation so that the
// truncation acts as floor over the whole clamp window (see requant_to_biased).
constexpr int kQBias = 256;

// Put the wave's double-precision rounding mode to round-toward-minus-infinity (MODE
// register FP_ROUND bits [3:2]).  Every kernel that calls requant_to_biased executes this
// first; the kernels use no other f64/f16 arithmetic whose rounding matters.
__device__ __forceinline__ void set_f64_round_down()
{
    asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 2, 2), 2");
}

// min(max(v, lo), hi); becomes one v_med3_i32 when lo and hi sit in vector registers or are
// inline constants (the instruction can read at most one scalar register).
__device__ __forceinline__ int clamp_i32(int v, int lo, int hi) { return min(max(v, lo), hi); }

// Median of three = clamp of v to [lo, hi] when lo <= hi.  Written as the instruction because
// the compiler cannot prove lo <= hi and would emit a max and a min.
__device__ __forceinline__ int med3_i32(int v, int lo, int hi)
{
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
    return r;
}

// Moves a wave-uniform value into a vector register and hides its origin from the optimiser,
// so that two such bounds can feed one v_med3_i32.
__device__ __forceinline__ int in_vgpr(int v)
{
    asm volatile("" : "+v"(v));
    return v;
}

// scale = mult * 2^-(31+shift), exact in double (mult has at most 31 significant bits).
__device__ __forceinline__ double make_scale(int mult, int shift)
{
    return __builtin_ldexp((double)mult, -(31 + shift));
}

// Returns clamp(q, lo, hi) + kQBias where q = floor(s*scale + 1/2) is the exact rounded
// quotient; lo_b = lo + kQBias, hi_b = hi + kQBias.
// Why it is exact: (double)s and scale are exact, and 256.5 is exact, so the FMA computes
// RD(s*scale + 256.5) with a single round-down.  Round-down never crosses an integer
// (integers of this magnitude are representable), hence floor(RD(v)) == floor(v).  The
// conversion truncates toward zero, which equals floor for v >= 0; for v < 0 it yields a
// value <= 0 < lo_b, and the true floor is also below lo_b, so both clamp to lo_b.  Values
// beyond int32 saturate in the conversion and clamp to hi_b or lo_b likewise.
__device__ __forceinline__ int requant_to_biased(int s, double scale, int lo_b, int hi_b)
{
    const double v = __builtin_fma((double)s, scale, 256.5);
    const int qe = (int)v;
    return clamp_i32(qe, lo_b, hi_b);
}

// ---- integer requantisation ------------------------------------------------------------------

// The four per-channel values the epilogue keeps in registers.
__device__ __forceinline__ v4i requant_params(int bias, int mult, int mult_neg, int shift, bool prelu)
{
    if (prelu) return v4i{bias, mult, mult_neg, shift};
    const long long C = (long long)bias * mult + (1LL << (30 + shift));
    return v4i{(int)(uint32_t)C, (int)(C >> 32), mult, shift};
}

// t = acc*mult + C; q = t >> (31 + shift); clamp to [lo, hi].  pr = (C lo, C hi, mult, s) with
// s = shift-1 when !GENERAL (the caller guarantees shift >= 1) and s = shift when GENERAL.
template <bool GENERAL>
__device__ __forceinline__ int requant_i64(int accv, const v4i &pr, int lo, int hi)
{
    const long long C = (long long)(((unsigned long long)(uint32_t)pr[1] << 32) | (uint32_t)pr[0]);
    const long long t = (long long)accv * (long long)pr[2] + C;
    int q;
    if constexpr (GENERAL)
        q = (int)(t >> 31) >> pr[3];
    else
        q = (int)(t >> 32) >> pr[3];
    return med3_i32(q, lo, hi);
}

// PReLU form: pr = (bias, mult, mult_neg, shift); the multiplier follows the sign of
// s = acc + bias, then q = floor((s*m + 2^(30+shift)) / 2^(31+shift)), clamp.  Computed as
// floor((floor(s*m / 2^shift) + 2^30) / 2^31), which is the same number (2^30 is an integer and
// nested floors of divisions by positive integers collapse) and needs no per-channel rounding
// constant: such constants are loop invariants the compiler would keep in registers, two more
// per channel.
__device__ __forceinline__ int requant_prelu_s(int s, int mult, int mult_neg, int shift, int lo, int hi)
{
    const int m = s < 0 ? mult_neg : mult;
    const long long u = ((long long)s * (long long)m) >> shift;
    const int q = (int)((u + (1LL << 30)) >> 31);
    return med3_i32(q, lo, hi);
}
__device__ __forceinline__ int requant_prelu_i64(int accv, const v4i &pr, int lo, int hi)
{
    return requant_prelu_s(accv + pr[0], pr[1], pr[2], pr[3], lo, hi);
}

// Epilogue forms: 0 = every shift of the wavefront's channels >= 1 (pr.w holds shift-1),
// 1 = any shift, 2 = PReLU.
template <int MODE>
__device__ __forceinline__ int requant_mode(int accv, const v4i &pr, int lo, int hi)
{
    if constexpr (MODE == 2)
        return requant_prelu_i64(accv, pr, lo, hi);
    else
        return requant_i64<MODE == 1>(accv, pr, lo, hi);
}

// Low bytes of four ints -> one dword (a in bits 0..7).
__device__ __forceinline__ uint32_t pack4_low_bytes(int a, int b, int c, int d)
{
    const uint32_t ab = __builtin_amdgcn_perm((uint32_t)b, (uint32_t)a, 0x0c0c0400u);
    const uint32_t cd = __builtin_amdgcn_perm((uint32_t)d, (uint32_t)c, 0x0c0c0400u);
    return __builtin_amdgcn_perm(cd, ab, 0x05040100u);
}

// Sign-extended byte i (0..3) of a dword.
__device__ __forceinline__ int sbyte(uint32_t v, int i)
{
    return (int)(v << (24 - 8 * i)) >> 24;
}

}  // namespace prom

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

// The definition itself for one value, with s = acc + bias already formed and the multiplier already
// chosen (PReLU: by the sign of s): q = floor((s*m + 2^(30+shift)) / 2^(31+shift)), clamp.  An
// arithmetic right shift of a 64-bit integer is a floor division; |s*m| < 2^62 and the rounding
// constant is at most 2^61.  Used by the one-thread-per-output kernels.
__device__ __forceinline__ int requant_s_i64(int s, int m, int shift, int lo, int hi)
{
    const long long t = (long long)s * (long long)m + (1LL << (30 + shift));
    return clamp_i32((int)(t >> (31 + shift)), lo, hi);
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

// 16-byte buffer store, offset in the vector operand, with its data registers protected in the
// source.  On gfx950 a buffer store of more than 8 bytes picked up, now and then, the NEW contents
// of its data registers when the instruction right behind it overwrote them (seen with a scalar
// offset register, the one form for which the compiler inserts no wait state).  The empty
// statement behind the store reads the four data registers, so no instruction that overwrites them
// can be scheduled before it, and its two wait states are what the store needs -- whatever form of
// offset a later compiler picks.
__device__ __forceinline__ void store_b128_guarded(const v4i v, __amdgpu_buffer_rsrc_t rsrc, int voffset)
{
    __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, voffset, 0, 0);
    asm volatile("s_nop 1" : : "v"(v));
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

// Device-side Philox-4x32 for gfx950 (paper Sec. 2.3: counter-based generator
// built on wide multiplies; round function and constants from the Philox
// publication the paper cites).
//
// One lane makes one call: counter (c0, c1, 0, 0), key (k0, k1).  The upper two
// counter words are always zero in this library's call numbering, which lets
// the first round drop one multiply; when c1 is wave-uniform (the 64 lanes of a
// group do not straddle a 2^32 boundary) the compiler also moves the second
// round's first multiply to the scalar unit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rov {

constexpr uint32_t kPhiloxM0 = 0xD2511F53u;
constexpr uint32_t kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u;
constexpr uint32_t kPhiloxW1 = 0xBB67AE85u;

__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);   // a ^ b ^ c in one VALU op
}

// llvm.amdgcn.writelane reached through its intrinsic name (clang exposes no builtin for it);
// the compiler then schedules v_writelane_b32 itself, wait states included.
extern "C" __device__ uint32_t rov_llvm_writelane_i32(uint32_t, uint32_t, uint32_t) __asm(
    "llvm.amdgcn.writelane.i32");

// Value `v` (wave-uniform) placed into lane `dst` (wave-uniform) of `old`; other lanes keep `old`.
__device__ __forceinline__ uint32_t write_lane(uint32_t v, uint32_t dst, uint32_t old) {
    return rov_llvm_writelane_i32(v, dst, old);
}

// R rounds on counter (c0, c1, c2, c3) with key (k0, k1).
template <int R>
__device__ __forceinline__ void philox4x32(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                           uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * c0;   // v_mad_u64_u32: hi and lo in one op
        const uint64_t p1 = (uint64_t)kPhiloxM1 * c2;
        const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
        const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Same result as philox4x32<R>(c0, c1u, 0, 0, k0, k1) for a WAVE-UNIFORM second
// counter word c1u.  With the upper counter words zero, round 0 needs one
// multiply instead of two, and in round 1 the product of the (uniform) first
// word runs on the scalar unit: 18 vector multiplies per call instead of 20.
// Plain ^ is used wherever an operand pair is uniform so that it stays scalar.
template <int R>
__device__ __forceinline__ void philox4x32_low_counter(uint32_t c0, uint32_t c1u, uint32_t k0,
                                                       uint32_t k1, uint32_t (&out)[4]) {
    static_assert(R >= 3, "the first three rounds are written out");
    // round 0: counter (c0, c1u, 0, 0)
    const uint64_t p0 = (uint64_t)kPhiloxM0 * c0;
    const uint32_t a0 = c1u ^ k0;                               // uniform
    const uint32_t a2 = (uint32_t)(p0 >> 32) ^ k1;
    const uint32_t a3 = (uint32_t)p0;                           // a1 = 0
    k0 += kPhiloxW0; k1 += kPhiloxW1;
    // round 1: counter (a0, 0, a2, a3)
    const uint64_t q0 = (uint64_t)kPhiloxM0 * a0;               // uniform: scalar multiply
    const uint64_t q1 = (uint64_t)kPhiloxM1 * a2;
    const uint32_t b0 = (uint32_t)(q1 >> 32) ^ k0;
    const uint32_t b1 = (uint32_t)q1;
    const uint32_t b2 = a3 ^ ((uint32_t)(q0 >> 32) ^ k1);       // parenthesis is uniform
    const uint32_t b3 = (uint32_t)q0;                           // uniform
    k0 += kPhiloxW0; k1 += kPhiloxW1;
    // round 2: counter (b0, b1, b2, b3)
    const uint64_t r0 = (uint64_t)kPhiloxM0 * b0;
    const uint64_t r1 = (uint64_t)kPhiloxM1 * b2;
    const uint32_t d0 = xor3((uint32_t)(r1 >> 32), b1, k0);
    const uint32_t d2 = (uint32_t)(r0 >> 32) ^ (b3 ^ k1);       // parenthesis is uniform
    k0 += kPhiloxW0; k1 += kPhiloxW1;
    philox4x32<R - 3>(d0, (uint32_t)r1, d2, (uint32_t)r0, k0, k1, out);
}

// Runtime round count (test hook only).
__device__ __forceinline__ void philox4x32_dyn(int rounds, uint32_t c0, uint32_t c1, uint32_t c2,
                                               uint32_t c3, uint32_t k0, uint32_t k1,
                                               uint32_t (&out)[4]) {
    for (int r = 0; r < rounds; ++r) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * c0;
        const uint64_t p1 = (uint64_t)kPhiloxM1 * c2;
        const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
        const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// The four keep-words of one group of 64 calls: call number = base + lane where
// `base` (64-bit) is wave-uniform.  keep bit = (x <= t_minus_1).  Returns the
// four 64-lane ballots (wave-uniform values).
// CARRY = false promises that lo32(base) + 63 does not wrap, so the second
// counter word is wave-uniform and part of the first two rounds runs on the
// scalar unit; CARRY = true handles the general case.
template <int R, bool CARRY>
__device__ __forceinline__ void philox_group_ballots(uint64_t base, uint32_t lane, uint32_t k0,
                                                     uint32_t k1, uint32_t t_minus_1,
                                                     uint64_t (&ballots)[4]) {
    const uint32_t blo = (uint32_t)base;
    const uint32_t bhi = (uint32_t)(base >> 32);
    uint32_t x[4];
    const uint32_t c0 = blo + lane;
    if (!CARRY) {
        philox4x32_low_counter<R>(c0, bhi, k0, k1, x);
    } else {
        const uint32_t c1 = bhi + (c0 < blo ? 1u : 0u);
        philox4x32<R>(c0, c1, 0u, 0u, k0, k1, x);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) ballots[r] = __ballot(x[r] <= t_minus_1);
}

}  // namespace rov

// fp32 -> OCP e4m3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, largest finite value 448,
// no infinities) on the device: round to nearest, ties to the even code, saturating at +-448; NaN
// gives the NaN code.  Used where the fp8 block quantises an activation (the paper measures in FP8,
// Sec. 1 and Sec. 6); plain integer arithmetic, so that the result is the same nearest-code choice
// on every input, independent of the hardware's own conversion modes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rov {

__device__ __forceinline__ uint32_t f32_to_e4m3(float v) {
    const uint32_t bits = __float_as_uint(v);
    const uint32_t sign = (bits >> 24) & 0x80u;
    const uint32_t a = bits & 0x7FFFFFFFu;
    uint32_t code;
    if (a > 0x7F800000u) {
        code = 0x7Fu;                                   // NaN
    } else if (a >= 0x43E80000u) {                      // |v| >= 464: beyond the tie point above 448
        code = 0x7Eu;
    } else if (a < 0x3C800000u) {                       // |v| < 2^-6: subnormal codes, units of 2^-9
        // rintf rounds to nearest, ties to even; 8 units is the smallest normal (code 0x08)
        code = (uint32_t)__builtin_rintf(__uint_as_float(a) * 512.0f);
    } else {
        // drop 20 mantissa bits with round-to-nearest-even; a carry moves into the exponent
        const uint32_t r = a + 0x7FFFFu + ((a >> 20) & 1u);
        code = ((r >> 20) & 0x7FFu) - ((127u - 7u) << 3);   // (exponent - 120) << 3 | mantissa
        code = code > 0x7Eu ? 0x7Eu : code;
    }
    return code | sign;
}

// Four values to four consecutive bytes (lowest address first).
__device__ __forceinline__ uint32_t pack_e4m3x4(float a, float b, float c, float d) {
    return f32_to_e4m3(a) | (f32_to_e4m3(b) << 8) | (f32_to_e4m3(c) << 16) | (f32_to_e4m3(d) << 24);
}

}  // namespace rov

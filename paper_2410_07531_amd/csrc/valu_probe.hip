// VALU issue-rate probe: measures how many cycles a wave64 spends issuing one
// instruction of a given kind on this device.  The RNG kernel is bound by VALU
// issue (paper Table 1: "Issue stage", "ALU pipe"), so its ceiling is derived
// from these measured costs rather than from an assumed datasheet rate.
//
// Each lane runs 8 independent dependency chains of the probed operation for
// `iters` iterations; s_memtime brackets the loop.  Per-wave cycle counts are
// written to out[2*wave_global .. +1] = (cycles, checksum).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "philox_device.h"
#include "rov_internal.h"

namespace rov {
namespace {

constexpr int kChains = 8;

template <int KIND>
__device__ __forceinline__ uint32_t probe_op(uint32_t x, uint32_t y, uint32_t z, uint32_t s) {
    if (KIND == 0) {   // 32x32 -> 64 product, both halves used (v_mad_u64_u32)
        const uint64_t p = (uint64_t)x * kPhiloxM0;
        return (uint32_t)(p >> 32) + (uint32_t)p;   // + one add: subtracted by the caller via kind 4
    } else if (KIND == 1) {   // low half only (v_mul_lo_u32)
        return x * z;   // z: a neighbouring chain, so that the products cannot be pre-combined
    } else if (KIND == 2) {   // high half only (v_mul_hi_u32)
        return __umulhi(x, kPhiloxM0);
    } else if (KIND == 3) {   // three-input xor (v_bitop3_b32)
        return xor3(x, y, s);
    } else if (KIND == 4) {   // add (v_add_u32)
        return x + z;
    } else {                  // compare + lane write: ballot(x < s) dropped into lane 5
        const uint64_t b = __ballot(x < s);
        return write_lane((uint32_t)b, 5u, x) + 1u;
    }
}

template <int KIND>
__global__ __launch_bounds__(256) void probe_kernel(uint64_t* __restrict__ out, int iters, uint32_t s) {
    uint32_t v[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c) v[c] = threadIdx.x * 2654435761u + c * 40503u + s;
    uint32_t y = threadIdx.x ^ s;
    const uint64_t t0 = __builtin_readcyclecounter();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int c = 0; c < kChains; ++c)
                v[c] = probe_op<KIND>(v[c], y, v[(c + 1) % kChains], s);
        }
    }
    const uint64_t t1 = __builtin_readcyclecounter();
    uint32_t acc = 0;
#pragma unroll
    for (int c = 0; c < kChains; ++c) acc ^= v[c];
    // one record per wave: lane 0 writes; the checksum keeps the chains alive
    const uint32_t sum = __builtin_amdgcn_readfirstlane(acc) ^ (uint32_t)__popcll(__ballot(acc & 1u));
    if ((threadIdx.x & 63u) == 0u) {
        const uint64_t wave = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
        out[2 * wave] = t1 - t0;
        out[2 * wave + 1] = sum;
    }
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// kind 6: back-to-back independent MFMA 32x32x16 bf16 (4 accumulators per wave, no memory
// traffic): the matrix-core rate this device sustains, i.e. the clock it holds under MFMA load.
__global__ __launch_bounds__(256) void probe_mfma_kernel(uint64_t* __restrict__ out, int iters, uint32_t s) {
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(float)((threadIdx.x + i) & 3);
        b[i] = (__bf16)(float)((threadIdx.x * 3 + i + s) & 3);
    }
    f32x16 acc[4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[c][e] = 0.0f;
    const uint64_t t0 = __builtin_readcyclecounter();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c)
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
    }
    const uint64_t t1 = __builtin_readcyclecounter();
    float sum = 0.0f;
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) sum += acc[c][e];
    if ((threadIdx.x & 63u) == 0u) {
        const uint64_t wave = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
        out[2 * wave] = t1 - t0;
        out[2 * wave + 1] = (uint64_t)__float_as_uint(sum);
    }
}

}  // namespace
}  // namespace rov

// Diagnostic entry point (declared in rov.h).
extern "C" int rov_valu_probe(int kind, int iters, int workgroups, uint64_t* out, void* stream) {
    if (kind < 0 || kind > 6 || iters <= 0 || workgroups <= 0 || out == nullptr) return ROV_ERR_INVALID;
    if (!rov::aligned(out, 8)) return ROV_ERR_INVALID;
    const dim3 grid((unsigned)workgroups), block(256);
    hipStream_t st = (hipStream_t)stream;
    const uint32_t s = 0x9E3779B9u;
    switch (kind) {
        case 0: hipLaunchKernelGGL(rov::probe_kernel<0>, grid, block, 0, st, out, iters, s); break;
        case 1: hipLaunchKernelGGL(rov::probe_kernel<1>, grid, block, 0, st, out, iters, s); break;
        case 2: hipLaunchKernelGGL(rov::probe_kernel<2>, grid, block, 0, st, out, iters, s); break;
        case 3: hipLaunchKernelGGL(rov::probe_kernel<3>, grid, block, 0, st, out, iters, s); break;
        case 4: hipLaunchKernelGGL(rov::probe_kernel<4>, grid, block, 0, st, out, iters, s); break;
        case 5: hipLaunchKernelGGL(rov::probe_kernel<5>, grid, block, 0, st, out, iters, s); break;
        default: hipLaunchKernelGGL(rov::probe_mfma_kernel, grid, block, 0, st, out, iters, s); break;
    }
    ROV_LAUNCH_CHECK();
    return ROV_OK;
}

// Row-wise glue of the transformer block (paper Fig. 2 / Sec. 3.2: the normalisation layers
// between the GEMMs, which the paper's analysis leaves out as cheap; here RMSNorm and the rotary
// embedding of a Llama-style block; the SwiGLU product lives in the GEMM epilogue).  All bf16
// in / bf16 out with fp32 arithmetic, 16-byte vector accesses, one pass over the data each.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fp8_device.h"
#include "rov_internal.h"

namespace rov {
namespace {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    f32x2 v = {lo, hi};
    bf16x2 h = __builtin_convertvector(v, bf16x2);
    return *reinterpret_cast<uint32_t*>(&h);
}
__device__ __forceinline__ float lo_f(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_f(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// y[row] = x[row] / sqrt(mean(x[row]^2) + eps) * weight ; one workgroup per row, n % 8 == 0.
// OUT8: y is written as OCP e4m3 bytes of (that value * out_inv): the normalised activation of the
// fp8 block, quantised with its per-tensor scale where it is produced.
template <bool OUT8>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const uint16_t* __restrict__ x,
                                                      const uint16_t* __restrict__ weight,
                                                      uint16_t* __restrict__ y, int n, float eps, float out_inv) {
    __shared__ float red[4];
    // beside a co-resident RNG grid (overlap schedules) this kernel's waves would wait for issue slots
    // behind the RNG's long integer multiplies (measured 0.05 -> 0.23 ms at 16384 x 4096): raise their
    // issue priority, as the GEMM kernels do
    __builtin_amdgcn_s_setprio(3);
    const uint16_t* xr = x + (size_t)blockIdx.x * n;
    uint16_t* yr = y + (size_t)blockIdx.x * n;
    float ss = 0.0f;
    for (int c = threadIdx.x * 8; c < n; c += 256 * 8) {
        const uint4 v = *reinterpret_cast<const uint4*>(xr + c);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float a = lo_f(w[i]), b = hi_f(w[i]);
            ss = __builtin_fmaf(a, a, ss);
            ss = __builtin_fmaf(b, b, ss);
        }
    }
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) ss += __shfl_xor(ss, s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = red[0] + red[1] + red[2] + red[3];
    const float inv = 1.0f / sqrtf(tot / (float)n + eps);
    for (int c = threadIdx.x * 8; c < n; c += 256 * 8) {
        const uint4 v = *reinterpret_cast<const uint4*>(xr + c);
        const uint4 g = *reinterpret_cast<const uint4*>(weight + c);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        const uint32_t gw[4] = {g.x, g.y, g.z, g.w};
        if constexpr (OUT8) {
            float f[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                f[2 * i] = lo_f(w[i]) * inv * lo_f(gw[i]) * out_inv;
                f[2 * i + 1] = hi_f(w[i]) * inv * hi_f(gw[i]) * out_inv;
            }
            uint8_t* y8 = reinterpret_cast<uint8_t*>(y) + (size_t)blockIdx.x * n;
            *reinterpret_cast<uint2*>(y8 + c) =
                make_uint2(pack_e4m3x4(f[0], f[1], f[2], f[3]), pack_e4m3x4(f[4], f[5], f[6], f[7]));
        } else {
            uint32_t o[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                o[i] = pack2(lo_f(w[i]) * inv * lo_f(gw[i]), hi_f(w[i]) * inv * hi_f(gw[i]));
            *reinterpret_cast<uint4*>(yr + c) = make_uint4(o[0], o[1], o[2], o[3]);
        }
    }
}

// Rotary embedding in place on the first `nheads` heads of each token row of a
// [tokens, row_elems] buffer: pair (2t, 2t+1) of token position s is rotated by
// s * theta^(-2t/d).  The angle is formed and reduced modulo 2*pi in double so
// that long sequences keep fp32-accurate sines.  A thread owns four pairs (8
// elements, 16 bytes) of one token and walks over the heads, which all turn by
// the same angles: the sines are computed once per token, not once per head.
__global__ __launch_bounds__(256) void rope_kernel(uint16_t* __restrict__ buf, int64_t row_elems,
                                                   int S, int nheads, int d, double log2_theta,
                                                   int64_t total_quads) {
    __builtin_amdgcn_s_setprio(3);
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total_quads) return;
    const int quads_per_head = d / 8;
    const int qd = (int)(idx % quads_per_head);
    const int64_t token = idx / quads_per_head;
    const int pos = (int)(token % S);
    float sn[4], cs[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = qd * 4 + i;
        const double inv_freq = exp2(-2.0 * (double)t / (double)d * log2_theta);
        double ang = (double)pos * inv_freq;
        ang -= 6.283185307179586476925 * rint(ang * 0.15915494309189533577);
        sincosf((float)ang, &sn[i], &cs[i]);
    }
    uint16_t* ptr = buf + token * row_elems + qd * 8;
#pragma unroll 4
    for (int head = 0; head < nheads; ++head, ptr += d) {
        const uint4 v = *reinterpret_cast<const uint4*>(ptr);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        uint32_t o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float xe = lo_f(w[i]), xo = hi_f(w[i]);
            o[i] = pack2(xe * cs[i] - xo * sn[i], xe * sn[i] + xo * cs[i]);
        }
        *reinterpret_cast<uint4*>(ptr) = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

}  // namespace

int launch_rmsnorm(const void* x, const void* weight, void* y, int64_t rows, int n, float eps,
                   hipStream_t stream) {
    if (rows <= 0 || n <= 0 || (n % 8) != 0 || rows > 0x7FFFFFFF) return ROV_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(rmsnorm_kernel<false>, dim3((unsigned)rows), dim3(256), 0, stream,
                       (const uint16_t*)x, (const uint16_t*)weight, (uint16_t*)y, n, eps, 1.0f);
    ROV_LAUNCH_CHECK();
    return ROV_OK;
}

int launch_rmsnorm_fp8(const void* x, const void* weight, void* y8, int64_t rows, int n, float eps, float scale,
                       hipStream_t stream) {
    if (rows <= 0 || n <= 0 || (n % 8) != 0 || rows > 0x7FFFFFFF) return ROV_ERR_UNSUPPORTED;
    if (!(scale > 0.0f)) return ROV_ERR_INVALID;
    hipLaunchKernelGGL(rmsnorm_kernel<true>, dim3((unsigned)rows), dim3(256), 0, stream,
                       (const uint16_t*)x, (const uint16_t*)weight, (uint16_t*)y8, n, eps, 1.0f / scale);
    ROV_LAUNCH_CHECK();
    return ROV_OK;
}

int launch_rope(void* buf, int64_t tokens, int64_t row_elems, int S, int nheads, int d, float theta,
                hipStream_t stream) {
    if (tokens <= 0 || nheads <= 0 || (d % 8) != 0 || theta <= 0.0f) return ROV_ERR_UNSUPPORTED;
    const int64_t quads = tokens * (d / 8);            // one thread per token and four pairs, all heads
    const int64_t blocks = (quads + 255) / 256;
    if (blocks > 0x7FFFFFFF) return ROV_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(rope_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (uint16_t*)buf,
                       row_elems, S, nheads, d, log2((double)theta), quads);
    ROV_LAUNCH_CHECK();
    return ROV_OK;
}

}  // namespace rov

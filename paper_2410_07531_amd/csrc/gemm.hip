// GEMM for the QKV / PROJ / FC1 / FC2 layers that the RNG kernel hides behind
// (paper Sec. 3.2, Table 1 GEMM column: MMA-bound, L2 read bandwidth second).
//
// bf16 fast path (A [M,K] and weights [N,K], both K-contiguous):
//   - workgroup tile 256 x 256, K step 64, 4 waves in a 2 x 2 grid, each wave
//     owning a 128 x 128 block as 4 x 4 MFMA 32x32x16 tiles (256 fp32
//     accumulators per lane);
//   - tiles go from global memory straight into LDS (global_load_lds, 16 bytes
//     per lane), two 64 KiB stages; a wave's 64 lanes always fill 1 KiB of
//     consecutive LDS, so the bank swizzle (16-byte chunk index XOR row%8) is
//     applied on the global-address side;
//   - the MFMA is issued with the weight fragment as first operand, so each
//     lane ends up with 4 consecutive output columns and stores 8 bytes at once;
//   - workgroup ids are remapped so that the workgroups that land on one XCD
//     (one L2) cover a compact block of output tiles.
// The register budget is capped below the full file so that RNG waves can be
// co-resident on every SIMD (the paper's carve-out, Sec. 6.2).
//
// fp8 (OCP e4m3) uses the same kernel: a tile row is 128 bytes either way (64
// bf16 or 128 fp8 values), and each 16-byte fragment feeds two MFMA 32x32x16
// fp8 instructions (which 8 of the 16 k-values a half-wave supplies is the same
// for both operands, so the sum is unchanged).
//
// Everything else (fp32, [K,N] weights, K not a multiple of the tile depth)
// takes a small LDS-tiled VALU kernel that is correct for any shape.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rov_internal.h"

namespace rov {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);   // quiet NaN
    u += 0x7FFFu + ((u >> 16) & 1u);   // round to nearest, ties to even
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
    return __uint_as_float((uint32_t)b << 16);
}

// ------------------------------------------------------------------ generic kernel
// 64 x 64 output tile, 16 x 16 threads, 4 x 4 outputs per thread, K step 16, fp32 FMA.
template <typename T>
__device__ __forceinline__ float load_as_f32(const T* p);
template <>
__device__ __forceinline__ float load_as_f32<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float load_as_f32<uint16_t>(const uint16_t* p) { return bf16_bits_to_f32(*p); }

// OCP e4m3: 1 sign, 4 exponent bits (bias 7), 3 mantissa bits; 0x7F / 0xFF are NaN; no infinities.
__device__ __forceinline__ float e4m3_to_f32(uint8_t c) {
    const uint32_t e = (c >> 3) & 0xFu, m = c & 0x7u;
    float v;
    if (e == 0xFu && m == 0x7u) v = __uint_as_float(0x7FC00000u);
    else if (e == 0u) v = (float)m * 0.001953125f;                       // m/8 * 2^-6
    else v = __uint_as_float(((e + 120u) << 23) | (m << 20));            // (1 + m/8) * 2^(e-7)
    return (c & 0x80u) ? -v : v;
}
template <>
__device__ __forceinline__ float load_as_f32<uint8_t>(const uint8_t* p) { return e4m3_to_f32(*p); }

template <typename T>
__device__ __forceinline__ void store_from_f32(T* p, float v);
template <>
__device__ __forceinline__ void store_from_f32<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_from_f32<uint16_t>(uint16_t* p, float v) { *p = f32_to_bf16_bits(v); }

template <typename T, typename TO, bool TRANSB>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const T* __restrict__ A,
                                                           const T* __restrict__ Bm,
                                                           TO* __restrict__ C, int M, int N, int K,
                                                           float alpha) {
    __shared__ float As[16][64 + 1];
    __shared__ float Bs[16][64 + 1];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int e = threadIdx.x; e < 64 * 16; e += 256) {
            const int r = e >> 4, kk = e & 15;          // A: row r, k kk (k fastest in memory)
            const int m = m0 + r, k = k0 + kk;
            As[kk][r] = (m < M && k < K) ? load_as_f32(A + (size_t)m * K + k) : 0.0f;
            if (TRANSB) {
                const int n = n0 + r;
                Bs[kk][r] = (n < N && k < K) ? load_as_f32(Bm + (size_t)n * K + k) : 0.0f;
            }
        }
        if (!TRANSB) {
            for (int e = threadIdx.x; e < 64 * 16; e += 256) {
                const int kk = e >> 6, c = e & 63;      // B: k kk, column c (n fastest in memory)
                const int k = k0 + kk, n = n0 + c;
                Bs[kk][c] = (n < N && k < K) ? load_as_f32(Bm + (size_t)k * N + n) : 0.0f;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m < M && n < N) store_from_f32(C + (size_t)m * N + n, alpha * acc[i][j]);
        }
}

// ------------------------------------------------------------------ MFMA kernel (bf16 / fp8)
constexpr int BM = 256, BN = 256;
constexpr int kRowBytes = 128;                      // one tile row: 64 bf16 or 128 fp8 values
constexpr int kStageBytes = (BM + BN) * kRowBytes;  // 64 KiB: A tile then W tile

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;
typedef int i32x4 __attribute__((ext_vector_type(4)));

// One operand tile (256 rows x 128 bytes of k) from global to LDS.  Wave w copies row
// blocks w, w+4, ... (8 rows each); within a block lane L fills physical chunk
// L%8 of row L/8, which holds logical chunk (L%8) ^ (row%8).  `panel` points at the first
// row of the 256-row operand panel plus the k offset (wave-uniform); voff[i] is the lane's
// constant byte offset inside the panel for row block i, so the address is a scalar base
// plus a 32-bit vector offset and the loop does no vector address arithmetic.
__device__ __forceinline__ void load_tile(const char* __restrict__ panel, const uint32_t (&voff)[8],
                                          char* lds_tile, int wave) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int blk = wave + 4 * i;                // 0..31
        __builtin_amdgcn_global_load_lds((gptr_t)(panel + voff[i]), (lptr_t)(lds_tile + blk * 8 * kRowBytes),
                                         16, 0, 0);
    }
}

__device__ __forceinline__ void lane_offsets(uint32_t (&voff)[8], size_t ld_bytes, int rows_valid, int wave,
                                             int lane) {
    const int rl = lane >> 3;                        // row within the 8-row block
    const int chunk = (lane & 7) ^ rl;               // logical 16-byte chunk this lane fetches
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int row = (wave + 4 * i) * 8 + rl;
        row = row < rows_valid ? row : rows_valid - 1;   // clamp: rows past the edge are never stored
        voff[i] = (uint32_t)((size_t)row * ld_bytes) + (uint32_t)(chunk * 16);
    }
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Reads one accumulator value where it is needed.  The "a" constraint keeps the value in its
// accumulation register until this point; without it the register allocator copies all 256
// accumulators to ordinary VGPRs at the loop exit and the kernel needs the whole register file,
// leaving no room for co-resident RNG waves.
__device__ __forceinline__ float acc_read(float v) {
    float r;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(r) : "a"(v));
    return r;
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    f32x2 v = {lo, hi};
    bf16x2 h = __builtin_convertvector(v, bf16x2);   // v_cvt_pk_bf16_f32: nearest, ties to even
    return *reinterpret_cast<uint32_t*>(&h);
}

// ESZ: bytes per input element (2 = bf16, 1 = fp8 e4m3).  Output and residual are bf16.
template <int ESZ>
__global__ __launch_bounds__(256, 1) void gemm_tn_kernel(const char* __restrict__ A,
                                                         const char* __restrict__ Wt,
                                                         uint16_t* __restrict__ C,
                                                         const uint16_t* __restrict__ R, int M, int N,
                                                         int K, float alpha, int tiles_m, int tiles_n) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    // Co-resident RNG waves only need the VALU issue slots this kernel leaves idle; raise this
    // wave's issue priority so that they never delay its MFMA / LDS instruction stream.
    __builtin_amdgcn_s_setprio(3);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    // XCD-aware tile id: workgroup ids are dealt round-robin to the 8 XCDs; give each XCD a
    // contiguous range of logical tiles, ordered in bands of 8 tile-rows with the row fastest.
    const int T = tiles_m * tiles_n;
    int id;
    {
        const int pid = blockIdx.x, per = T >> 3, rem = T & 7;
        const int xcd = pid & 7, loc = pid >> 3;
        id = xcd < rem ? xcd * (per + 1) + loc : rem * (per + 1) + (xcd - rem) * per + loc;
    }
    constexpr int GM = 8;
    const int band = id / (GM * tiles_n);
    const int band_rows = (tiles_m - band * GM) < GM ? (tiles_m - band * GM) : GM;
    const int in_band = id - band * GM * tiles_n;
    const int tm = band * GM + in_band % band_rows;
    const int tn = in_band / band_rows;
    const int m0 = tm * BM, n0 = tn * BN;

    f32x16 acc[4][4];   // [weight-row block j][activation-row block i]
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[j][i][e] = 0.0f;

    // per-lane fragment addressing: row = base + lane%32, k-chunk = 2*kk + lane/32, swizzled by row%8
    const int frow = lane & 31;
    const int fhalf = lane >> 5;
    const int swz = lane & 7;
    int foff[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) foff[kk] = frow * kRowBytes + (((2 * kk + fhalf) ^ swz) << 4);
    const int a_base = (wm * 128) * kRowBytes;
    const int w_base = BM * kRowBytes + (wn * 128) * kRowBytes;

    i32x4 af[2][4], wf[2][4];   // 16-byte fragments of the current and the next k-step
    auto read_frags = [&](int buf, const char* stage, int kk) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            af[buf][i] = *reinterpret_cast<const i32x4*>(stage + a_base + i * 32 * kRowBytes + foff[kk]);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            wf[buf][j] = *reinterpret_cast<const i32x4*>(stage + w_base + j * 32 * kRowBytes + foff[kk]);
    };

    const size_t ld_bytes = (size_t)K * ESZ;
    const int nk = (int)(ld_bytes / kRowBytes);
    uint32_t voff_a[8], voff_w[8];
    lane_offsets(voff_a, ld_bytes, M - m0 < BM ? M - m0 : BM, wave, lane);
    lane_offsets(voff_w, ld_bytes, N - n0 < BN ? N - n0 : BN, wave, lane);
    const char* a_panel = A + (size_t)m0 * ld_bytes;
    const char* w_panel = Wt + (size_t)n0 * ld_bytes;
    load_tile(a_panel, voff_a, lds, wave);
    load_tile(w_panel, voff_w, lds + BM * kRowBytes, wave);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __syncthreads();
    if (nk > 1) {
        load_tile(a_panel + kRowBytes, voff_a, lds + kStageBytes, wave);
        load_tile(w_panel + kRowBytes, voff_w, lds + kStageBytes + BM * kRowBytes, wave);
    }
    read_frags(0, lds, 0);

    auto mfma_one = [&](int buf, int j, int i) {
        if (ESZ == 2) {
            acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wf[buf][j]),
                                                                __builtin_bit_cast(bf16x8, af[buf][i]),
                                                                acc[j][i], 0, 0, 0);
        } else {
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const i32x4 wv = wf[buf][j], av = af[buf][i];
                const long wl = ((long)(uint32_t)wv[2 * hf]) | ((long)wv[2 * hf + 1] << 32);
                const long al = ((long)(uint32_t)av[2 * hf]) | ((long)av[2 * hf + 1] << 32);
                acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(wl, al, acc[j][i], 0, 0, 0);
            }
        }
    };

    for (int kt = 0; kt < nk; ++kt) {
        const char* cur = lds + (kt & 1) * kStageBytes;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (kk < 3) {
                // the 8 fragment reads of the next k-step ride between this k-step's 16 MFMAs:
                // an LDS read issued in the shadow of a running MFMA costs the matrix pipe nothing
#pragma unroll
                for (int idx = 0; idx < 16; ++idx) {
                    mfma_one(kk & 1, idx >> 2, idx & 3);
                    if ((idx & 1) == 0) {
                        if (idx < 8)
                            af[(kk + 1) & 1][idx >> 1] = *reinterpret_cast<const i32x4*>(
                                cur + a_base + (idx >> 1) * 32 * kRowBytes + foff[kk + 1]);
                        else
                            wf[(kk + 1) & 1][(idx - 8) >> 1] = *reinterpret_cast<const i32x4*>(
                                cur + w_base + ((idx - 8) >> 1) * 32 * kRowBytes + foff[kk + 1]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
                // Tile boundary: the next stage must have landed for every wave, and every wave
                // must be done reading this stage before it is refilled.  The refill (tile kt+2)
                // and the first fragments of the next stage are issued between the 16 MFMAs of
                // this k-step, one load per MFMA, so the matrix pipe keeps running while they
                // issue.  The path is the same on the last tiles, where it reloads the final
                // tile and reads fragments that nobody uses: a branch here would split the
                // accumulators' live ranges and cost far more than the wasted loads.
                __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0)
                __syncthreads();
                char* refill = lds + (kt & 1) * kStageBytes;
                const char* nxt = lds + ((kt + 1) & 1) * kStageBytes;
                const size_t k_bytes = (size_t)(kt + 2 < nk ? kt + 2 : nk - 1) * kRowBytes;
                const char* ap = a_panel + k_bytes;
                const char* wp = w_panel + k_bytes;
#pragma unroll
                for (int idx = 0; idx < 16; ++idx) {
                    mfma_one(1, idx >> 2, idx & 3);
                    if (idx < 8)
                        __builtin_amdgcn_global_load_lds((gptr_t)(ap + voff_a[idx]),
                                                         (lptr_t)(refill + (wave + 4 * idx) * 8 * kRowBytes), 16, 0, 0);
                    else
                        __builtin_amdgcn_global_load_lds(
                            (gptr_t)(wp + voff_w[idx - 8]),
                            (lptr_t)(refill + BM * kRowBytes + (wave + 4 * (idx - 8)) * 8 * kRowBytes), 16, 0, 0);
                    if ((idx & 1) == 0) {
                        if (idx < 8)
                            af[0][idx >> 1] = *reinterpret_cast<const i32x4*>(nxt + a_base + (idx >> 1) * 32 * kRowBytes + foff[0]);
                        else
                            wf[0][(idx - 8) >> 1] = *reinterpret_cast<const i32x4*>(nxt + w_base + ((idx - 8) >> 1) * 32 * kRowBytes + foff[0]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): no LDS load may outlive the loop

    // D'[r][c] = C[m = c][n = r]: lane holds column c = lane%32 (an activation row) and, for
    // register e, weight row 8*(e/4) + 4*(lane/32) + e%4: four consecutive n per e/4.
    // N is a multiple of 4 here, so a group of four columns is inside or outside as a whole.
    const int mrow = lane & 31;
    const int nsub = (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + wm * 128 + i * 32 + mrow;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // keep the accumulator read-out block by block: a hoisted read-out of all 256
            // values would double the kernel's register footprint
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wn * 128 + j * 32 + q * 8 + nsub;
                float c0 = alpha * acc_read(acc[j][i][q * 4 + 0]);
                float c1 = alpha * acc_read(acc[j][i][q * 4 + 1]);
                float c2 = alpha * acc_read(acc[j][i][q * 4 + 2]);
                float c3 = alpha * acc_read(acc[j][i][q * 4 + 3]);
                if (m < M && n < N) {
                    if (R != nullptr) {   // fused residual add (wave-uniform branch)
                        const uint2 r = *reinterpret_cast<const uint2*>(R + (size_t)m * N + n);
                        c0 += __uint_as_float(r.x << 16);
                        c1 += __uint_as_float(r.x & 0xFFFF0000u);
                        c2 += __uint_as_float(r.y << 16);
                        c3 += __uint_as_float(r.y & 0xFFFF0000u);
                    }
                    uint2 v;
                    v.x = pack_bf16x2(c0, c1);
                    v.y = pack_bf16x2(c2, c3);
                    *reinterpret_cast<uint2*>(C + (size_t)m * N + n) = v;
                }
            }
        }
    }
}

}  // namespace

int launch_gemm(const void* A, const void* Bm, void* C, int M, int N, int K, int dtype, int transB,
                float scaleA, float scaleB, hipStream_t stream) {
    return launch_gemm_residual(A, Bm, C, nullptr, M, N, K, dtype, transB, scaleA, scaleB, stream);
}

int launch_gemm_residual(const void* A, const void* Bm, void* C, const void* R, int M, int N, int K,
                         int dtype, int transB, float scaleA, float scaleB, hipStream_t stream) {
    if (A == nullptr || Bm == nullptr || C == nullptr || M <= 0 || N <= 0 || K <= 0)
        return ROV_ERR_INVALID;
    if (!aligned(A, 16) || !aligned(Bm, 16) || !aligned(C, 16)) return ROV_ERR_INVALID;
    if (dtype != ROV_F32 && dtype != ROV_BF16 && dtype != ROV_FP8_E4M3) return ROV_ERR_INVALID;
    const float alpha = scaleA * scaleB;
    const bool tb = transB != 0;
    const int esz = dtype == ROV_BF16 ? 2 : 1;

    if (dtype != ROV_F32 && tb && ((size_t)K * esz) % kRowBytes == 0 && (N % 4) == 0) {
        const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
        const long long T = (long long)tiles_m * tiles_n;
        if (T > 0x7FFFFFFFLL) return ROV_ERR_UNSUPPORTED;
        auto kern = esz == 2 ? gemm_tn_kernel<2> : gemm_tn_kernel<1>;
        static bool attr_set[2] = {false, false};
        if (!attr_set[esz - 1]) {
            ROV_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                            2 * kStageBytes));
            attr_set[esz - 1] = true;
        }
        hipLaunchKernelGGL(kern, dim3((unsigned)T), dim3(256), 2 * kStageBytes, stream, (const char*)A,
                           (const char*)Bm, (uint16_t*)C, (const uint16_t*)R, M, N, K, alpha, tiles_m,
                           tiles_n);
        ROV_LAUNCH_CHECK();
        return ROV_OK;
    }

    if (R != nullptr) return ROV_ERR_UNSUPPORTED;   // the residual epilogue exists on the MFMA path only
    const dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64)), block(256);
    if (grid.y > 65535u) return ROV_ERR_UNSUPPORTED;
    if (dtype == ROV_F32) {
        if (tb)
            hipLaunchKernelGGL((gemm_generic_kernel<float, float, true>), grid, block, 0, stream,
                               (const float*)A, (const float*)Bm, (float*)C, M, N, K, alpha);
        else
            hipLaunchKernelGGL((gemm_generic_kernel<float, float, false>), grid, block, 0, stream,
                               (const float*)A, (const float*)Bm, (float*)C, M, N, K, alpha);
    } else if (dtype == ROV_BF16) {
        if (tb)
            hipLaunchKernelGGL((gemm_generic_kernel<uint16_t, uint16_t, true>), grid, block, 0, stream,
                               (const uint16_t*)A, (const uint16_t*)Bm, (uint16_t*)C, M, N, K, alpha);
        else
            hipLaunchKernelGGL((gemm_generic_kernel<uint16_t, uint16_t, false>), grid, block, 0, stream,
                               (const uint16_t*)A, (const uint16_t*)Bm, (uint16_t*)C, M, N, K, alpha);
    } else {
        if (tb)
            hipLaunchKernelGGL((gemm_generic_kernel<uint8_t, uint16_t, true>), grid, block, 0, stream,
                               (const uint8_t*)A, (const uint8_t*)Bm, (uint16_t*)C, M, N, K, alpha);
        else
            hipLaunchKernelGGL((gemm_generic_kernel<uint8_t, uint16_t, false>), grid, block, 0, stream,
                               (const uint8_t*)A, (const uint8_t*)Bm, (uint16_t*)C, M, N, K, alpha);
    }
    ROV_LAUNCH_CHECK();
    return ROV_OK;
}

}  // namespace rov

extern "C" int rov_gemm(const void* A, const void* Bm, void* C, int M, int N, int K, int dtype,
                        int transB, float scaleA, float scaleB, void* stream) {
    return rov::launch_gemm(A, Bm, C, M, N, K, dtype, transB, scaleA, scaleB, (hipStream_t)stream);
}

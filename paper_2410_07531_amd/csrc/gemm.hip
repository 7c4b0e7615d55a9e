// GEMM for the QKV / PROJ / FC1 / FC2 layers that the RNG kernel hides behind
// (paper Sec. 3.2, Table 1 GEMM column: MMA-bound, L2 read bandwidth second).
//
// bf16 fast path (A [M,K] and weights [N,K], both K-contiguous):
//   - workgroup tile 256 x 256, 4 waves in a 2 x 2 grid, each wave owning a
//     128 x 128 block as 8 x 8 MFMA 16x16x32 tiles (256 fp32 accumulators per
//     lane, kept in AGPRs).  The 16x16x32 shape is used because under the
//     board's power limit it sustains about a quarter more flop/s on random
//     data than 32x32x16 (measured with a register-only loop: 2.05 against
//     1.66 PFLOP/s).  Narrower tiles (256 x 224 ... 128) are instances of the
//     same kernel; the launch picks the width that leaves least of the last
//     round of workgroups over the compute units empty;
//   - operands go from global memory straight into LDS (buffer_load ... lds,
//     16 bytes per lane) through two 64 KiB slots of 128-byte rows (two MFMA
//     k-steps per slot), loaded two slot-steps ahead and issued one load per
//     six MFMAs, so that the texture-address unit shared by the four waves
//     never sees a burst; a wave's 64 lanes always fill 1 KiB of consecutive
//     LDS, so the bank swizzle is applied on the global-address side;
//   - the fragments of a k-step are read from LDS during the k-step before
//     it, so no MFMA waits for an LDS read issued just before it;
//   - the MFMA is issued with the weight fragment as first operand, so each
//     lane ends up with 4 consecutive output columns and stores 8 bytes at once;
//   - workgroup ids are remapped so that the workgroups that land on one XCD
//     (one L2) cover a compact block of output tiles, and the k loop of a
//     workgroup starts at a k offset that depends on its tile row, so that the
//     workgroups of an XCD do not all fetch the same 128-byte column of every
//     row (the same cache channel) at the same time.
// The register budget (at most 408 of 512 registers, accumulators included)
// leaves room for RNG waves on every SIMD (the paper's carve-out, Sec. 6.2).
//
// fp8 (OCP e4m3) is the same kernel with another main loop: a 128-byte LDS row
// is one k-step of the double-rate MFMA 16x16x128 of the f8f6f4 family (twice
// the flop per byte; on random data under the power limit this shape sustains
// 4.55 PFLOP/s in a register-only loop against 4.0 for 32x32x64).
//
// Everything else (fp32, [K,N] weights, K not a multiple of the tile depth)
// takes a small LDS-tiled VALU kernel that is correct for any shape.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fp8_device.h"
#include "mask_device.h"
#include "philox_device.h"
#include "rov_internal.h"

#include <atomic>

namespace rov {
namespace {

std::atomic<int> g_tile_cols{0};   // rov_set_gemm_tile_cols: 0 = per shape


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
constexpr int BM = 256, BN = 256;                   // tile height; width of the widest tile
constexpr int kRowBytes = 128;                      // k per LDS row: 64 bf16 or 128 fp8 values
constexpr int kLdsBytes = 2 * (BM + BN) * kRowBytes;   // two slots of A rows then W rows: 128 KiB

typedef __attribute__((address_space(3))) void* lptr_t;
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Reads one accumulator value where it is needed.  The "a" constraint keeps the value in its
// accumulation register until this point, so the epilogue never needs a second copy of the
// 256 accumulators in ordinary VGPRs.
__device__ __forceinline__ float acc_read(float v) {
    float r;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(r) : "a"(v));
    return r;
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    f32x2 v = {lo, hi};
    bf16x2 h = __builtin_convertvector(v, bf16x2);
    return *reinterpret_cast<uint32_t*>(&h);
}

// What the epilogue does with the bf16 side input R[m][n] (four consecutive n per lane):
// EPI_ADD: C = acc + R (residual connection); EPI_SILU_MUL: C = silu(R) * acc (SwiGLU: R is the
// gate projection, acc the up projection, so the activation costs no kernel and no extra pass).
__device__ __forceinline__ void epilogue_combine(int epi, uint2 r, float& c0, float& c1, float& c2, float& c3) {
    const float r0 = __uint_as_float(r.x << 16), r1 = __uint_as_float(r.x & 0xFFFF0000u);
    const float r2 = __uint_as_float(r.y << 16), r3 = __uint_as_float(r.y & 0xFFFF0000u);
    if (epi == EPI_SILU_MUL) {
        c0 *= r0 / (1.0f + __expf(-r0));
        c1 *= r1 / (1.0f + __expf(-r1));
        c2 *= r2 / (1.0f + __expf(-r2));
        c3 *= r3 / (1.0f + __expf(-r3));
    } else {
        c0 += r0; c1 += r1; c2 += r2; c3 += r3;
    }
}

// bf16 inputs; output and side input are bf16.  NJ = weight-row blocks (16 rows) per wave: the
// workgroup tile is 256 x 32*NJ.  NJ = 8 moves the fewest bytes per flop; the narrower tiles exist
// for shapes whose tile count would otherwise leave the last round over the compute units partly
// empty (2048 x 14336: 448 tiles of 256 x 256 are 1.75 rounds over 256 units and take the time of
// 2; 512 tiles of 256 x 224 are 2 rounds of 7/8 the work each).
// FP8: the operands are OCP e4m3 bytes and a slot row (128 bytes) is one k-step of the double-rate
// MFMA 16x16x128 of the f8f6f4 family; everything but the main loop is shared with bf16.
// The tile of workgroup blockIdx.x, computed by the workgroup's waves 0-3 (`wave`; `lane` = lane
// in the wave).  Its barriers are workgroup barriers: 1 + 2*(K*2/128) of them for bf16, 1 + K/128
// for fp8, whatever the tile; any other wave of the workgroup has to arrive at as many.
// DUAL (SwiGLU, bf16): the tile's weight rows are, per wave, 8*NJ rows of Wt (the gate
// projection) followed by the same 8*NJ rows of Wt2 (the up projection); the epilogue writes
// silu(gate) * up for those 8*NJ output columns, both still in fp32, so the gate projection is
// neither stored nor read back and the activation panel is fetched once for the two products.
// OUT8 (dual form only): the result is written as OCP e4m3 bytes, out_inv * silu(alpha * gate) *
// (alpha2 * up) rounded to the nearest code, the SwiGLU output of the fp8 block quantised where it
// is produced; C then points at bytes.
template <int NJ, bool FP8, bool DUAL = false, bool OUT8 = false>
__device__ __forceinline__ void gemm_tile(const char* __restrict__ A, const char* __restrict__ Wt,
                                          const char* __restrict__ Wt2, uint16_t* __restrict__ C,
                                          const uint16_t* __restrict__ R, int M, int N, int K, float alpha,
                                          int tiles_m, int tiles_n, int epi, char* lds, const int lane,
                                          const int wave, float alpha2 = 1.0f, float out_inv = 1.0f) {
    static_assert(!DUAL || NJ == 8 || NJ == 4, "dual form: 8 or 4 weight blocks per wave");
    static_assert(!OUT8 || DUAL, "e4m3 output exists in the dual form only");
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
    constexpr int BNT = DUAL ? 16 * NJ : 32 * NJ;   // tile width in output columns
    const int m0 = tm * BM, n0 = tn * BNT;

    constexpr int ESZ = FP8 ? 1 : 2;
    f32x4 acc[NJ][8];   // [weight-row block j (16 rows)][activation-row block i (16 rows)]
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[j][i][e] = 0.0f;

    // Ring slot of this kernel: 128 bytes of k per row (two MFMA k-steps), A rows then W rows,
    // 64 KiB; two slots.  A load instruction moves 8 rows x 128 bytes, i.e. whole 128-byte lines of
    // the row-major operand: with 64-byte row pieces the same L2 -> LDS stream reached 15 TB/s on
    // this chip, with whole lines 26 TB/s, and this kernel is bound by that stream.
    constexpr int kRow = kRowBytes;
    constexpr int kSlot = (BM + BN) * kRow;      // slot stride (the widest tile's); W rows follow the A rows
    static_assert(2 * kSlot <= kLdsBytes, "two slots fit the launch's LDS");
    // 16-byte chunk swizzle of a 128-byte LDS row (8 chunks, two rows per 256 bytes of banks): the
    // chunk index is XORed with (row / 2) % 8.  A 64-lane ds_read_b128 is served 16 lanes at a time
    // over 64 banks of 4 bytes, and the lanes that go together are not consecutive: measured on
    // gfx950 with a two-lane probe and the bank-conflict counter, they are {0-3, 12-15, 20-27},
    // {4-11, 16-19, 28-31} and the same two sets + 32.  A fragment read has lane = 16*chunk + row;
    // such a set then holds, per row parity, 8 rows whose XOR values are all different: 16
    // different bank groups (counter: 0 conflict cycles).
    auto swz = [](int row) { return (row >> 1) & 7; };
    // fragment of MFMA 16x16x32: lane holds row lane%16, k-chunk (8 bf16) lane/16 of k-step h (fp8:
    // the same two 16-byte pieces together are the lane's operand of the one MFMA 16x16x128)
    const int frow = lane & 15;
    const int fchunk = lane >> 4;
    int foff[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) foff[h] = frow * kRow + (((4 * h + fchunk) ^ swz(frow)) << 4);   // block bases are multiples of 16
    const int a_base = (wm * 128) * kRow;
    const int w_base = BM * kRow + (wn * 16 * NJ) * kRow;

    // Loads: wave w issues row blocks (8 rows) w, w+4, ... of each operand: 8 + NJ instructions
    // per slot.  Lane L fills physical chunk L%8 of row L/8, i.e. fetches logical chunk (L%8) ^ swz(row).
    const size_t ld_bytes = (size_t)K * ESZ;
    const int ns = (int)(ld_bytes / kRow);            // slots to walk
    const int rows_a = M - m0 < BM ? M - m0 : BM;
    const int rows_w = N - n0 < BNT ? N - n0 : BNT;
    uint32_t voff_a[8], voff_w[NJ];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int row = (wave + 4 * j) * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ swz(row);
        const int ra = row < rows_a ? row : rows_a - 1;   // rows past the edge are never stored
        // dual: LDS rows [16*NJ*h, +8*NJ) are gate rows of output columns 8*NJ*h .., the next 8*NJ the up rows
        const int wcol = DUAL ? (row / (16 * NJ)) * (8 * NJ) + row % (8 * NJ) : row;
        const int rw = wcol < rows_w ? wcol : rows_w - 1;
        voff_a[j] = (uint32_t)((size_t)ra * ld_bytes) + (uint32_t)(chunk * 16);
        if (j < NJ) voff_w[j] = (uint32_t)((size_t)rw * ld_bytes) + (uint32_t)(chunk * 16);
    }
    const char* a_panel = A + (size_t)m0 * ld_bytes;
    const char* w_panel = Wt + (size_t)n0 * ld_bytes;
    // slot at which this workgroup starts its cyclic walk over k (the sum does not depend on the
    // order; the fp32 rounding does, deterministically)
    const int kstart = (int)((unsigned)tm % (unsigned)ns);
    // Buffer resources over the two operand panels (scalar base, per-lane 32-bit offset, scalar k
    // offset; the range ends with the last valid row, so an offset beyond it would read zeros).
    auto make_rsrc = [](const char* base, size_t bytes) {
        const uint64_t b = (uint64_t)(uintptr_t)base;
        i32x4 r;
        r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)b);
        r[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)((b >> 32) & 0xFFFFu));
        r[2] = __builtin_amdgcn_readfirstlane((int)(uint32_t)bytes);
        r[3] = 0x00020000;
        return r;
    };
    const i32x4 rsrc_a = make_rsrc(a_panel, (size_t)rows_a * ld_bytes);
    const i32x4 rsrc_w = make_rsrc(w_panel, (size_t)rows_w * ld_bytes);
    const i32x4 rsrc_w2 = DUAL ? make_rsrc(Wt2 + (size_t)n0 * ld_bytes, (size_t)rows_w * ld_bytes) : rsrc_w;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lptr_t)lds;

    // Load instruction q (0..7 = A row blocks, 8..7+NJ = W row blocks) of slot-step `step` into the
    // slot at LDS byte address `slot`.  Inline assembly, so that the compiler's wait-count pass does
    // not see an LDS write it cannot tell apart from the fragment reads (it would force vmcnt(0)
    // before every LDS read); the waits are placed by hand below.  M0 (the LDS base of the
    // transfer) is a reserved register that compiled code only sets right before its own uses.
    auto issue = [&](int q, int step, uint32_t slot) {
        int st = step < ns ? step : ns - 1;       // past the end: harmless reload of the last slot
        st += kstart;
        st = st >= ns ? st - ns : st;
        const int koff = st * kRow;
        if (q < 8) {
            const uint32_t dst = slot + (uint32_t)((wave + 4 * q) * 1024);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                         :: "s"(dst), "v"(voff_a[q]), "s"(rsrc_a), "s"(koff) : "memory");
        } else {
            const uint32_t dst = slot + (uint32_t)(BM * kRow + (wave + 4 * (q - 8)) * 1024);
            // dual: row block wave + 4*(q-8) holds up rows iff it lies in the second half of its wave's
            // 2*NJ row blocks; with NJ = 8 or 4 that does not depend on the wave
            const bool up = DUAL && (4 * (q - 8)) % (2 * NJ) >= NJ;
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                         :: "s"(dst), "v"(voff_w[q - 8]), "s"(up ? rsrc_w2 : rsrc_w), "s"(koff) : "memory");
        }
    };

    if constexpr (FP8) {
        // fp8: one slot-step is ONE k-step of NM = 8*NJ MFMAs 16x16x128 (32 cycles each).  A lane's
        // 32-byte operand is made of the same two 16-byte pieces the bf16 path reads (chunk lane/16 of
        // each half row): which k values a lane group holds does not matter as long as both operands
        // agree, and it keeps the bf16 swizzle and its conflict-free reads.
        // All fragments of a step must be in registers when it starts and there is no room for a
        // second set (256 accumulators + 128 fragment registers), so the next step's fragments
        // replace the current ones as these retire: the MFMAs go weight block by weight block, weight
        // fragment j of slot-step S+1 is read once row j is done, activation fragment i after the last
        // row's MFMA i (the last of each kind at the start of step S+1, from what is then the current
        // slot).  One barrier per step, after row 0: by then a wave has read the last of LDS slot S
        // and its loads of slot-step S+1 (all issued during step S-1) are waited for; after it, slot
        // S+1 is read and slot S takes the loads of slot-step S+2, one per G MFMAs.
        i32x8 a8[8], w8[NJ];
        auto read_half = [&](const char* slot, int f /*0..7 = A block, 8..7+NJ = W block*/, int h) {
            const i32x4 v = *reinterpret_cast<const i32x4*>(
                slot + (f < 8 ? a_base + f * 16 * kRow : w_base + (f - 8) * 16 * kRow) + foff[h]);
            i32x8& dst = f < 8 ? a8[f] : w8[f - 8];
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[4 * h + e] = v[e];
        };
        auto mfma8 = [&](int j, int i) {
            asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0" : "+a"(acc[j][i]) : "v"(w8[j]), "v"(a8[i]));
        };
        constexpr int NM = 8 * NJ, NL = 8 + NJ;
        constexpr int G0 = (NM - 17) / (NL - 1);
        constexpr int G = G0 < 1 ? 1 : (G0 > 3 ? 3 : G0);
        static_assert(9 + G * (NL - 1) < NM, "the loads of a slot-step are issued within one step");
#pragma unroll
        for (int q = 0; q < NL; ++q) issue(q, 0, lds_base);
#pragma unroll
        for (int q = 0; q < NL; ++q) issue(q, 1, lds_base + kSlot);
        __builtin_amdgcn_s_waitcnt(0x0F70 | (NL & 15) | ((NL >> 4) << 14));   // vmcnt(NL): slot-step 0 has landed
        __syncthreads();
#pragma unroll
        for (int f = 0; f < 7; ++f) { read_half(lds, f, 0); read_half(lds, f, 1); }
#pragma unroll
        for (int f = 8; f < 8 + NJ - 1; ++f) { read_half(lds, f, 0); read_half(lds, f, 1); }
        // nothing pending at loop entry: the waits the compiler places in the loop are then those of
        // the loop's own read order, not of whatever order it gave the reads above
        __builtin_amdgcn_s_waitcnt(0xC07F);
        for (int S = 0; S < ns; ++S) {
            const char* cur = lds + (S & 1) * kSlot;
            const char* nxt = lds + ((S + 1) & 1) * kSlot;
#pragma unroll
            for (int idx = 0; idx < NM; ++idx) {
                if (idx == 8) {
                    __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0)
                    __syncthreads();
                }
                mfma8(idx >> 3, idx & 7);
                // the last activation and the last weight fragment of this step: their registers were
                // in use until the last MFMA of the step before
                if (idx == 0) { read_half(cur, 7, 0); read_half(cur, 7, 1); }
                if (idx == 1) { read_half(cur, 8 + NJ - 1, 0); read_half(cur, 8 + NJ - 1, 1); }
                if (idx >= 9 && (idx & 7) == 1) read_half(nxt, 8 + (idx >> 3) - 1, 0);
                if (idx >= 9 && (idx & 7) == 2) read_half(nxt, 8 + (idx >> 3) - 1, 1);
                if (idx >= NM - 7) {                      // MFMA (NJ-1, i) has been issued one MFMA ago for i = idx - (NM-7)
                    read_half(nxt, idx - (NM - 7), 0);
                    read_half(nxt, idx - (NM - 7), 1);
                }
                if (idx >= 9 && (idx - 9) % G == 0 && (idx - 9) / G < NL) issue((idx - 9) / G, S + 2, lds_base + (S & 1) * kSlot);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    } else {
        i32x4 af[2][8], wf[2][NJ];   // fragments of the two k-steps of a slot
        auto read_frag = [&](int h, const char* slot, int f /*0..7 = A block, 8..7+NJ = W block*/) {
            if (f < 8)
                af[h][f] = *reinterpret_cast<const i32x4*>(slot + a_base + f * 16 * kRow + foff[h]);
            else
                wf[h][f - 8] = *reinterpret_cast<const i32x4*>(slot + w_base + (f - 8) * 16 * kRow + foff[h]);
        };
        // The MFMAs are written as inline assembly with explicit register classes (accumulators in
        // AGPRs, fragments in VGPRs): left to itself the register allocator mixes the two files for 64
        // four-register accumulators and fills the loop with accumulator moves and spills.
        auto mfma_one = [&](int h, int j, int i) {
            asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[j][i]) : "v"(wf[h][j]), "v"(af[h][i]));
        };

        // Two slots; slot-step S lives in slot S % 2 and is two k-steps, (S,0) and (S,1), of NM = 8*NJ
        // MFMAs each.
        //   (S,0): MFMAs on the fragments of (S,0); the NF = 8+NJ fragments of (S,1) are read from slot S.
        //   then:  own LDS reads done, barrier: slot S is free.
        //   (S,1): MFMAs on (S,1); at MFMA HB = NM - 2*NF: own loads of slot-step S+1 landed, barrier
        //          (slot S+1 is complete for every wave), then the fragments of (S+1,0) are read from it,
        //          one per 2 MFMAs, which takes the rest of the k-step.
        // Loads of slot-step S+2 (into slot S), NL = 8+NJ per wave, go out one per G MFMAs: P1 of them
        // in (S,1), the rest in (S+1,0).  The four waves share one texture-address unit that takes 16
        // cycles per load, as long as an MFMA runs, and a wave issues nothing while its load waits
        // there: at one load per 2 MFMAs per wave the unit is oversubscribed and the matrix pipe starves
        // (measured with loads that touch no memory, zero operands: 1.79 PFLOP/s at one per 2, 1.94 at
        // one per 4).  At the barrier inside (S,1) a wave has issued VMB younger loads: vmcnt(VMB).
        // Letting the waves take turns behind different MFMAs would remove the rest of the queueing,
        // but a taken branch around the load costs more than the load, and a load under an empty EXEC
        // mask still costs its 16 cycles (both measured: 20 % and 35 % slower).
        constexpr int NM = 8 * NJ, NF = 8 + NJ, NL = 8 + NJ;
        constexpr int G = NJ >= 5 ? 6 : 5;
        constexpr int HB = NM - 2 * NF;
        constexpr int P1 = (NM - 2) / G + 1;               // load slots idx % G == 1 of a k-step
        constexpr int P0 = NM >= 4 ? (NM - 4) / G + 1 : 0; // load slots idx % G == 3 of a k-step
        constexpr int VMB = HB >= 2 ? (HB - 2) / G + 1 : 0;
        static_assert(HB >= 0 && P1 <= NL && NL - P1 <= P0 && VMB < 16, "load schedule fits the k-steps");
#pragma unroll
        for (int q = 0; q < NL; ++q) issue(q, 0, lds_base);
#pragma unroll
        for (int q = 0; q < P1; ++q) issue(q, 1, lds_base + kSlot);   // its other loads go out in (0,0) like everywhere below
        __builtin_amdgcn_s_waitcnt(0x0F70 | P1);   // vmcnt(P1): slot-step 0 has landed
        __syncthreads();
#pragma unroll
        for (int f = 0; f < NF; ++f) read_frag(0, lds, f);

        for (int S = 0; S < ns; ++S) {
            const char* cur = lds + (S & 1) * kSlot;
            const char* nxt = lds + ((S + 1) & 1) * kSlot;
            __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): fragments of (S,0)
#pragma unroll
            for (int idx = 0; idx < NM; ++idx) {
                mfma_one(0, idx >> 3, idx & 7);
                if (idx < 2 * NF && (idx & 1) == 0) read_frag(1, cur, idx >> 1);
                if (idx % G == 3 && P1 + idx / G < NL) issue(P1 + idx / G, S + 1, lds_base + ((S + 1) & 1) * kSlot);   // the other loads of slot-step S+1
                __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): fragments of (S,1)
            __syncthreads();
#pragma unroll
            for (int idx = 0; idx < NM; ++idx) {
                if (idx == HB) {
                    __builtin_amdgcn_s_waitcnt(0x0F70 | VMB);   // vmcnt(VMB)
                    __syncthreads();
                }
                mfma_one(1, idx >> 3, idx & 7);
                if (idx % G == 1) issue(idx / G, S + 2, lds_base + (S & 1) * kSlot);          // loads 0..P1-1 of slot-step S+2
                if (idx >= HB && ((idx - HB) & 1) == 0) read_frag(0, nxt, (idx - HB) >> 1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): no LDS load may outlive the loop
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");   // the last MFMA results are in the accumulators before they are read

    // D'[r][c] = C[m = c][n = r]: lane holds activation row lane%16 and weight rows 4*(lane/16) + e
    const int mrow = lane & 15;
    const int nsub = (lane >> 4) * 4;
    if constexpr (DUAL) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int m = m0 + wm * 128 + i * 16 + mrow;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < NJ / 2; ++j) {
                const int n = n0 + wn * 8 * NJ + j * 16 + nsub;
                float o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float gte = alpha * acc_read(acc[j][i][e]);
                    const float upv = (DUAL && OUT8 ? alpha2 : alpha) * acc_read(acc[j + NJ / 2][i][e]);
                    o[e] = gte / (1.0f + __expf(-gte)) * upv;
                }
                if (m < M && n < N) {
                    if constexpr (OUT8) {
                        *reinterpret_cast<uint32_t*>(reinterpret_cast<uint8_t*>(C) + (size_t)m * N + n) =
                            pack_e4m3x4(o[0] * out_inv, o[1] * out_inv, o[2] * out_inv, o[3] * out_inv);
                    } else {
                        uint2 v;
                        v.x = pack_bf16x2(o[0], o[1]);
                        v.y = pack_bf16x2(o[2], o[3]);
                        *reinterpret_cast<uint2*>(C + (size_t)m * N + n) = v;
                    }
                }
            }
        }
        return;
    }
    // The side input of row block i+1 is requested before row block i is combined and stored, so
    // its latency is paid once per tile, not once per element group (the wave is alone on its SIMD).
    uint2 rv[2][NJ];
    auto load_side = [&](int i, uint2 (&dst)[NJ]) {
        const int m = m0 + wm * 128 + i * 16 + mrow;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int n = n0 + wn * 16 * NJ + j * 16 + nsub;
            dst[j] = make_uint2(0u, 0u);
            if (m < M && n < N) dst[j] = *reinterpret_cast<const uint2*>(R + (size_t)m * N + n);
        }
    };
    if (R != nullptr) load_side(0, rv[0]);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int m = m0 + wm * 128 + i * 16 + mrow;
        __builtin_amdgcn_sched_barrier(0);
        if (R != nullptr && i + 1 < 8) load_side(i + 1, rv[(i + 1) & 1]);
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int n = n0 + wn * 16 * NJ + j * 16 + nsub;
            float c0 = alpha * acc_read(acc[j][i][0]);
            float c1 = alpha * acc_read(acc[j][i][1]);
            float c2 = alpha * acc_read(acc[j][i][2]);
            float c3 = alpha * acc_read(acc[j][i][3]);
            if (m < M && n < N) {
                if (R != nullptr) epilogue_combine(epi, rv[i & 1][j], c0, c1, c2, c3);
                uint2 v;
                v.x = pack_bf16x2(c0, c1);
                v.y = pack_bf16x2(c2, c3);
                *reinterpret_cast<uint2*>(C + (size_t)m * N + n) = v;
            }
        }
    }
}

template <int NJ, bool FP8 = false>
__global__ __launch_bounds__(256, 1) void gemm_tn_kernel(const char* __restrict__ A,
                                                         const char* __restrict__ Wt,
                                                         uint16_t* __restrict__ C,
                                                         const uint16_t* __restrict__ R, int M, int N,
                                                         int K, float alpha, int tiles_m, int tiles_n, int epi) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    // Co-resident RNG waves only need the VALU issue slots this kernel leaves idle; raise this
    // wave's issue priority so that they never delay its MFMA / LDS instruction stream.
    __builtin_amdgcn_s_setprio(3);
    gemm_tile<NJ, FP8>(A, Wt, nullptr, C, R, M, N, K, alpha, tiles_m, tiles_n, epi, lds, threadIdx.x & 63,
                       __builtin_amdgcn_readfirstlane(threadIdx.x >> 6));
}

// C[M, N] = silu(A Wg^T) * (A Wu^T): the SwiGLU of the block's feed-forward as one product with
// twice the weight rows (see gemm_tile, DUAL).
template <int NJ>
__global__ __launch_bounds__(256, 1) void gemm_swiglu_kernel(const char* __restrict__ A, const char* __restrict__ Wg,
                                                            const char* __restrict__ Wu, uint16_t* __restrict__ C,
                                                            int M, int N, int K, int tiles_m, int tiles_n) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    __builtin_amdgcn_s_setprio(3);
    gemm_tile<NJ, false, true>(A, Wg, Wu, C, nullptr, M, N, K, 1.0f, tiles_m, tiles_n, EPI_ADD, lds,
                               threadIdx.x & 63, __builtin_amdgcn_readfirstlane(threadIdx.x >> 6));
}

// The same for the fp8 block: e4m3 activations and weights (alpha_g, alpha_u: activation scale times
// the weight's scale), e4m3 result, out_inv = 1 / (the result's dequantisation scale).
template <int NJ>
__global__ __launch_bounds__(256, 1) void gemm_swiglu_fp8_kernel(const char* __restrict__ A, const char* __restrict__ Wg,
                                                                const char* __restrict__ Wu, uint8_t* __restrict__ C,
                                                                int M, int N, int K, int tiles_m, int tiles_n,
                                                                float alpha_g, float alpha_u, float out_inv) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    __builtin_amdgcn_s_setprio(3);
    gemm_tile<NJ, true, true, true>(A, Wg, Wu, reinterpret_cast<uint16_t*>(C), nullptr, M, N, K, alpha_g, tiles_m, tiles_n,
                                    EPI_ADD, lds, threadIdx.x & 63, __builtin_amdgcn_readfirstlane(threadIdx.x >> 6),
                                    alpha_u, out_inv);
}

// Wave-specialised GEMM + RNG (paper Sec. 6.1 names this form beside the two-kernel one): a
// workgroup of eight waves, two per SIMD; waves 0-3 compute a 256 x 128 bf16 tile exactly as
// gemm_tn_kernel<4> does (the only tile whose 244 registers leave room for a second wave on the
// SIMD: every wave of a kernel gets the same allocation), waves 4-7 generate keep-mask chunks
// pulled from a work queue, one group of 64 Philox calls per 128 bytes of k, arriving at every
// barrier the tile's waves arrive at (a group per barrier interval made the tile's waves wait
// longer: measured 341 against 333 us on 2048 x 14336 x 4096 with a 32 x 2048^2-bit mask).  A chunk that was started is
// finished after the tile's k loop, while the other waves store the tile; chunks never started
// stay in the queue for whoever drains it next.
__global__ __launch_bounds__(512, 1) void gemm_rng_kernel(const char* __restrict__ A, const char* __restrict__ Wt,
                                                         uint16_t* __restrict__ C, int M, int N, int K,
                                                         int tiles_m, int tiles_n, uint64_t* __restrict__ mask,
                                                         uint64_t words, uint64_t nchunks, uint64_t offset,
                                                         uint32_t k0, uint32_t k1, uint32_t t_minus_1,
                                                         QueueCounter* queues, uint64_t qper) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (wave < 4) {
        __builtin_amdgcn_s_setprio(3);
        gemm_tile<4, false>(A, Wt, nullptr, C, nullptr, M, N, K, 1.0f, tiles_m, tiles_n, EPI_ADD, lds, lane, wave);
    } else {
        ChunkSource src;
        src.queues = queues; src.nchunks = nchunks; src.stride = 0; src.per = qper; src.batch = 1u;
        src.lane = (uint32_t)lane;
        bool have = false, popped = false, dry = false;
        int gi = 0;
        uint32_t vlo = 0u, vhi = 0u;
        // one group of the current chunk: four keep words into lanes 4*gi .. 4*gi+3; the 16th group
        // stores the chunk.  A chunk is popped only when its first group is about to be computed, so
        // that none is taken from the queue and then left undone.
        auto unit = [&]() {
            if (!have) {
                if (dry) return;
                have = popped ? src.next() : src.first((uint64_t)blockIdx.x * 4u + (uint32_t)(wave - 4));
                popped = true;
                if (!have) {
                    dry = true;
                    return;
                }
            }
            const uint64_t base = offset + 64u * kGroupsPerChunk * src.cur;   // first call of the chunk
            uint64_t b[4];
            if ((uint32_t)base <= 0xFFFFFFFFu - (64u * kGroupsPerChunk - 1u))
                philox_group_ballots<10, false>(base + 64u * (uint64_t)gi, (uint32_t)lane, k0, k1, t_minus_1, b);
            else
                philox_group_ballots<10, true>(base + 64u * (uint64_t)gi, (uint32_t)lane, k0, k1, t_minus_1, b);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const uint32_t dst = 4u * (uint32_t)gi + (uint32_t)r;
                vlo = write_lane((uint32_t)b[r], dst, vlo);
                vhi = write_lane((uint32_t)(b[r] >> 32), dst, vhi);
            }
            if (++gi == kGroupsPerChunk) {
                const uint64_t widx = src.cur * 64u + (uint32_t)lane;
                if (widx < words) mask[widx] = ((uint64_t)vhi << 32) | vlo;
                gi = 0;
                vlo = 0u;
                vhi = 0u;
                have = false;
            }
        };
        // the tile's barriers: one before its k loop, two per 128 bytes of k
        const int ns = (int)(((size_t)K * 2) / kRowBytes);
        __syncthreads();
        for (int S = 0; S < ns; ++S) {
            unit();
            __syncthreads();   // the tile's "slot free" barrier
            __syncthreads();   // the tile's "next slot complete" barrier
        }
        while (have) unit();   // finish the chunk that was started
    }
}

}  // namespace

int check_gemm_swiglu(const void* A, const void* Wg, const void* Wu, const void* C, int M, int N, int K) {
    if (A == nullptr || Wg == nullptr || Wu == nullptr || C == nullptr || M <= 0 || N <= 0 || K <= 0)
        return ROV_ERR_INVALID;
    if (!aligned(A, 16) || !aligned(Wg, 16) || !aligned(Wu, 16) || !aligned(C, 16)) return ROV_ERR_INVALID;
    if (((size_t)K * 2) % kRowBytes != 0 || (N % 4) != 0) return ROV_ERR_UNSUPPORTED;
    if ((unsigned long long)BM * (unsigned long long)K * 2ull > 0xFFFFFFFFull) return ROV_ERR_UNSUPPORTED;
    if ((long long)((M + BM - 1) / BM) * ((N + 63) / 64) > 0x7FFFFFFFLL) return ROV_ERR_UNSUPPORTED;
    return ROV_OK;
}

int launch_gemm_swiglu(const void* A, const void* Wg, const void* Wu, void* C, int M, int N, int K,
                       hipStream_t stream) {
    {
        const int rc = check_gemm_swiglu(A, Wg, Wu, C, M, N, K);
        if (rc != ROV_OK) return rc;
    }
    // 128 or 64 output columns per tile (8 or 4 weight blocks per wave, half gate, half up).  The
    // narrow tile takes 0.67 of the wide tile's time for half of its work (measured on
    // 2048...8192 x 14336 x 4096), so it is chosen only where it saves more than a third of the rounds
    const long long tiles_m = (M + BM - 1) / BM, ncu = device_cu_count();
    const long long t8 = tiles_m * ((N + 127) / 128), t4 = tiles_m * ((N + 63) / 64);
    const int forced = g_tile_cols.load();    // rov_set_gemm_tile_cols: 256 forces the wide tile, 128 the narrow one
    const bool wide = forced == 256 ? true : forced == 128 ? false
                                                           : ((t8 + ncu - 1) / ncu) * 3 <= ((t4 + ncu - 1) / ncu) * 2;
    const long long T = wide ? t8 : t4;
    if (T > 0x7FFFFFFFLL) return ROV_ERR_UNSUPPORTED;
    typedef void (*kern_t)(const char*, const char*, const char*, uint16_t*, int, int, int, int, int);
    const kern_t kern = wide ? (kern_t)gemm_swiglu_kernel<8> : (kern_t)gemm_swiglu_kernel<4>;
    {
        const int rc = set_max_dynamic_lds((const void*)kern, kLdsBytes);
        if (rc != ROV_OK) return rc;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)T), dim3(256), kLdsBytes, stream, (const char*)A, (const char*)Wg,
                       (const char*)Wu, (uint16_t*)C, M, N, K, (int)tiles_m, (int)(T / tiles_m));
    ROV_LAUNCH_CHECK();
    return ROV_OK;
}

int check_gemm_rng(const void* A, const void* Bm, const void* C, int M, int N, int K, int B, int H, int S, float p,
                   const uint64_t* mask) {
    if (A == nullptr || Bm == nullptr || C == nullptr || mask == nullptr || M <= 0 || N <= 0 || K <= 0 ||
        B <= 0 || H <= 0 || S <= 0)
        return ROV_ERR_INVALID;
    if (!aligned(A, 16) || !aligned(Bm, 16) || !aligned(C, 16) || !aligned(mask, 8)) return ROV_ERR_INVALID;
    uint32_t tm1;
    if (!keep_threshold_minus_1(p, &tm1)) return ROV_ERR_INVALID;
    if (((size_t)K * 2) % kRowBytes != 0 || (N % 4) != 0 || (S % 32) != 0) return ROV_ERR_UNSUPPORTED;
    if ((unsigned long long)BM * (unsigned long long)K * 2ull > 0xFFFFFFFFull) return ROV_ERR_UNSUPPORTED;
    const uint64_t Tt = (uint64_t)S / 32u;
    const long double wd = (long double)B * H * Tt * Tt * 16.0L;
    if (wd > 1099511627776.0L) return ROV_ERR_UNSUPPORTED;
    if ((long long)((M + BM - 1) / BM) * ((N + 127) / 128) > 0x7FFFFFFFLL) return ROV_ERR_UNSUPPORTED;
    return ROV_OK;
}

int check_gemm_swiglu_fp8(const void* A, const void* Wg, const void* Wu, const void* C, int M, int N, int K,
                          float scaleC) {
    if (A == nullptr || Wg == nullptr || Wu == nullptr || C == nullptr || M <= 0 || N <= 0 || K <= 0)
        return ROV_ERR_INVALID;
    if (!aligned(A, 16) || !aligned(Wg, 16) || !aligned(Wu, 16) || !aligned(C, 4)) return ROV_ERR_INVALID;
    if (!(scaleC > 0.0f)) return ROV_ERR_INVALID;
    if (((size_t)K) % kRowBytes != 0 || (N % 4) != 0) return ROV_ERR_UNSUPPORTED;
    if ((unsigned long long)BM * (unsigned long long)K > 0xFFFFFFFFull) return ROV_ERR_UNSUPPORTED;
    if ((long long)((M + BM - 1) / BM) * ((N + 63) / 64) > 0x7FFFFFFFLL) return ROV_ERR_UNSUPPORTED;
    return ROV_OK;
}

int launch_gemm_swiglu_fp8(const void* A, const void* Wg, const void* Wu, void* C, int M, int N, int K,
                           float scaleA, float scaleWg, float scaleWu, float scaleC, hipStream_t stream) {
    {
        const int rc = check_gemm_swiglu_fp8(A, Wg, Wu, C, M, N, K, scaleC);
        if (rc != ROV_OK) return rc;
    }
    const long long tiles_m = (M + BM - 1) / BM, ncu = device_cu_count();
    const long long t8 = tiles_m * ((N + 127) / 128), t4 = tiles_m * ((N + 63) / 64);
    const int forced = g_tile_cols.load();
    const bool wide = forced == 256 ? true : forced == 128 ? false
                                                           : ((t8 + ncu - 1) / ncu) * 3 <= ((t4 + ncu - 1) / ncu) * 2;
    const long long T = wide ? t8 : t4;
    typedef void (*kern_t)(const char*, const char*, const char*, uint8_t*, int, int, int, int, int, float, float, float);
    const kern_t kern = wide ? (kern_t)gemm_swiglu_fp8_kernel<8> : (kern_t)gemm_swiglu_fp8_kernel<4>;
    {
        const int rc = set_max_dynamic_lds((const void*)kern, kLdsBytes);
        if (rc != ROV_OK) return rc;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)T), dim3(256), kLdsBytes, stream, (const char*)A, (const char*)Wg,
                       (const char*)Wu, (uint8_t*)C, M, N, K, (int)tiles_m, (int)(T / tiles_m), scaleA * scaleWg,
                       scaleA * scaleWu, 1.0f / scaleC);
    ROV_LAUNCH_CHECK();
    return ROV_OK;
}

int launch_gemm_rng(const void* A, const void* Bm, void* C, int M, int N, int K, uint64_t seed, uint64_t offset,
                    int B, int H, int S, float p, uint64_t* mask, int qslot, hipStream_t stream) {
    {
        const int rc0 = check_gemm_rng(A, Bm, C, M, N, K, B, H, S, p, mask);
        if (rc0 != ROV_OK) return rc0;
    }
    uint32_t tm1;
    (void)keep_threshold_minus_1(p, &tm1);
    const uint64_t Tt = (uint64_t)S / 32u;
    const uint64_t words = (uint64_t)B * (uint64_t)H * Tt * Tt * 16u, nchunks = (words + 63u) / 64u;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + 127) / 128;
    const long long T = (long long)tiles_m * tiles_n;
    if (T > 0x7FFFFFFFLL) return ROV_ERR_UNSUPPORTED;
    void* q = nullptr;
    int rc = mask_queue_device_ptr(qslot, &q);
    if (rc != ROV_OK) return rc;
    uint64_t qper = 0;
    uint32_t qbatch = 1;
    mask_queue_geometry(nchunks, &qper, &qbatch);
    rc = set_max_dynamic_lds((const void*)gemm_rng_kernel, kLdsBytes);
    if (rc != ROV_OK) return rc;
    hipLaunchKernelGGL(gemm_rng_kernel, dim3((unsigned)T), dim3(512), kLdsBytes, stream, (const char*)A,
                       (const char*)Bm, (uint16_t*)C, M, N, K, tiles_m, tiles_n, mask, words, nchunks, offset,
                       (uint32_t)seed, (uint32_t)(seed >> 32), tm1, (QueueCounter*)q, qper);
    ROV_LAUNCH_CHECK();
    return ROV_OK;
}

// Tile width (output columns, 32*nj) for an M x N product.  The workgroups run in rounds of one per
// compute unit; a tile costs about nj + 1 units (its A panel does not shrink with it), so the width
// with the smallest rounds x (nj + 1) is taken, the widest on ties; a width set through
// rov_set_gemm_tile_cols overrides the rule.
int pick_tile_cols(int M, int N) {
    const int forced = g_tile_cols.load();
    if (forced != 0) return forced;
    const long long tiles_m = (M + BM - 1) / BM, ncu = device_cu_count();
    long long best = -1;
    int nj = 8;
    for (int c = 8; c >= 4; --c) {
        const long long t = tiles_m * ((N + 32 * c - 1) / (32 * c));
        const long long cost = ((t + ncu - 1) / ncu) * (c + 1);
        if (best < 0 || cost < best) { best = cost; nj = c; }
    }
    return 32 * nj;
}

int launch_gemm(const void* A, const void* Bm, void* C, int M, int N, int K, int dtype, int transB,
                float scaleA, float scaleB, hipStream_t stream) {
    return launch_gemm_residual(A, Bm, C, nullptr, M, N, K, dtype, transB, scaleA, scaleB, stream);
}

int launch_gemm_residual(const void* A, const void* Bm, void* C, const void* R, int M, int N, int K,
                         int dtype, int transB, float scaleA, float scaleB, hipStream_t stream) {
    return launch_gemm_epilogue(A, Bm, C, R, EPI_ADD, M, N, K, dtype, transB, scaleA, scaleB, stream);
}

// Everything launch_gemm_epilogue refuses, without launching: the schedules call this for every
// product of a sequence before they enqueue the first kernel.
int check_gemm(const void* A, const void* Bm, const void* C, const void* R, int epi, int M, int N, int K,
               int dtype, int transB) {
    if (epi != EPI_ADD && epi != EPI_SILU_MUL) return ROV_ERR_INVALID;
    if (R != nullptr && !aligned(R, 8)) return ROV_ERR_INVALID;
    if (A == nullptr || Bm == nullptr || C == nullptr || M <= 0 || N <= 0 || K <= 0)
        return ROV_ERR_INVALID;
    if (!aligned(A, 16) || !aligned(Bm, 16) || !aligned(C, 16)) return ROV_ERR_INVALID;
    if (dtype != ROV_F32 && dtype != ROV_BF16 && dtype != ROV_FP8_E4M3) return ROV_ERR_INVALID;
    const int esz = dtype == ROV_BF16 ? 2 : 1;
    if (dtype != ROV_F32 && transB != 0 && ((size_t)K * esz) % kRowBytes == 0 && (N % 4) == 0) {
        if ((unsigned long long)BM * (unsigned long long)K * (unsigned long long)esz > 0xFFFFFFFFull)
            return ROV_ERR_UNSUPPORTED;
        // (tile count of the narrowest tile: an upper bound for every width)
        if ((long long)((M + BM - 1) / BM) * ((N + 127) / 128) > 0x7FFFFFFFLL) return ROV_ERR_UNSUPPORTED;
        return ROV_OK;
    }
    if (R != nullptr) return ROV_ERR_UNSUPPORTED;   // the side-input epilogues exist on the MFMA path only
    if ((unsigned)((M + 63) / 64) > 65535u) return ROV_ERR_UNSUPPORTED;
    return ROV_OK;
}

int launch_gemm_epilogue(const void* A, const void* Bm, void* C, const void* R, int epi, int M, int N, int K,
                         int dtype, int transB, float scaleA, float scaleB, hipStream_t stream) {
    {
        const int rc = check_gemm(A, Bm, C, R, epi, M, N, K, dtype, transB);
        if (rc != ROV_OK) return rc;
    }
    const float alpha = scaleA * scaleB;
    const bool tb = transB != 0;
    const int esz = dtype == ROV_BF16 ? 2 : 1;

    if (dtype != ROV_F32 && tb && ((size_t)K * esz) % kRowBytes == 0 && (N % 4) == 0) {
        // a 256-row operand panel is addressed with 32-bit byte offsets
        if ((unsigned long long)BM * (unsigned long long)K * (unsigned long long)esz > 0xFFFFFFFFull)
            return ROV_ERR_UNSUPPORTED;
        const int tiles_m = (M + BM - 1) / BM;
        const int nj = pick_tile_cols(M, N) / 32;
        const int tiles_n = (N + 32 * nj - 1) / (32 * nj);
        const long long T = (long long)tiles_m * tiles_n;
        if (T > 0x7FFFFFFFLL) return ROV_ERR_UNSUPPORTED;
        typedef void (*kern_t)(const char*, const char*, uint16_t*, const uint16_t*, int, int, int, float, int, int, int);
        static const kern_t kerns[10] = {gemm_tn_kernel<4>,       gemm_tn_kernel<5>,       gemm_tn_kernel<6>,
                                         gemm_tn_kernel<7>,       gemm_tn_kernel<8>,       gemm_tn_kernel<4, true>,
                                         gemm_tn_kernel<5, true>, gemm_tn_kernel<6, true>, gemm_tn_kernel<7, true>,
                                         gemm_tn_kernel<8, true>};
        const int ki = nj - 4 + (esz == 2 ? 0 : 5);
        const kern_t kern = kerns[ki];
        {
            const int rc = set_max_dynamic_lds((const void*)kern, kLdsBytes);
            if (rc != ROV_OK) return rc;
        }
        hipLaunchKernelGGL(kern, dim3((unsigned)T), dim3(256), kLdsBytes, stream, (const char*)A,
                           (const char*)Bm, (uint16_t*)C, (const uint16_t*)R, M, N, K, alpha, tiles_m,
                           tiles_n, epi);
        ROV_LAUNCH_CHECK();
        return ROV_OK;
    }

    if (R != nullptr) return ROV_ERR_UNSUPPORTED;   // the side-input epilogues exist on the MFMA path only
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

extern "C" int rov_gemm_tile_cols(int M, int N) {
    if (M <= 0 || N <= 0) return ROV_ERR_INVALID;
    return rov::pick_tile_cols(M, N);
}

extern "C" int rov_set_gemm_tile_cols(int cols) {
    if (cols != 0 && (cols < 128 || cols > 256 || cols % 32 != 0)) return ROV_ERR_INVALID;
    return rov::g_tile_cols.exchange(cols);
}

extern "C" int rov_gemm(const void* A, const void* Bm, void* C, int M, int N, int K, int dtype,
                        int transB, float scaleA, float scaleB, void* stream) {
    return rov::launch_gemm(A, Bm, C, M, N, K, dtype, transB, scaleA, scaleB, (hipStream_t)stream);
}

// Flash-attention forward with dropout after softmax (paper Sec. 2.2, Sec. 6.1).
//
// Three ways to get the keep bits, all giving the same bits:
//   MODE_NONE  p == 0, no dropout;
//   MODE_MASK  the paper's "attention with element dropping": keep-mask words written
//              earlier by the stand-alone RNG kernel; a word is the 64 lanes' keep bits for
//              one accumulator register, fetched with scalar loads and applied with one
//              select per element;
//   MODE_FUSED the paper's fusion baseline: every lane runs Philox for its own elements.
//
// bf16 kernel, head dimension 64 or 128, on the matrix cores.  Everything is
// computed transposed, S^T = K Q^T and O^T = V^T P^T with MFMA 32x32x16, because
// then one lane owns one query column: the softmax statistics, the rescale of
// O and the mask word are per-lane scalars and only the row maximum needs one
// exchange between the two half-waves.  The S^T accumulator registers are, as
// they stand, the P^T operand of the second product if the 16 keys of a k-step
// are taken in the order the accumulator holds them; the matching V^T operand
// comes out of the row-major V tile with the gfx950 transpose load
// (ds_read_b64_tr_b16), two per fragment, so V is never copied transposed.
//
// A wave owns 32 query rows and walks the keys 64 at a time; the 8 waves of a
// workgroup (two per SIMD: while one waits for LDS or the matrix pipe the other
// issues) share each K / V tile through LDS, filled straight from global memory
// with buffer loads that write LDS (two stages, the next tile in flight while
// the current one is used).
//
// Any other case (fp32, other head dimensions) takes a small one-wave-per-row
// kernel that is correct for every shape.
#include <hip/hip_runtime.h>

#include <type_traits>
#include <stdint.h>

#include "fp8_device.h"
#include "philox_device.h"
#include "rov_internal.h"

namespace rov {
namespace {

enum { MODE_NONE = 0, MODE_MASK = 1, MODE_FUSED = 2 };

struct AttnParams {
    const void* Q;
    const void* K;
    const void* V;
    void* O;
    const uint64_t* mask;
    int64_t sq[3], sk[3], sv[3], so[3];   // element strides (batch, token, head)
    int B, H, Hkv, S, d;
    int W;                                // mask tiles per side, ceil(S/32)
    int nq;                               // query blocks per (batch, head)
    int q_begin, q_end;                   // query rows computed by this launch: [q_begin, q_end)
    int mask_qt0, mask_nqt;               // tile rows the mask buffer holds: [mask_qt0, mask_qt0 + mask_nqt)
    int causal;
    float scale_log2;                     // log2(e) / sqrt(d)
    float inv_keep;                       // 1 / (1 - p)
    uint64_t offset;                      // Philox call offset (fused)
    uint32_t k0, k1;                      // Philox key (fused)
    uint32_t t_minus_1;                   // keep iff x <= t_minus_1 (fused)
    int rounds;                           // Philox rounds (fused)
    int bits;                             // random bits per element (fused): 8, 16 or 32
    uint32_t tb;                          // bits < 32: keep iff field < tb (fused)
    int o_fp8;                            // O is written as OCP e4m3 bytes of (value * o_inv_scale): fp8 block
    float o_inv_scale;
};

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void* lptr_t;

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    f32x2 v = {lo, hi};
    bf16x2 h = __builtin_convertvector(v, bf16x2);
    return *reinterpret_cast<uint32_t*>(&h);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// max(v[lane], v[lane ^ 32]) in every lane.  v_permlane32_swap exchanges the upper 32 lanes of its
// first operand with the lower 32 of its second: with both operands v, one result holds the lower
// half-wave's values in both halves and the other the upper half-wave's.
__device__ __forceinline__ float half_wave_max(float v) {
    const uint32_t u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_wave_sum(float v) {
    const uint32_t u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

constexpr int BKV = 64;   // keys per tile = one mask word per query row

template <int D>
struct Tile {
    static constexpr int kKRow = D * 2;                // bytes per K row in LDS
    static constexpr int kKBytes = BKV * kKRow;
    static constexpr int kStage = 2 * kKBytes;         // K tile then V tile, both [key][feature]
    static constexpr int kChunks = D / 8;              // 16-byte chunks per K row
};

// Swizzle of the 16-byte chunks of an LDS tile row (XORed into the chunk index), chosen for the
// way gfx950 serves LDS reads over its 64 banks of 4 bytes (lane sets measured with a two-lane
// probe and the bank-conflict counter):
//  * ds_read_b128 goes 16 lanes at a time, in the sets {0-3, 12-15, 20-27}, {4-11, 16-19, 28-31}
//    and the same + 32.  A K fragment read has lane = row (mod 32), chunk fixed, so a set holds
//    16 rows that need 16 (D = 128: row = 256 bytes) or, per row parity, 8 (D = 64) different
//    swizzle values: the position of the row within its set.
//  * ds_read_b64 (and its transposing form) goes 32 lanes at a time.  A V transpose read has, per
//    half-wave, 4 consecutive rows x 4 adjacent chunks x 2 halves; all rows alias (256-byte
//    rows) or alias by parity (128-byte rows), so the rows' groups of 4 chunks must differ.
template <int D, bool VTILE>
__device__ __forceinline__ int swizzle_of_row(int row) {
    if (VTILE) return D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2);
    return D == 128 ? ((((row >> 3) & 3) << 2) | (row & 3)) : ((((row >> 3) & 3) << 1) | ((row >> 1) & 1));
}

// K or V tile: global -> LDS directly.  One wave instruction fills 1 KiB = 1024 / kKRow rows;
// lane L lands on physical chunk L % kChunks of its row and therefore fetches the logical
// chunk (L % kChunks) ^ swizzle(row).  The loads are buffer loads: a buffer resource over the
// rows [0, S) of this (batch, kv head) as scalar base, the lane's byte offset from the tile's
// first row (the same for every tile, computed once) as vector offset, and the tile's first
// row as scalar offset -- no per-lane address arithmetic in the loop.  Rows at or beyond S lie
// outside the resource's range and read as zeros (their scores are masked anyway).
// Inline assembly on purpose: the compiler's wait-count pass cannot tell the LDS write of such
// a load from the fragment reads of the other stage and would force vmcnt(0) before the
// second product of every tile, i.e. wait for the prefetch in the middle of the tile it was
// meant to run under; the kernel places its one vmcnt(0) per tile itself.  M0 (the LDS base of
// the transfer) is a reserved register that compiled code only sets right before its own uses.
typedef int i32x4 __attribute__((ext_vector_type(4)));
template <int D, int NW, bool VTILE>
struct KvTileLoad {
    static constexpr int kChunks = Tile<D>::kChunks;
    static constexpr int kRowsPerInst = 64 / kChunks;          // 4 (D = 128) or 8 (D = 64)
    static constexpr int kInst = BKV / kRowsPerInst;           // 16 or 8 per tile
    static constexpr int kPerWave = kInst / NW;
    uint32_t off[kPerWave];
    uint32_t row_bytes;
    i32x4 rsrc;

    __device__ __forceinline__ void init(const uint16_t* Xp, int64_t tok_stride, int S, int wave, int lane) {
        const int rl = lane / kChunks, pc = lane % kChunks;
        row_bytes = (uint32_t)tok_stride * 2u;
#pragma unroll
        for (int i = 0; i < kPerWave; ++i) {
            const int row = (wave + NW * i) * kRowsPerInst + rl;          // 0..63
            const int chunk = pc ^ swizzle_of_row<D, VTILE>(row);
            off[i] = (uint32_t)row * row_bytes + (uint32_t)chunk * 16u;
        }
        const uint64_t base = (uint64_t)(uintptr_t)Xp;
        rsrc[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)base);
        rsrc[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)((base >> 32) & 0xFFFFu));
        rsrc[2] = __builtin_amdgcn_readfirstlane((int)((uint32_t)(S - 1) * row_bytes + (uint32_t)(D * 2)));
        rsrc[3] = 0x00020000;
    }

    // lds_tile: LDS byte address of the tile
    __device__ __forceinline__ void load(int kv0, uint32_t lds_tile, int wave) const {
        const uint32_t soff = (uint32_t)kv0 * row_bytes;
#pragma unroll
        for (int i = 0; i < kPerWave; ++i) {
            const uint32_t dst = lds_tile + (uint32_t)((wave + NW * i) * 1024);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                         :: "s"(dst), "v"(off[i]), "s"(rsrc), "s"(soff) : "memory");
        }
    }
};

typedef const __attribute__((address_space(4))) uint64_t* const_u64_ptr;
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) i16x4* lds_i16x4_ptr;

// ds_read_b64_tr_b16: within each group of 16 lanes, source lane r = 4*j + s supplies the
// address of 4 consecutive 16-bit elements, and lane i of the group receives element i%4 of
// the rows supplied by source lanes 4*j + i/4, j = 0..3.  If the four source lanes 4*j + s
// (s = 0..3) point at row key_j, columns c0 + 4*s .. +3, then lane i ends up with column
// c0 + i of rows key_0 .. key_3: a column fragment of a row-major tile, i.e. the transposed
// operand the second product needs, with no transposed copy of V anywhere.
__device__ __forceinline__ bf16x4 lds_read_transposed(const char* p) {
    const i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)p);
    return __builtin_bit_cast(bf16x4, v);
}

// NW waves per workgroup, each owning NQ*32 query rows.  (NQ, NW) = (2, 4) keeps one wave per
// SIMD with K/V fragments reused for two query tiles; (1, 8) puts two waves on every SIMD so
// that one wave's softmax VALU work runs under the other's MFMAs.
template <int D, int NQ, int NW, int MODE, int R = 10, int BITS = 32>
__global__ __launch_bounds__(NW * 64) void attn_bf16_kernel(const AttnParams p) {
    constexpr int BQ = NW * 32 * NQ;   // query rows per workgroup
    using T = Tile<D>;
    constexpr int KS = D / 16;    // k-steps of the first product
    constexpr int DVT = D / 32;   // dv tiles of the second product
    extern __shared__ __attribute__((aligned(1024))) char lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ql = lane & 31;     // query column within a 32-wide tile
    const int half = lane >> 5;
    const int S = p.S;
    // Workgroup ids are dealt round-robin to the 8 XCDs.  All query blocks of one (batch, head)
    // go to the same XCD, so its K and V are fetched into one L2 only; within an XCD the order
    // is query block first, then head, so co-resident workgroups walk the same K/V in step.
    int qblk, bh;
    {
        const int pid = blockIdx.x, G = p.B * p.H, nq = p.nq;
        if ((G & 7) == 0) {
            const int xcd = pid & 7, j = pid >> 3, gpx = G >> 3;
            qblk = j / gpx;
            bh = (j % gpx) * 8 + xcd;
        } else {
            qblk = pid / G;
            bh = pid % G;
        }
        if (p.causal) qblk = nq - 1 - qblk;   // heaviest query blocks first
    }
    const int b = bh / p.H, h = bh % p.H;
    const int hk = h / (p.H / p.Hkv);
    const int q0 = p.q_begin + qblk * BQ + wave * (32 * NQ);
    const int q_end = p.q_end;

    const uint16_t* Qp = (const uint16_t*)p.Q + b * p.sq[0] + h * p.sq[2];
    const uint16_t* Kp = (const uint16_t*)p.K + b * p.sk[0] + hk * p.sk[2];
    const uint16_t* Vp = (const uint16_t*)p.V + b * p.sv[0] + hk * p.sv[2];
    uint16_t* Op = (uint16_t*)p.O + b * p.so[0] + h * p.so[2];

    // Q fragments (second operand of K Q^T): lane holds query ql, features 16*ks + 8*half .. +7
    bf16x8 qf[NQ][KS];
    int qrow[NQ];
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
        int q = q0 + 32 * n + ql;
        qrow[n] = q;
        q = q < q_end ? q : q_end - 1;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qf[n][ks] = *reinterpret_cast<const bf16x8*>(Qp + (int64_t)q * p.sq[1] + 16 * ks + 8 * half);
    }

    f32x16 o[DVT][NQ];
#pragma unroll
    for (int t = 0; t < DVT; ++t)
#pragma unroll
        for (int n = 0; n < NQ; ++n)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[t][n][e] = 0.0f;
    float m_run[NQ], l_run[NQ];
#pragma unroll
    for (int n = 0; n < NQ; ++n) { m_run[n] = -INFINITY; l_run[n] = 0.0f; }

    // number of KV tiles this workgroup walks (causal: up to its last query row)
    const int q_last = min(p.q_begin + qblk * BQ + BQ, q_end) - 1;
    const int kv_end = p.causal ? min(S, q_last + 1) : S;
    const int ntiles = (kv_end + BKV - 1) / BKV;

    // Keep words.  The mask is stored as 32 x 32 tiles of 16 words in accumulator order (see
    // rov.h): word e of tile (qt, kt) holds, in bit l, the keep bit of the element that lane l
    // has in accumulator register e of S^T tile (keys 32*kt.., queries 32*qt..).  The wave's
    // query tile is fixed, so its words for a KV tile are 2 x 16 consecutive, wave-uniform words:
    // MODE_MASK fetches them with scalar loads and applies each with one select; MODE_FUSED
    // needs no words at all, every lane draws the Philox outputs of its own elements.
    const uint32_t Tt = (uint32_t)p.W;                                    // tiles per side
    const uint64_t bh_tiles = ((uint64_t)b * p.H + h) * Tt;
    const uint64_t* mtile[NQ];      // words of tile (qt, 0) for each of the wave's query tiles
    uint64_t wtile[NQ];             // index of that word in the whole mask (fused: Philox numbering)
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
        uint32_t qt = (uint32_t)(q0 / 32 + n);
        const uint32_t qt_last = (uint32_t)(p.mask_qt0 + p.mask_nqt - 1);
        qt = qt < qt_last ? qt : qt_last;                                 // rows past q_end are never stored
        wtile[n] = ((bh_tiles + qt) * Tt) * 16u;
        // the buffer holds mask_nqt tile rows per (batch, head), starting at tile row mask_qt0
        mtile[n] = p.mask + ((((uint64_t)b * p.H + h) * (uint32_t)p.mask_nqt + (qt - (uint32_t)p.mask_qt0)) * Tt) * 16u;
    }

    KvTileLoad<D, NW, false> kload;
    KvTileLoad<D, NW, true> vload;
    kload.init(Kp, p.sk[1], S, wave, lane);
    vload.init(Vp, p.sv[1], S, wave, lane);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lptr_t)lds;
    kload.load(0, lds_base, wave);
    vload.load(0, lds_base + T::kKBytes, wave);

    // transpose-load addressing of the V tile (see lds_read_transposed): lane l = 16*g + 4*j + s
    // supplies row 16*u + 8*x + 4*(g/2) + j, columns 32*t + 16*(g%2) + 4*s .. +3
    int vt_off[DVT];
    {
        const int g = lane >> 4, j = (lane >> 2) & 3, sl = lane & 3, hh = g >> 1;
        const int row_part = (4 * hh + j) * T::kKRow + (sl & 1) * 8;
        const int f = swizzle_of_row<D, true>(4 * hh + j);      // the row is 16u + 8x + 4hh + j: same value
#pragma unroll
        for (int t = 0; t < DVT; ++t)
            vt_off[t] = row_part + (((4 * t + 2 * (g & 1) + (sl >> 1)) ^ f) << 4);
    }

    const int kswz = swizzle_of_row<D, false>(ql);   // K fragment rows are 32t + ql: same value
    static_assert(NQ == 1, "the keep-word warm-up load covers one query tile per wave");
    uint32_t warm = 0u, sink = 0u;   // L2 warm-up of the next tile's keep words (MODE_MASK)

    // One KV tile.  The LDS stage is a compile-time constant (the loop below alternates the two
    // instantiations), so every fragment read is a loop-invariant lane address plus an immediate.
    auto tile_step = [&](const int jt, auto stage_tag) __attribute__((always_inline)) {
        constexpr int STAGE = decltype(stage_tag)::value;
        const int kv0 = jt * BKV;
        char* cur = lds + STAGE * T::kStage;
        __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0): this wave's K / V loads have landed
        __syncthreads();
        const bool has_next = jt + 1 < ntiles;
        if (has_next) {
            kload.load(kv0 + BKV, lds_base + (STAGE ^ 1) * T::kStage, wave);
            vload.load(kv0 + BKV, lds_base + (STAGE ^ 1) * T::kStage + T::kKBytes, wave);
        }
        // ---- S^T = K Q^T for 64 keys x NQ*32 queries
        f32x16 s[2][NQ];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int n = 0; n < NQ; ++n)
#pragma unroll
                for (int e = 0; e < 16; ++e) s[t][n][e] = 0.0f;
        // K fragments are read kAhead k-steps before the MFMAs that use them: the scheduling
        // groups below pin that order (3 k-steps of reads, then per k-step its MFMAs followed by
        // the reads of the k-step kAhead further on), so the LDS latency is paid once per tile
        // and not once per k-step.
        constexpr int kAhead = 3;
        bf16x8 kf[KS][2];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int t = 0; t < 2; ++t)
                kf[ks][t] = *reinterpret_cast<const bf16x8*>(
                    cur + (32 * t + ql) * T::kKRow + (((2 * ks + half) ^ kswz) << 4));
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int n = 0; n < NQ; ++n)
                    s[t][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks][t], qf[n][ks], s[t][n], 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * kAhead, 0);          // DS reads
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            __builtin_amdgcn_sched_group_barrier(0x008, 2 * NQ, 0);          // MFMAs of k-step ks
            if (ks + kAhead < KS) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
        // nothing below moves up into the first product: a scalar load of keep words between its
        // LDS reads would turn every wait for a fragment into a wait for that load as well (the
        // two share one counter, and scalar loads return out of order)
        __builtin_amdgcn_sched_barrier(0);

        // ---- keep words of this KV tile: 2 key tiles x 16 words per query tile, wave-uniform.
        // They are requested here, right after the Q K^T MFMAs have been issued, through the
        // constant address space (memory nobody writes while this kernel runs), i.e. with
        // scalar loads into the SGPR pairs that the selects below use as lane predicates.  The
        // lines were pulled into L2 one tile earlier by `warm` (a vector load whose value is
        // only folded into a sink), so the scalar loads return while the row maxima and
        // exponentials are being computed.
        uint64_t mw[NQ][2][16];
        if (MODE == MODE_MASK) {
#pragma unroll
            for (int n = 0; n < NQ; ++n)
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    uint32_t kt = (uint32_t)(2 * jt + t);
                    kt = kt < Tt ? kt : Tt - 1;
                    const const_u64_ptr wp = (const_u64_ptr)(uintptr_t)(mtile[n] + (uint64_t)kt * 16u);
#pragma unroll
                    for (int e = 0; e < 16; ++e) mw[n][t][e] = wp[e];
                }
            sink ^= warm;                       // the previous warm-up load has long landed
            // 64 lanes x 4 bytes = the 32 words of the next two key tiles (16 words if the tile
            // row has a single tile); clamped so that it never leaves this query tile's row
            uint32_t ktn = (uint32_t)(2 * jt + 2);
            ktn = ktn + 1 < Tt ? ktn : (Tt >= 2 ? Tt - 2 : 0);
            warm = reinterpret_cast<const uint32_t*>(mtile[0] + (uint64_t)ktn * 16u)[lane & (Tt >= 2 ? 63 : 31)];
        }

        // ---- online softmax, dropout, P^T fragments
        bf16x8 pf[NQ][4];
        const bool tail = kv0 + BKV > S;
        const bool diag = p.causal && (kv0 + BKV - 1 > q0);   // some key of the tile may exceed a query
#pragma unroll
        for (int n = 0; n < NQ; ++n) {
            // the maximum is taken on the raw scores (the scale is positive) and the scale is folded
            // into the exponent's multiply-add below: one VALU op less per element
            float mx = -INFINITY;
            if (tail || diag) {   // wave-uniform: only the tiles on the diagonal and the last one
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int key = kv0 + 32 * t + 8 * (e >> 2) + 4 * half + (e & 3);
                        const bool ok = key < S && (!p.causal || key <= qrow[n]);
                        s[t][n][e] = ok ? s[t][n][e] : -INFINITY;
                    }
            }
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[t][n][e]);
            // the other half-wave's maximum of the same query: a lane swap in the VALU (gfx950
            // v_permlane32_swap), not an LDS permute: the LDS counter is shared with the scalar
            // keep-word loads in flight, so waiting for a permute here would wait for them too
            mx = half_wave_max(mx) * p.scale_log2;
            // The reference of the exponent follows the maximum lazily: it moves only when the
            // tile's maximum exceeds it by more than kLazy (in log2 units), so entries reach at
            // most 2^kLazy, far inside fp32 and bf16 range, the quotient by the row sum is the
            // same softmax, and the rescale of the output accumulators below runs in the first
            // tile and hardly ever again (with the exact maximum about a third of all tiles of a
            // 16k sequence move some row's maximum).
            constexpr float kLazy = 8.0f;
            const float m_new = mx > m_run[n] + kLazy ? mx : m_run[n];
            const float m_safe = m_new == -INFINITY ? 0.0f : m_new;
            const float alpha = fast_exp2(m_run[n] - m_safe);
            m_run[n] = m_new;
            float sum = 0.0f;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                uint32_t kt = (uint32_t)(2 * jt + t);
                kt = kt < Tt ? kt : Tt - 1;        // a key tile past S: its scores are -inf already
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float pe = fast_exp2(__builtin_fmaf(s[t][n][e], p.scale_log2, -m_safe));
                    sum += pe;   // the normaliser counts dropped entries too
                    s[t][n][e] = pe;
                }
                if (MODE == MODE_MASK) {
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        s[t][n][e] = __builtin_amdgcn_inverse_ballot_w64(mw[n][t][e]) ? s[t][n][e] : 0.0f;
                }
                if (MODE == MODE_FUSED) {
                    // Words are taken in groups of E = 4 * 32 / BITS; word e = E*c + 4*f + r of this tile is
                    // decided by field f of output r of the lane's Philox call offset + 64*(first_word/E + c) + lane
                    // (BITS = 32: one field, the whole word)
                    constexpr int NF = 32 / BITS, E = 4 * NF;
                    const uint64_t g0 = (wtile[n] + (uint64_t)kt * 16u) / (uint32_t)E;
#pragma unroll
                    for (int c = 0; c < 16 / E; ++c) {
                        const uint64_t base = p.offset + 64u * (g0 + (uint64_t)c);
                        const uint32_t blo = (uint32_t)base, bhi = (uint32_t)(base >> 32);
                        const uint32_t c0 = blo + (uint32_t)lane;
                        uint32_t x[4];
                        if (blo <= 0xFFFFFFFFu - 63u) {
                            philox4x32_low_counter<R>(c0, bhi, p.k0, p.k1, x);
                        } else {
                            philox4x32<R>(c0, bhi + (c0 < blo ? 1u : 0u), 0u, 0u, p.k0, p.k1, x);
                        }
#pragma unroll
                        for (int f = 0; f < NF; ++f)
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const int e = E * c + 4 * f + r;
                                bool keep;
                                if (BITS == 32) keep = x[r] <= p.t_minus_1;
                                else keep = ((x[r] >> (BITS * f)) & ((1u << (BITS & 31)) - 1u)) < p.tb;
                                s[t][n][e] = keep ? s[t][n][e] : 0.0f;
                            }
                    }
                }
            }
            l_run[n] = l_run[n] * alpha + sum;
            // the running maximum settles after the first tiles; the rescale of the 64 output
            // accumulators is skipped while no lane of the wave has a new maximum (alpha == 1)
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0ull) {
#pragma unroll
                for (int t = 0; t < DVT; ++t)
#pragma unroll
                    for (int e = 0; e < 16; ++e) o[t][n][e] *= alpha;
            }
            // k-step u = 2*t + v of the second product takes registers 8*v .. 8*v+7 of tile t
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int t = u >> 1, v8 = (u & 1) * 8;
                uint32_t w[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = pack_bf16x2(s[t][n][v8 + 2 * e], s[t][n][v8 + 2 * e + 1]);
                pf[n][u] = *reinterpret_cast<bf16x8*>(w);
            }
        }

        // ---- O^T += V^T P^T
        const char* vt = cur + T::kKBytes;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int t = 0; t < DVT; ++t) {
                // keys 16u + 4*half + 0..3 and 16u + 8 + 4*half + 0..3 of feature 32t + lane%32
                const bf16x4 lo = lds_read_transposed(vt + (16 * u) * T::kKRow + vt_off[t]);
                const bf16x4 hi = lds_read_transposed(vt + (16 * u + 8) * T::kKRow + vt_off[t]);
                const bf16x8 vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int n = 0; n < NQ; ++n)
                    o[t][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[n][u], o[t][n], 0, 0, 0);
            }
        }
    };
    for (int jt = 0; jt < ntiles; jt += 2) {
        tile_step(jt, std::integral_constant<int, 0>{});
        if (jt + 1 < ntiles) tile_step(jt + 1, std::integral_constant<int, 1>{});
    }

    // the warm-up values only have to look used (no mask pattern makes this condition true
    // for a lane id >= 64)
    if (MODE == MODE_MASK && (sink ^ warm) == 0x9E3779B9u && lane == 1000) m_run[0] = 0.0f;

    // ---- normalise, scale kept entries by 1/(1-p), store O (lane: query ql, 4 consecutive dv per e/4)
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
        const float l = half_wave_sum(l_run[n]);
        const float f = l > 0.0f ? p.inv_keep / l : 0.0f;
        if (qrow[n] < q_end && p.o_fp8) {
            // the fp8 block quantises the attention output where it is produced (strides count bytes here)
            uint8_t* orow = (uint8_t*)p.O + b * p.so[0] + h * p.so[2] + (int64_t)qrow[n] * p.so[1];
            const float fq = f * p.o_inv_scale;
#pragma unroll
            for (int t = 0; t < DVT; ++t)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *reinterpret_cast<uint32_t*>(orow + 32 * t + 8 * g + 4 * half) =
                        pack_e4m3x4(o[t][n][4 * g + 0] * fq, o[t][n][4 * g + 1] * fq, o[t][n][4 * g + 2] * fq,
                                    o[t][n][4 * g + 3] * fq);
        } else if (qrow[n] < q_end) {
            uint16_t* orow = Op + (int64_t)qrow[n] * p.so[1];
#pragma unroll
            for (int t = 0; t < DVT; ++t)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    uint2 v;
                    v.x = pack_bf16x2(o[t][n][4 * g + 0] * f, o[t][n][4 * g + 1] * f);
                    v.y = pack_bf16x2(o[t][n][4 * g + 2] * f, o[t][n][4 * g + 3] * f);
                    *reinterpret_cast<uint2*>(orow + 32 * t + 8 * g + 4 * half) = v;
                }
        }
    }
}

// ------------------------------------------------------------------ generic kernel
// One wave per query row, keys in chunks of 256 with an online softmax; any dtype / head
// dimension up to 256.  Correct for every shape; used for fp32 and odd head dimensions.
template <typename TT>
__device__ __forceinline__ float ld(const TT* p);
template <>
__device__ __forceinline__ float ld<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float ld<uint16_t>(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }
template <typename TT>
__device__ __forceinline__ void st(TT* p, float v);
template <>
__device__ __forceinline__ void st<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void st<uint16_t>(uint16_t* p, float v) {
    *p = (uint16_t)(pack_bf16x2(v, 0.0f) & 0xFFFFu);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) v = fmaxf(v, __shfl_xor(v, s));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) v += __shfl_xor(v, s);
    return v;
}

template <typename TT, int MODE>
__global__ __launch_bounds__(256) void attn_generic_kernel(const AttnParams p) {
    __shared__ float qs[4][256];
    __shared__ float ps[4][256];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = p.q_begin + blockIdx.x * 4 + wave;
    const int b = blockIdx.z, h = blockIdx.y;
    const int hk = h / (p.H / p.Hkv);
    const int S = p.S, d = p.d;
    if (row >= p.q_end) return;   // whole wave leaves; no block-wide barrier below
    const TT* Qp = (const TT*)p.Q + b * p.sq[0] + h * p.sq[2] + (int64_t)row * p.sq[1];
    const TT* Kp = (const TT*)p.K + b * p.sk[0] + hk * p.sk[2];
    const TT* Vp = (const TT*)p.V + b * p.sv[0] + hk * p.sv[2];
    TT* Op = (TT*)p.O + b * p.so[0] + h * p.so[2] + (int64_t)row * p.so[1];
    for (int t = lane; t < d; t += 64) qs[wave][t] = ld(Qp + t);
    __builtin_amdgcn_wave_barrier();
    float acc[4] = {0.f, 0.f, 0.f, 0.f};   // output features lane, lane+64, lane+128, lane+192
    float m_run = -INFINITY, l_run = 0.0f;
    const int kv_end = p.causal ? row + 1 : S;
    // tile row of this query row in the mask: words of tile (row/32, kt) start at wrow + 16*kt;
    // element (row, key) is bit 32*((key%32)/4 % 2) + row%32 of word 4*((key%32)/8) + key%4
    const uint64_t wrow = ((((uint64_t)b * p.H + h) * p.W + (uint64_t)(row >> 5)) * p.W) * 16u;
    // same tile row inside the mask buffer, which holds tile rows [mask_qt0, mask_qt0 + mask_nqt)
    const uint64_t mrow = ((((uint64_t)b * p.H + h) * p.mask_nqt + (uint64_t)((row >> 5) - p.mask_qt0)) * p.W) * 16u;
    for (int c0 = 0; c0 < kv_end; c0 += 256) {
        float sc[4];
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int key = c0 + lane + 64 * i;
            float v = -INFINITY;
            if (key < kv_end) {
                const TT* kr = Kp + (int64_t)key * p.sk[1];
                float dot = 0.0f;
                for (int t = 0; t < d; ++t) dot = __builtin_fmaf(qs[wave][t], ld(kr + t), dot);
                v = dot * p.scale_log2;
            }
            sc[i] = v;
            mx = fmaxf(mx, v);
        }
        mx = wave_max(mx);
        const float m_new = fmaxf(m_run, mx);
        const float alpha = fast_exp2(m_run - m_new);   // chunk 0 always has an admissible key
        m_run = m_new;
        float sum = 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int key = c0 + lane + 64 * i;
            float pe = 0.0f;
            if (key < kv_end) {
                pe = fast_exp2(sc[i] - m_new);
                sum += pe;
                bool keep = true;
                const int kl = key & 31;
                const uint64_t wo = (uint64_t)(key >> 5) * 16u + (uint64_t)(4 * (kl >> 3) + (kl & 3));
                const uint64_t w = wrow + wo;
                const uint32_t bit = 32u * ((uint32_t)(kl >> 2) & 1u) + ((uint32_t)row & 31u);
                if (MODE == MODE_MASK) {
                    keep = (p.mask[mrow + wo] >> bit) & 1ull;
                } else if (MODE == MODE_FUSED) {
                    const uint32_t E = 128u / (uint32_t)p.bits;            // mask words per group of calls
                    const uint64_t ncall = p.offset + 64u * (w / E) + (uint64_t)bit;
                    uint32_t x[4];
                    philox4x32_dyn(p.rounds, (uint32_t)ncall, (uint32_t)(ncall >> 32), 0u, 0u, p.k0, p.k1, x);
                    const uint32_t k = (uint32_t)(w % E), sel = k & 3u, f = k >> 2;
                    const uint32_t xv = sel == 0 ? x[0] : sel == 1 ? x[1] : sel == 2 ? x[2] : x[3];
                    if (p.bits == 32) keep = xv <= p.t_minus_1;
                    else keep = ((xv >> ((uint32_t)p.bits * f)) & ((1u << p.bits) - 1u)) < p.tb;
                }
                pe = keep ? pe : 0.0f;
            }
            ps[wave][lane + 64 * i] = pe;
        }
        l_run = l_run * alpha + wave_sum(sum);
        __builtin_amdgcn_wave_barrier();
        const int nkeys = min(256, kv_end - c0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = lane + 64 * j;
            if (t < d) {
                float a = acc[j] * alpha;
                for (int kk = 0; kk < nkeys; ++kk)
                    a = __builtin_fmaf(ps[wave][kk], ld(Vp + (int64_t)(c0 + kk) * p.sv[1] + t), a);
                acc[j] = a;
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    const float f = l_run > 0.0f ? p.inv_keep / l_run : 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int t = lane + 64 * j;
        if (t < d) st(Op + t, acc[j] * f);
    }
}

template <int D, int NQ, int NW>
int launch_bf16(const AttnParams& prm, int mode, hipStream_t stream) {
    const int bq = NW * 32 * NQ;
    AttnParams prm2 = prm;
    prm2.nq = (prm.q_end - prm.q_begin + bq - 1) / bq;
    const long long nblocks = (long long)prm2.nq * prm.H * prm.B;
    if (nblocks > 0x7FFFFFFFLL) return ROV_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)nblocks), block(NW * 64);
    const int lds_bytes = 2 * Tile<D>::kStage;   // two K/V stages
    void (*kern)(const AttnParams) = mode == MODE_NONE ? attn_bf16_kernel<D, NQ, NW, MODE_NONE>
                                                       : attn_bf16_kernel<D, NQ, NW, MODE_MASK>;
    if (mode == MODE_FUSED) {   // the round count is a compile-time constant of the fused kernel
        if (prm.bits == 16) { if (prm.rounds != 10) return ROV_ERR_UNSUPPORTED; kern = attn_bf16_kernel<D, NQ, NW, MODE_FUSED, 10, 16>; }
        else if (prm.bits == 8) { if (prm.rounds != 10) return ROV_ERR_UNSUPPORTED; kern = attn_bf16_kernel<D, NQ, NW, MODE_FUSED, 10, 8>; }
        else switch (prm.rounds) {
            case 10: kern = attn_bf16_kernel<D, NQ, NW, MODE_FUSED, 10>; break;
            case 7: kern = attn_bf16_kernel<D, NQ, NW, MODE_FUSED, 7>; break;
            case 5: kern = attn_bf16_kernel<D, NQ, NW, MODE_FUSED, 5>; break;
            case 3: kern = attn_bf16_kernel<D, NQ, NW, MODE_FUSED, 3>; break;
            default: return ROV_ERR_INVALID;
        }
    }
    {
        const int rc = set_max_dynamic_lds((const void*)kern, lds_bytes);
        if (rc != ROV_OK) return rc;
    }
    hipLaunchKernelGGL(kern, grid, block, lds_bytes, stream, prm2);
    ROV_LAUNCH_CHECK();
    return ROV_OK;
}

template <typename TT>
int launch_generic(const AttnParams& prm, int mode, hipStream_t stream) {
    const dim3 grid((unsigned)((prm.q_end - prm.q_begin + 3) / 4), (unsigned)prm.H, (unsigned)prm.B), block(256);
    if (mode == MODE_NONE)
        hipLaunchKernelGGL((attn_generic_kernel<TT, MODE_NONE>), grid, block, 0, stream, prm);
    else if (mode == MODE_MASK)
        hipLaunchKernelGGL((attn_generic_kernel<TT, MODE_MASK>), grid, block, 0, stream, prm);
    else
        hipLaunchKernelGGL((attn_generic_kernel<TT, MODE_FUSED>), grid, block, 0, stream, prm);
    ROV_LAUNCH_CHECK();
    return ROV_OK;
}

}  // namespace

int launch_attention(const void* Q, const void* K, const void* V, void* O, int B, int H, int Hkv,
                     int S, int d, const int64_t strides[12], int dtype, int causal, float p,
                     const uint64_t* mask, uint64_t seed, uint64_t offset, hipStream_t stream, int rounds,
                     int bits) {
    return launch_attention_rows(Q, K, V, O, B, H, Hkv, S, d, strides, dtype, causal, p, mask, false, seed,
                                 offset, 0, S, stream, rounds, bits);
}

// Everything launch_attention_rows refuses, without launching: the schedules call this before
// they enqueue the first kernel of a sequence.
int check_attention_rows(const void* Q, const void* K, const void* V, const void* O, int B, int H, int Hkv,
                         int S, int d, const int64_t strides[12], int dtype, float p, const uint64_t* mask,
                         int q_begin, int q_rows, int rounds, int bits) {
    if (rounds != 10 && rounds != 7 && rounds != 5 && rounds != 3) return ROV_ERR_INVALID;
    if (bits != 32 && bits != 16 && bits != 8) return ROV_ERR_INVALID;
    if (bits != 32 && rounds != 10) return ROV_ERR_UNSUPPORTED;
    if (S <= 0 || q_begin < 0 || q_rows <= 0 || q_begin >= S || (q_begin & 31) != 0) return ROV_ERR_INVALID;
    if (Q == nullptr || K == nullptr || V == nullptr || O == nullptr || strides == nullptr)
        return ROV_ERR_INVALID;
    if (B <= 0 || H <= 0 || Hkv <= 0 || S <= 0 || d <= 0 || (H % Hkv) != 0) return ROV_ERR_INVALID;
    if (dtype != ROV_F32 && dtype != ROV_BF16) return dtype == ROV_FP8_E4M3 ? ROV_ERR_UNSUPPORTED : ROV_ERR_INVALID;
    uint32_t tm1 = 0xFFFFFFFFu;
    if (!keep_threshold_minus_1(p, &tm1)) return ROV_ERR_INVALID;
    if (B > 65535 || H > 65535) return ROV_ERR_UNSUPPORTED;
    if (d > 256) return ROV_ERR_UNSUPPORTED;
    if (mask != nullptr && !aligned(mask, 8)) return ROV_ERR_INVALID;
    // workgroups of the matrix-core kernel (256 query rows each) fit the grid's 31 bits
    const long long q_end = (long long)q_begin + q_rows < S ? (long long)q_begin + q_rows : S;
    if (((q_end - q_begin + 255) / 256) * (long long)H * B > 0x7FFFFFFFLL) return ROV_ERR_UNSUPPORTED;
    return ROV_OK;
}

int launch_attention_rows(const void* Q, const void* K, const void* V, void* O, int B, int H, int Hkv,
                          int S, int d, const int64_t strides[12], int dtype, int causal, float p,
                          const uint64_t* mask, bool mask_is_rows, uint64_t seed, uint64_t offset,
                          int q_begin, int q_rows, hipStream_t stream, int rounds, int bits, float o_fp8_scale) {
    {
        const int rc = check_attention_rows(Q, K, V, O, B, H, Hkv, S, d, strides, dtype, p, mask, q_begin, q_rows,
                                            rounds, bits);
        if (rc != ROV_OK) return rc;
    }
    uint32_t tm1 = 0xFFFFFFFFu;
    (void)keep_threshold_minus_1(p, &tm1);

    AttnParams prm;
    prm.Q = Q; prm.K = K; prm.V = V; prm.O = O; prm.mask = mask;
    for (int i = 0; i < 3; ++i) {
        prm.sq[i] = strides[i]; prm.sk[i] = strides[3 + i];
        prm.sv[i] = strides[6 + i]; prm.so[i] = strides[9 + i];
    }
    prm.B = B; prm.H = H; prm.Hkv = Hkv; prm.S = S; prm.d = d;
    prm.W = (S + 31) / 32;
    prm.q_begin = q_begin;
    prm.q_end = (int64_t)q_begin + q_rows < S ? q_begin + q_rows : S;
    // a mask of rows holds exactly the tile rows of [q_begin, q_end); a full mask holds all of them
    prm.mask_qt0 = mask_is_rows ? q_begin / 32 : 0;
    prm.mask_nqt = mask_is_rows ? (prm.q_end - q_begin + 31) / 32 : prm.W;
    prm.causal = causal != 0;
    prm.scale_log2 = 1.4426950408889634f / sqrtf((float)d);
    prm.inv_keep = p > 0.0f ? 1.0f / (1.0f - p) : 1.0f;
    prm.offset = offset;
    prm.k0 = (uint32_t)seed; prm.k1 = (uint32_t)(seed >> 32);
    prm.t_minus_1 = tm1;
    prm.rounds = rounds;
    prm.bits = bits;
    // keep iff field < tb, tb = floor((1 - p) * 2^bits) in double from the float p
    prm.tb = bits < 32 ? (uint32_t)(uint64_t)((1.0 - (double)p) * (double)(1u << bits)) : 0u;
    prm.o_fp8 = o_fp8_scale > 0.0f;
    prm.o_inv_scale = prm.o_fp8 ? 1.0f / o_fp8_scale : 1.0f;
    const int mode = p == 0.0f ? MODE_NONE : (mask != nullptr ? MODE_MASK : MODE_FUSED);

    if (dtype == ROV_BF16 && (d == 64 || d == 128)) {
        // 16-byte vector access needs 8-element alignment of every row start
        bool ok = aligned(Q, 16) && aligned(K, 16) && aligned(V, 16) && aligned(O, 8);
        for (int i = 0; i < 12; ++i) ok = ok && (strides[i] % 8) == 0;
        // K / V of one (batch, kv head) are addressed through a buffer resource: 32-bit byte offsets
        for (int t = 4; t <= 7; t += 3)
            ok = ok && strides[t] >= 0 && (uint64_t)(S - 1) * (uint64_t)strides[t] * 2u + 2u * (uint64_t)d < (1ull << 32);
        if (prm.o_fp8) {   // four bytes per store: O and its strides (in bytes) are multiples of 4
            ok = ok && aligned(O, 4);
            for (int i = 9; i < 12; ++i) ok = ok && (strides[i] % 4) == 0;
            if (!ok) return ROV_ERR_UNSUPPORTED;
        }
        if (ok) {
            // 8 waves x 32 query rows: two waves per SIMD (measured 1.5x faster than 4 waves x 64
            // rows at S = 16384: 905 vs 602 TFLOP/s without dropout)
            if (d == 128) return launch_bf16<128, 1, 8>(prm, mode, stream);
            return launch_bf16<64, 1, 8>(prm, mode, stream);
        }
    }
    if (prm.o_fp8) return ROV_ERR_UNSUPPORTED;   // the e4m3 output exists in the matrix-core kernel only
    if (dtype == ROV_BF16) return launch_generic<uint16_t>(prm, mode, stream);
    return launch_generic<float>(prm, mode, stream);
}

}  // namespace rov

extern "C" int rov_attention_fwd_dropout_rows(const void* Q, const void* K, const void* V, void* O, int B,
                                              int H, int Hkv, int S, int d, const int64_t strides[12],
                                              int dtype, int causal, float p, const uint64_t* mask_rows,
                                              uint64_t seed, uint64_t offset, int q_begin, int q_rows,
                                              void* stream) {
    return rov::launch_attention_rows(Q, K, V, O, B, H, Hkv, S, d, strides, dtype, causal, p, mask_rows, true,
                                      seed, offset, q_begin, q_rows, (hipStream_t)stream);
}

extern "C" int rov_attention_fwd_dropout(const void* Q, const void* K, const void* V, void* O, int B,
                                         int H, int Hkv, int S, int d, const int64_t strides[12],
                                         int dtype, int causal, float p, const uint64_t* mask,
                                         uint64_t seed, uint64_t offset, void* stream) {
    return rov::launch_attention(Q, K, V, O, B, H, Hkv, S, d, strides, dtype, causal, p, mask, seed,
                                 offset, (hipStream_t)stream);
}

extern "C" int rov_attention_fwd_dropout_rounds(const void* Q, const void* K, const void* V, void* O, int B,
                                                int H, int Hkv, int S, int d, const int64_t strides[12],
                                                int dtype, int causal, float p, const uint64_t* mask,
                                                uint64_t seed, uint64_t offset, int rounds, void* stream) {
    return rov::launch_attention(Q, K, V, O, B, H, Hkv, S, d, strides, dtype, causal, p, mask, seed,
                                 offset, (hipStream_t)stream, rounds);
}

extern "C" int rov_attention_fwd_dropout_bits(const void* Q, const void* K, const void* V, void* O, int B,
                                              int H, int Hkv, int S, int d, const int64_t strides[12],
                                              int dtype, int causal, float p, const uint64_t* mask,
                                              uint64_t seed, uint64_t offset, int bits, void* stream) {
    return rov::launch_attention(Q, K, V, O, B, H, Hkv, S, d, strides, dtype, causal, p, mask, seed,
                                 offset, (hipStream_t)stream, 10, bits);
}

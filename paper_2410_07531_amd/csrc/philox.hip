// Stand-alone RNG kernel: Philox-4x32 keep-mask written to HBM (paper Sec. 6.1,
// scenario 2 of the dropout kernel; storage B*nH*SQ^2 bits, Sec. 7.2), plus the
// raw-stream test hook.
//
// Shape of the work on gfx950: the kernel reads nothing and is bound by VALU
// issue (20 wide multiplies per call, Table 1 "ALU pipe"/"Issue stage").  One
// wave owns a chunk of 64 consecutive mask words = 16 groups of 4 words = 4
// tiles of 32 x 32 score elements.  For each group every lane makes one Philox
// call; the four compares of its output words are, as 64-lane ballots, exactly
// the four mask words of the group (a mask word is the 64 lanes' bits for one
// accumulator register of a 32 x 32 MFMA tile, see rov.h).
// Each ballot is dropped into the lane that will store it (v_writelane), and
// after 16 groups the wave issues one fully coalesced 512-byte store.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <mutex>

#include "mask_device.h"
#include "philox_device.h"
#include "rov_internal.h"

namespace rov {

namespace {

constexpr int kWavesPerBlock = 4;

// The work queues' counters (see mask_device.h): one line per sub-queue.
__device__ QueueCounter g_queues[kQueueSlots][kSubQueues];
std::atomic<unsigned> g_queue_cursor{0};

__global__ void queue_reset_kernel(int slot) { g_queues[slot][threadIdx.x].next = 0ull; }

std::atomic<int> g_rng_max_workgroups{0};
std::atomic<int> g_rng_overlap_wgs_per_cu{0};   // 0 = by the register rule in mask_grid_cap

// One chunk: 16 groups -> 64 mask words = 4 whole tiles of 32 x 32 elements; word 4*gi + r is
// parked in lane 4*gi + r of (vhi:vlo).  RAGGED (S % 32 != 0): bits whose row or column lies
// beyond S are cleared; (qt, kt) are the tile coordinates of the chunk's first tile.
template <int R, bool RAGGED, bool CARRY>
__device__ __forceinline__ void mask_chunk(uint64_t base, uint32_t lane, uint32_t k0, uint32_t k1,
                                           uint32_t t_minus_1, uint32_t T, uint32_t S, uint32_t qt,
                                           uint32_t kt, uint32_t& vlo, uint32_t& vhi) {
#pragma unroll 2
    for (int gi = 0; gi < kGroupsPerChunk; ++gi) {
        uint64_t b[4];
        philox_group_ballots<R, CARRY>(base + 64u * (uint64_t)gi, lane, k0, k1, t_minus_1, b);
        uint32_t row_mask = 0xFFFFFFFFu;
        if (RAGGED) {
            const uint32_t rows_valid = S - 32u * qt;          // >= 1
            if (rows_valid < 32u) row_mask = (1u << rows_valid) - 1u;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            uint32_t lo = (uint32_t)b[r], hi = (uint32_t)(b[r] >> 32);
            if (RAGGED) {
                // word e = 4*(gi%4) + r: lanes 0-31 hold column 32*kt + 8*(gi%4) + r, lanes 32-63 that + 4
                const uint32_t col = 32u * kt + 8u * ((uint32_t)gi & 3u) + (uint32_t)r;
                lo = col < S ? (lo & row_mask) : 0u;
                hi = col + 4u < S ? (hi & row_mask) : 0u;
            }
            const uint32_t dst = 4u * (uint32_t)gi + (uint32_t)r;
            vlo = write_lane(lo, dst, vlo);
            vhi = write_lane(hi, dst, vhi);
        }
        if (RAGGED && (gi & 3) == 3) {   // next tile
            kt = kt + 1u == T ? 0u : kt + 1u;
            if (kt == 0u) qt = qt + 1u == T ? 0u : qt + 1u;
        }
    }
}

// lower_only: skip every chunk (4 consecutive tiles) none of whose tiles has key tile <= query
// tile, i.e. which causal attention never reads; what is written has the same bits either way.
// (at most 24 vector registers for the 10-round kernel: three of its waves then fit on a SIMD beside
// the GEMM kernels, see mask_grid_cap)
template <int R, bool RAGGED>
__global__ __launch_bounds__(kWavesPerBlock * 64) __attribute__((amdgpu_num_vgpr(24))) void mask_kernel(
    uint64_t* __restrict__ out, uint64_t words, uint64_t nchunks, uint64_t offset, uint32_t k0,
    uint32_t k1, uint32_t t_minus_1, uint32_t T, uint32_t Tm, uint32_t S, int lower_only, int qslot, uint64_t qper,
    uint32_t qbatch) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // qslot < 0: the grid strides over the chunks; qslot >= 0: waves pull chunks from a queue that
    // another launch of this kernel may be draining too
    ChunkSource src;
    src.queues = qslot >= 0 ? g_queues[qslot] : nullptr; src.nchunks = nchunks; src.stride = (uint64_t)gridDim.x * kWavesPerBlock;
    src.per = qper; src.batch = qbatch; src.lane = lane;
    for (bool more = src.first((uint64_t)blockIdx.x * kWavesPerBlock + wave); more; more = src.next()) {
        const uint64_t chunk = src.cur;
        uint32_t vlo = 0u, vhi = 0u;
        uint32_t qt = 0u, kt = 0u;   // tile coordinates of the chunk's first tile
        if (RAGGED || lower_only) {
            tile_coords(chunk * 4u, T, Tm, qt, kt);
            // the chunk's tiles are (qt, kt) .. (qt, kt+3), wrapping into row qt+1 at kt = T;
            // a wrapped tile (qt+1, 0) is always needed, so only a chunk that stays inside its
            // row with kt > qt can be skipped
            if (lower_only && kt > qt && kt + 3u < T) continue;
        }
        // first call number of the chunk; its 1024 calls are base .. base + 1023
        const uint64_t base = offset + 64u * kGroupsPerChunk * chunk;
        if ((uint32_t)base <= 0xFFFFFFFFu - (64u * kGroupsPerChunk - 1u)) {
            mask_chunk<R, RAGGED, false>(base, lane, k0, k1, t_minus_1, T, S, qt, kt, vlo, vhi);
        } else {
            mask_chunk<R, RAGGED, true>(base, lane, k0, k1, t_minus_1, T, S, qt, kt, vlo, vhi);
        }
        const uint64_t widx = chunk * 64u + lane;
        if (widx < words) out[widx] = ((uint64_t)vhi << 32) | vlo;
    }
}

// Rows of tiles [qt0, qt0 + nqt) of every (batch, head), written compactly as
// [B*H][nqt][T][16]: the bits are those of the full mask (call numbers come from the global word
// index), only the destination differs.  One "segment" per (batch, head): seg_words = nqt*T*16
// words in `out`, starting at global word seg*seg_stride + seg_first.
template <int R, bool RAGGED>
__global__ __launch_bounds__(kWavesPerBlock * 64) void mask_rows_kernel(
    uint64_t* __restrict__ out, uint64_t seg_words, uint64_t chunks_per_seg, uint64_t nseg,
    uint64_t seg_stride, uint64_t seg_first, uint64_t offset, uint32_t k0, uint32_t k1,
    uint32_t t_minus_1, uint32_t T, uint32_t Tm, uint32_t cps_m, uint32_t S, int qslot, uint64_t qper, uint32_t qbatch) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    ChunkSource src;
    src.queues = qslot >= 0 ? g_queues[qslot] : nullptr; src.nchunks = nseg * chunks_per_seg; src.stride = (uint64_t)gridDim.x * kWavesPerBlock;
    src.per = qper; src.batch = qbatch; src.lane = lane;
    for (bool more = src.first((uint64_t)blockIdx.x * kWavesPerBlock + wave); more; more = src.next()) {
        const uint64_t c = src.cur;
        uint64_t seg, lc;
        if ((c >> 32) == 0u && (chunks_per_seg >> 32) == 0u) {
            uint32_t q, r;
            divmod_u32((uint32_t)c, (uint32_t)chunks_per_seg, cps_m, q, r);
            seg = q; lc = r;
        } else {
            seg = c / chunks_per_seg; lc = c - seg * chunks_per_seg;
        }
        const uint64_t gw = seg * seg_stride + seg_first + lc * 64u;   // first global word (multiple of 16)
        uint32_t kt, qt;
        tile_coords(gw >> 4, T, Tm, qt, kt);
        uint32_t vlo = 0u, vhi = 0u;
        const uint64_t base = offset + 16u * gw;   // 64 calls per 4 words
        if ((uint32_t)base <= 0xFFFFFFFFu - (64u * kGroupsPerChunk - 1u)) {
            mask_chunk<R, RAGGED, false>(base, lane, k0, k1, t_minus_1, T, S, qt, kt, vlo, vhi);
        } else {
            mask_chunk<R, RAGGED, true>(base, lane, k0, k1, t_minus_1, T, S, qt, kt, vlo, vhi);
        }
        const uint64_t lw = lc * 64u + lane;
        if (lw < seg_words) out[seg * seg_words + lw] = ((uint64_t)vhi << 32) | vlo;
    }
}

// Narrow-threshold chunk: BITS (8 or 16) random bits per element.  One Philox call per lane now
// serves E = 4 * 32/BITS mask words: field s of output word r decides word E*gi + 4*s + r of the
// chunk.  A chunk is still 64 words = 4 tiles; tile t of the chunk has coordinates (qts[t], kts[t]).
template <int BITS, bool RAGGED, bool CARRY>
__device__ __forceinline__ void mask_chunk_bits(uint64_t base, uint32_t lane, uint32_t k0, uint32_t k1,
                                                uint32_t tb, uint32_t S, const uint32_t (&qts)[4],
                                                const uint32_t (&kts)[4], uint32_t& vlo, uint32_t& vhi) {
    constexpr int NF = 32 / BITS;          // fields per output word
    constexpr int E = 4 * NF;              // mask words per group
#pragma unroll
    for (int gi = 0; gi < 64 / E; ++gi) {
        const uint64_t b = base + 64u * (uint64_t)gi;
        const uint32_t blo = (uint32_t)b, bhi = (uint32_t)(b >> 32);
        const uint32_t c0 = blo + lane;
        uint32_t x[4];
        if (!CARRY) {
            philox4x32_low_counter<10>(c0, bhi, k0, k1, x);
        } else {
            philox4x32<10>(c0, bhi + (c0 < blo ? 1u : 0u), 0u, 0u, k0, k1, x);
        }
#pragma unroll
        for (int s = 0; s < NF; ++s)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const uint32_t field = (x[r] >> (BITS * s)) & ((1u << BITS) - 1u);
                const uint64_t bal = __ballot(field < tb);
                uint32_t lo = (uint32_t)bal, hi = (uint32_t)(bal >> 32);
                const int dst = E * gi + 4 * s + r;            // word of the chunk
                if (RAGGED) {
                    const int t = dst >> 4, ew = dst & 15;     // tile of the chunk, word of the tile
                    const uint32_t rows_valid = S - 32u * qts[t];
                    const uint32_t row_mask = rows_valid < 32u ? (1u << rows_valid) - 1u : 0xFFFFFFFFu;
                    const uint32_t col = 32u * kts[t] + 8u * (uint32_t)(ew >> 2) + (uint32_t)(ew & 3);
                    lo = col < S ? (lo & row_mask) : 0u;
                    hi = col + 4u < S ? (hi & row_mask) : 0u;
                }
                vlo = write_lane(lo, (uint32_t)dst, vlo);
                vhi = write_lane(hi, (uint32_t)dst, vhi);
            }
    }
}

template <int BITS, bool RAGGED>
__global__ __launch_bounds__(kWavesPerBlock * 64) void mask_bits_kernel(
    uint64_t* __restrict__ out, uint64_t words, uint64_t nchunks, uint64_t offset, uint32_t k0,
    uint32_t k1, uint32_t tb, uint32_t T, uint32_t Tm, uint32_t S) {
    constexpr uint32_t kCallsPerChunk = 64u * (64u / (4u * (32u / BITS)));   // 256 (8 bits) or 512 (16 bits)
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t stride = (uint64_t)gridDim.x * kWavesPerBlock;
    for (uint64_t chunk = (uint64_t)blockIdx.x * kWavesPerBlock + wave; chunk < nchunks;
         chunk += stride) {
        uint32_t vlo = 0u, vhi = 0u;
        uint32_t qts[4] = {0u, 0u, 0u, 0u}, kts[4] = {0u, 0u, 0u, 0u};
        if (RAGGED) {
            uint32_t kt, qt;
            tile_coords(chunk * 4u, T, Tm, qt, kt);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                qts[t] = qt;
                kts[t] = kt;
                kt = kt + 1u == T ? 0u : kt + 1u;
                if (kt == 0u) qt = qt + 1u == T ? 0u : qt + 1u;
            }
        }
        const uint64_t base = offset + (uint64_t)kCallsPerChunk * chunk;
        if ((uint32_t)base <= 0xFFFFFFFFu - (kCallsPerChunk - 1u)) {
            mask_chunk_bits<BITS, RAGGED, false>(base, lane, k0, k1, tb, S, qts, kts, vlo, vhi);
        } else {
            mask_chunk_bits<BITS, RAGGED, true>(base, lane, k0, k1, tb, S, qts, kts, vlo, vhi);
        }
        const uint64_t widx = chunk * 64u + lane;
        if (widx < words) out[widx] = ((uint64_t)vhi << 32) | vlo;
    }
}

__global__ __launch_bounds__(256) void raw_kernel(uint32_t* __restrict__ out, uint64_t ncalls,
                                                  uint64_t first, uint32_t k0, uint32_t k1,
                                                  int rounds) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < ncalls; i += stride) {
        const uint64_t n = first + i;
        uint32_t x[4];
        philox4x32_dyn(rounds, (uint32_t)n, (uint32_t)(n >> 32), 0u, 0u, k0, k1, x);
        reinterpret_cast<uint4*>(out)[i] = make_uint4(x[0], x[1], x[2], x[3]);
    }
}

// Workgroups to launch.  Alone: enough to fill every SIMD's wave slots several times over.
// Beside a GEMM: a persistent grid of a few workgroups per compute unit, so that the GEMM's
// workgroup (most of the registers, most of the LDS) always still fits.  Helper: a persistent
// grid that fills the device once (8 waves per SIMD) and drains what the queue still holds.
// Queue geometry for a mask of nchunks chunks: batch size and chunks per sub-queue.  Batches of
// up to 8 chunks keep the atomic rate far below what one address sustains; small masks get
// smaller batches so that every compute unit still sees several of them.
void queue_geometry(uint64_t nchunks, uint64_t* per, uint32_t* batch) {
    uint64_t b = nchunks / ((uint64_t)kSubQueues * 128u);
    b = b < 1u ? 1u : (b > 8u ? 8u : b);
    uint64_t p = (nchunks + kSubQueues - 1) / kSubQueues;
    p = (p + b - 1) / b * b;
    *per = p;
    *batch = (uint32_t)b;
}

// kernel_regs: vector registers a wave of the mask kernel variant about to be launched is allocated
// (24 or 32).  Beside a GEMM the grid is as many workgroups per compute unit (one wave per SIMD each)
// as fit next to the largest GEMM kernel of this library on every SIMD: that kernel keeps 420 of a
// SIMD's 512 registers (fp8; bf16 408), so 92 are left: three 24-register waves or two 32-register
// ones.  One workgroup more and the GEMM's own workgroups can no longer be placed until the RNG
// grid, which is persistent, has drained (measured: the block's PROJ GEMM 0.47 -> 1.36 ms).  More
// RNG waves per SIMD finish the mask sooner at the same cost to the GEMMs (block at S = 16384:
// 1.96 / 1.53 / 1.25 ms of the RNG exposed with 1 / 2 / 3 waves per SIMD, the GEMMs 8 / 12 / 12 %
// slower).
int mask_grid_cap(int grid_mode, int kernel_regs) {
    const int cap = g_rng_max_workgroups.load();
    if (cap > 0) return cap;
    if (grid_mode == MASK_GRID_BESIDE) {
        const int forced = g_rng_overlap_wgs_per_cu.load();
        const int fit = (512 - 420) / (kernel_regs <= 24 ? 24 : 32);
        return device_cu_count() * (forced > 0 ? forced : (fit < 3 ? fit : 3));
    }
    if (grid_mode == MASK_GRID_HELPER) return device_cu_count() * 8;
    return device_cu_count() * 64;
}

template <int R>
int launch_mask_r(uint64_t* out, uint64_t words, uint64_t offset, uint32_t k0, uint32_t k1,
                  uint32_t t_minus_1, int S, int grid_mode, int qslot, bool lower_only, hipStream_t stream) {
    const uint32_t T = (uint32_t)(((uint64_t)S + 31u) / 32u);
    const uint64_t nchunks = (words + 63u) / 64u;
    uint64_t blocks = (nchunks + kWavesPerBlock - 1) / kWavesPerBlock;
    // registers per wave: 24 for 10 and 3 rounds (and every ragged variant), 25 -> 32 for 7 and 5
    const int cap = mask_grid_cap(grid_mode, ((S & 31) != 0 || R == 10 || R == 3) ? 24 : 32);
    if (blocks > (uint64_t)cap) blocks = (uint64_t)cap;
    // Causal masks with a grid that strides over the chunks: a wave's chunks are `stride` apart, and when
    // the stride is a multiple of a tile row's chunks (T / 4; power-of-two sequence lengths) every
    // chunk of a wave has the same key-tile position - the wave skips all of them or none, half of the
    // waves leave at once and the other half do the whole job in the time of the full mask.  Take a
    // few workgroups off the grid so that the stride advances the key-tile position by about 0.62 of a
    // row per step (and by an odd multiple of four chunks, which visits every fourth position of a
    // power-of-two row): every wave then skips its fair share.
    if (lower_only && qslot < 0 && (T & 3u) == 0u && T >= 32u) {
        const uint64_t row = T / 4u;
        uint64_t want = (uint64_t)((double)row * 0.618) & ~(uint64_t)7u;
        want += 4u;                                            // = 4 (mod 8)
        const uint64_t have = (blocks * kWavesPerBlock) % row;
        const uint64_t off = ((have + row - want % row) % row) / kWavesPerBlock;   // workgroups to drop
        if (off < blocks && blocks - off >= blocks / 2u) blocks -= off;
    }
    const dim3 grid((unsigned)blocks), block(kWavesPerBlock * 64);
    uint64_t qper = 0;
    uint32_t qbatch = 1;
    queue_geometry(nchunks, &qper, &qbatch);
    if ((S & 31) == 0) {
        hipLaunchKernelGGL((mask_kernel<R, false>), grid, block, 0, stream, out, words, nchunks,
                           offset, k0, k1, t_minus_1, T, div_magic(T), (uint32_t)S, (int)lower_only, qslot, qper, qbatch);
    } else {
        hipLaunchKernelGGL((mask_kernel<R, true>), grid, block, 0, stream, out, words, nchunks,
                           offset, k0, k1, t_minus_1, T, div_magic(T), (uint32_t)S, (int)lower_only, qslot, qper, qbatch);
    }
    ROV_LAUNCH_CHECK();
    return ROV_OK;
}

template <int BITS>
int launch_mask_bits_b(uint64_t* out, uint64_t words, uint64_t offset, uint32_t k0, uint32_t k1,
                       uint32_t tb, int S, int grid_mode, hipStream_t stream) {
    const uint32_t T = (uint32_t)(((uint64_t)S + 31u) / 32u);
    const uint64_t nchunks = (words + 63u) / 64u;
    uint64_t blocks = (nchunks + kWavesPerBlock - 1) / kWavesPerBlock;
    const int cap = mask_grid_cap(grid_mode, 24);
    if (blocks > (uint64_t)cap) blocks = (uint64_t)cap;
    const dim3 grid((unsigned)blocks), block(kWavesPerBlock * 64);
    if ((S & 31) == 0) {
        hipLaunchKernelGGL((mask_bits_kernel<BITS, false>), grid, block, 0, stream, out, words, nchunks,
                           offset, k0, k1, tb, T, div_magic(T), (uint32_t)S);
    } else {
        hipLaunchKernelGGL((mask_bits_kernel<BITS, true>), grid, block, 0, stream, out, words, nchunks,
                           offset, k0, k1, tb, T, div_magic(T), (uint32_t)S);
    }
    ROV_LAUNCH_CHECK();
    return ROV_OK;
}

}  // namespace

bool keep_threshold_minus_1(float p, uint32_t* t_minus_1) {
    if (!(p >= 0.0f) || !(p < 1.0f)) return false;
    const double t = (1.0 - (double)p) * 4294967296.0;
    const uint64_t T = (uint64_t)t;   // floor; 256 <= T <= 2^32 for float p in [0,1)
    *t_minus_1 = (uint32_t)(T - 1u);
    return true;
}

int mask_queue_device_ptr(int slot, void** ptr) {
    if (slot < 0 || slot >= kQueueSlots || ptr == nullptr) return ROV_ERR_INVALID;
    // every device holds its own copy of g_queues at its own address
    constexpr int kMaxDevices = 64;
    static std::atomic<QueueCounter*> base[kMaxDevices];
    int dev = 0;
    ROV_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return ROV_ERR_UNSUPPORTED;
    QueueCounter* b = base[dev].load();
    if (b == nullptr) {
        ROV_HIP_TRY(hipGetSymbolAddress((void**)&b, HIP_SYMBOL(g_queues)));
        base[dev].store(b);
    }
    *ptr = b + (size_t)slot * kSubQueues;
    return ROV_OK;
}

void mask_queue_geometry(uint64_t nchunks, uint64_t* per, uint32_t* batch) { queue_geometry(nchunks, per, batch); }

// A slot's last user records `done` behind its last launch that touches the slot
// (mask_queue_release); the next user of the slot makes its stream wait for that event before it
// resets the counters, so a slot is never reset under a grid that still pops from it, whatever
// streams or host threads the two calls came from.  Streams under graph capture are left out of
// the tracking (a captured call neither waits for nor records the event; capture orders its own
// work, and replays of one graph serialise).
namespace {
struct SlotState {
    hipEvent_t done = nullptr;
    bool recorded = false;
    bool in_use = false;     // handed out and not yet released (a mask left in flight keeps its slot across calls)
};
SlotState g_slot_state[kQueueSlots];
std::mutex g_slot_mu;

bool stream_is_capturing(hipStream_t st) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return cs != hipStreamCaptureStatusNone;
}
}  // namespace

int mask_queue_acquire(hipStream_t stream, int* slot) {
    std::lock_guard<std::mutex> lock(g_slot_mu);
    const bool capturing = stream_is_capturing(stream);
    int s = -1;
    for (int tries = 0; tries < kQueueSlots; ++tries) {
        const int c = (int)(g_queue_cursor.fetch_add(1u) % (unsigned)kQueueSlots);
        if (!g_slot_state[c].in_use) {
            s = c;
            break;
        }
    }
    if (s < 0) return ROV_ERR_UNSUPPORTED;   // every slot belongs to a mask that is still in flight
    SlotState& st = g_slot_state[s];
    if (st.recorded && !capturing) ROV_HIP_TRY(hipStreamWaitEvent(stream, st.done, 0));
    hipLaunchKernelGGL(queue_reset_kernel, dim3(1), dim3(kSubQueues), 0, stream, s);
    ROV_LAUNCH_CHECK();
    if (!capturing) st.in_use = true;
    *slot = s;
    return ROV_OK;
}

int mask_queue_release(int slot, hipStream_t stream) {
    if (slot < 0 || slot >= kQueueSlots) return ROV_OK;
    if (stream_is_capturing(stream)) return ROV_OK;
    std::lock_guard<std::mutex> lock(g_slot_mu);
    SlotState& st = g_slot_state[slot];
    st.in_use = false;
    if (st.done == nullptr) ROV_HIP_TRY(hipEventCreateWithFlags(&st.done, hipEventDisableTiming));
    ROV_HIP_TRY(hipEventRecord(st.done, stream));
    st.recorded = true;
    return ROV_OK;
}

// What every mask launch refuses, without launching (rounds: 3, 5, 7, 10; bits: 8, 16, 32).
int check_mask(int B, int H, int S, float p, int rounds, int bits, const uint64_t* out) {
    if (B <= 0 || H <= 0 || S <= 0 || out == nullptr) return ROV_ERR_INVALID;
    if (!aligned(out, 8)) return ROV_ERR_INVALID;
    if (rounds != 10 && rounds != 7 && rounds != 5 && rounds != 3) return ROV_ERR_INVALID;
    if (bits != 32 && bits != 16 && bits != 8) return ROV_ERR_INVALID;
    uint32_t tm1;
    if (!keep_threshold_minus_1(p, &tm1)) return ROV_ERR_INVALID;
    const uint64_t T = ((uint64_t)S + 31u) / 32u;
    // words = B*H*T*T*16; refuse anything that cannot be a real buffer (> 2^40 words)
    const long double wd = (long double)B * H * T * T * 16.0L;
    if (wd > 1099511627776.0L) return ROV_ERR_UNSUPPORTED;
    return ROV_OK;
}

int launch_mask(uint64_t seed, uint64_t offset, int B, int H, int S, float p, int rounds,
                uint64_t* out, hipStream_t stream, int grid_mode, int qslot, bool lower_only) {
    if (qslot >= kQueueSlots) return ROV_ERR_INVALID;
    {
        const int rc = check_mask(B, H, S, p, rounds, 32, out);
        if (rc != ROV_OK) return rc;
    }
    uint32_t tm1;
    (void)keep_threshold_minus_1(p, &tm1);
    const uint64_t T = ((uint64_t)S + 31u) / 32u;
    const uint64_t words = (uint64_t)B * (uint64_t)H * T * T * 16u;
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    switch (rounds) {
        case 10: return launch_mask_r<10>(out, words, offset, k0, k1, tm1, S, grid_mode, qslot, lower_only, stream);
        case 7: return launch_mask_r<7>(out, words, offset, k0, k1, tm1, S, grid_mode, qslot, lower_only, stream);
        case 5: return launch_mask_r<5>(out, words, offset, k0, k1, tm1, S, grid_mode, qslot, lower_only, stream);
        case 3: return launch_mask_r<3>(out, words, offset, k0, k1, tm1, S, grid_mode, qslot, lower_only, stream);
        default: return ROV_ERR_INVALID;
    }
}

int launch_mask_rows(uint64_t seed, uint64_t offset, int B, int H, int S, float p, int q_begin,
                     int q_rows, uint64_t* out, hipStream_t stream, int grid_mode, int qslot) {
    if (qslot >= kQueueSlots) return ROV_ERR_INVALID;
    if (B <= 0 || H <= 0 || S <= 0 || out == nullptr || !aligned(out, 8)) return ROV_ERR_INVALID;
    if (q_begin < 0 || q_rows <= 0 || q_begin >= S || (q_begin & 31) != 0) return ROV_ERR_INVALID;
    uint32_t tm1;
    if (!keep_threshold_minus_1(p, &tm1)) return ROV_ERR_INVALID;
    const uint64_t T = ((uint64_t)S + 31u) / 32u;
    const long double wd = (long double)B * H * T * T * 16.0L;
    if (wd > 1099511627776.0L) return ROV_ERR_UNSUPPORTED;
    const int64_t q_end = (int64_t)q_begin + q_rows < S ? (int64_t)q_begin + q_rows : S;
    const uint64_t nqt = (uint64_t)((q_end - q_begin + 31) / 32);
    const uint64_t seg_words = nqt * T * 16u;
    const uint64_t cps = (seg_words + 63u) / 64u;
    const uint64_t nseg = (uint64_t)B * (uint64_t)H;
    uint64_t blocks = (nseg * cps + kWavesPerBlock - 1) / kWavesPerBlock;
    // registers per wave: 26 (allocated as 32) without the ragged edge handling, 24 with it
    const int cap = mask_grid_cap(grid_mode, (S & 31) == 0 ? 32 : 24);
    if (blocks > (uint64_t)cap) blocks = (uint64_t)cap;
    const dim3 grid((unsigned)blocks), block(kWavesPerBlock * 64);
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    uint64_t qper = 0;
    uint32_t qbatch = 1;
    queue_geometry(nseg * cps, &qper, &qbatch);
    const uint64_t seg_first = (uint64_t)(q_begin / 32) * T * 16u;
    if ((S & 31) == 0) {
        hipLaunchKernelGGL((mask_rows_kernel<10, false>), grid, block, 0, stream, out, seg_words, cps, nseg,
                           T * T * 16u, seg_first, offset, k0, k1, tm1, (uint32_t)T, div_magic(T), div_magic(cps), (uint32_t)S, qslot, qper, qbatch);
    } else {
        hipLaunchKernelGGL((mask_rows_kernel<10, true>), grid, block, 0, stream, out, seg_words, cps, nseg,
                           T * T * 16u, seg_first, offset, k0, k1, tm1, (uint32_t)T, div_magic(T), div_magic(cps), (uint32_t)S, qslot, qper, qbatch);
    }
    ROV_LAUNCH_CHECK();
    return ROV_OK;
}

// `bits` (8 or 16; 32 = launch_mask) random bits per element; grid stride only (no work queue):
// beside a GEMM the grid is the small persistent one and simply runs until it is done.
int launch_mask_bits(uint64_t seed, uint64_t offset, int B, int H, int S, float p, int bits, uint64_t* out,
                     hipStream_t stream, int grid_mode) {
    if (bits == 32) return launch_mask(seed, offset, B, H, S, p, 10, out, stream, grid_mode, -1, false);
    if (bits != 8 && bits != 16) return ROV_ERR_INVALID;
    if (B <= 0 || H <= 0 || S <= 0 || out == nullptr || !aligned(out, 8)) return ROV_ERR_INVALID;
    if (!(p >= 0.0f) || !(p < 1.0f)) return ROV_ERR_INVALID;
    const uint64_t T = ((uint64_t)S + 31u) / 32u;
    const long double wd = (long double)B * H * T * T * 16.0L;
    if (wd > 1099511627776.0L) return ROV_ERR_UNSUPPORTED;
    const uint64_t words = (uint64_t)B * (uint64_t)H * T * T * 16u;
    // keep iff field < Tb, Tb = floor((1 - p) * 2^bits) in double from the float p (0 <= Tb <= 2^bits)
    const uint32_t tb = (uint32_t)(uint64_t)((1.0 - (double)p) * (double)(1u << bits));
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    return bits == 8 ? launch_mask_bits_b<8>(out, words, offset, k0, k1, tb, S, grid_mode, stream)
                     : launch_mask_bits_b<16>(out, words, offset, k0, k1, tb, S, grid_mode, stream);
}

}  // namespace rov

extern "C" {

uint64_t rov_mask_words(int B, int H, int S) {
    if (B <= 0 || H <= 0 || S <= 0) return 0;
    const uint64_t T = ((uint64_t)S + 31u) / 32u;
    return (uint64_t)B * (uint64_t)H * T * T * 16u;
}

uint64_t rov_mask_words_rows(int B, int H, int S, int q_begin, int q_rows) {
    if (B <= 0 || H <= 0 || S <= 0 || q_begin < 0 || q_rows <= 0 || q_begin >= S || (q_begin & 31) != 0)
        return 0;
    const uint64_t T = ((uint64_t)S + 31u) / 32u;
    const int64_t q_end = (int64_t)q_begin + q_rows < S ? (int64_t)q_begin + q_rows : S;
    return (uint64_t)B * (uint64_t)H * (uint64_t)((q_end - q_begin + 31) / 32) * T * 16u;
}

int rov_dropout_mask_generate_rows(uint64_t seed, uint64_t offset, int B, int H, int S, float p,
                                   int q_begin, int q_rows, uint64_t* out, void* stream) {
    return rov::launch_mask_rows(seed, offset, B, H, S, p, q_begin, q_rows, out, (hipStream_t)stream,
                                 rov::MASK_GRID_FULL, -1);
}

uint64_t rov_mask_philox_calls(int B, int H, int S) {
    const uint64_t words = rov_mask_words(B, H, S);
    return 64u * ((words + 3u) / 4u);
}

int rov_set_rng_overlap_workgroups_per_cu(int n) {
    return rov::g_rng_overlap_wgs_per_cu.exchange(n > 0 ? n : 0);
}

int rov_set_rng_max_workgroups(int max_workgroups) {
    return rov::g_rng_max_workgroups.exchange(max_workgroups > 0 ? max_workgroups : 0);
}

int rov_philox_raw(uint64_t seed, uint64_t first_counter, uint64_t ncalls, int rounds,
                   uint32_t* out, void* stream) {
    if (rounds < 1 || rounds > 16) return ROV_ERR_INVALID;
    if (ncalls == 0) return ROV_OK;
    if (out == nullptr || !rov::aligned(out, 16)) return ROV_ERR_INVALID;
    if (ncalls > (1ull << 40)) return ROV_ERR_UNSUPPORTED;
    uint64_t blocks = (ncalls + 255u) / 256u;
    const uint64_t cap = (uint64_t)rov::device_cu_count() * 64u;
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(rov::raw_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       out, ncalls, first_counter, (uint32_t)seed, (uint32_t)(seed >> 32), rounds);
    ROV_LAUNCH_CHECK();
    return ROV_OK;
}

int rov_dropout_mask_generate(uint64_t seed, uint64_t offset, int B, int H, int S, float p,
                              uint64_t* out, void* stream) {
    return rov::launch_mask(seed, offset, B, H, S, p, 10, out, (hipStream_t)stream);
}

int rov_dropout_mask_generate_causal(uint64_t seed, uint64_t offset, int B, int H, int S, float p,
                                     uint64_t* out, void* stream) {
    return rov::launch_mask(seed, offset, B, H, S, p, 10, out, (hipStream_t)stream, rov::MASK_GRID_FULL, -1, true);
}

int rov_dropout_mask_generate_rounds(uint64_t seed, uint64_t offset, int B, int H, int S, float p,
                                     int rounds, uint64_t* out, void* stream) {
    return rov::launch_mask(seed, offset, B, H, S, p, rounds, out, (hipStream_t)stream);
}

uint64_t rov_mask_philox_calls_bits(int B, int H, int S, int bits) {
    if (bits != 8 && bits != 16 && bits != 32) return 0;
    const uint64_t words = rov_mask_words(B, H, S);
    const uint64_t E = 4u * (32u / (unsigned)bits);
    return 64u * ((words + E - 1u) / E);
}

int rov_dropout_mask_generate_bits(uint64_t seed, uint64_t offset, int B, int H, int S, float p,
                                   int bits, uint64_t* out, void* stream) {
    return rov::launch_mask_bits(seed, offset, B, H, S, p, bits, out, (hipStream_t)stream, rov::MASK_GRID_FULL);
}

}  // extern "C"

// Device-side pieces of the keep-mask kernels that more than one translation unit uses: the
// chunk geometry and the work queue through which several launches share one mask.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rov {

constexpr int kGroupsPerChunk = 16;   // 16 groups x 4 words = 64 words = one 8-byte store per lane

// Division of a wave-uniform 32-bit index by a launch constant d without the compiler's software
// 64-bit division (hundreds of instructions, paid once per chunk - also by the chunks a causal mask
// skips, which made skipping them gain nothing).  m = floor(2^32 / d) from the host (0xFFFFFFFF for
// d = 1): mulhi(n, m) is floor(n / d) or one less, so one correction step gives the exact pair.
__host__ __device__ inline uint32_t div_magic(uint64_t d) {
    return d <= 1u ? 0xFFFFFFFFu : (uint32_t)(0x100000000ull / d);
}
__device__ __forceinline__ void divmod_u32(uint32_t n, uint32_t d, uint32_t m, uint32_t& q, uint32_t& r) {
    q = __umulhi(n, m);
    r = n - q * d;
    if (r >= d) { ++q; r -= d; }
}
// (query tile, key tile) of tile number `tile` of a [..][T][T] tile array.
__device__ __forceinline__ void tile_coords(uint64_t tile, uint32_t T, uint32_t Tm, uint32_t& qt, uint32_t& kt) {
    if ((tile >> 32) == 0u) {
        uint32_t row, unused;
        divmod_u32((uint32_t)tile, T, Tm, row, kt);
        divmod_u32(row, T, Tm, unused, qt);
    } else {   // masks beyond 2^32 tiles (4 Tbit): the plain division
        kt = (uint32_t)(tile % T);
        qt = (uint32_t)((tile / T) % T);
    }
}

// Work queues for masks that two launches produce together.  A queue slot is 32 sub-queues, each
// with its own 128-byte line and its own contiguous share of the mask's 64-word chunks: atomics
// on one address retire one after the other (about 10 ns each on this chip, measured), so a
// single counter popped once per chunk would take longer than the Philox work itself.  A wave
// pops `batch` chunks at a time from its home sub-queue and moves on to the next sub-queue when
// that one is empty; empty sub-queues are recognised with a plain load.  The counter of a
// sub-queue is the number of its chunks already handed out, so launches may pop with different
// batch sizes.  A slot is reset before its launches; slots are handed out round-robin so that
// back-to-back schedule calls never share one.
constexpr int kQueueSlots = 64;
constexpr int kSubQueues = 32;
struct alignas(128) QueueCounter {
    unsigned long long next;
    unsigned long long pad[15];
};

// Where a wave's chunks come from: the grid striding over [0, nchunks) (queues == nullptr), or a
// queue slot (the kSubQueues counters at `queues`).
struct ChunkSource {
    QueueCounter* queues;
    uint64_t nchunks, stride;      // static mode: next = cur + stride
    uint64_t per;                  // queue mode: chunks per sub-queue
    uint32_t batch, q, tried, lane;
    uint64_t cur, end;             // queue mode: chunks [cur, end) are this wave's

    __device__ __forceinline__ bool refill() {
        while (tried < (uint32_t)kSubQueues) {
            unsigned long long* ctr = &queues[q].next;
            const uint64_t lo = (uint64_t)q * per;
            uint64_t hi = lo + per;
            hi = hi < nchunks ? hi : nchunks;
            if (lo < hi && __hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < hi - lo) {
                unsigned long long v = 0ull;
                if (lane == 0u) v = atomicAdd(ctr, (unsigned long long)batch);
                const uint32_t vl = __builtin_amdgcn_readfirstlane((uint32_t)v);
                const uint32_t vh = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
                const uint64_t got = ((uint64_t)vh << 32) | vl;
                if (got < hi - lo) {
                    cur = lo + got;
                    end = cur + batch < hi ? cur + batch : hi;
                    return true;
                }
            }
            q = q + 1u == (uint32_t)kSubQueues ? 0u : q + 1u;
            ++tried;
        }
        return false;
    }
    __device__ __forceinline__ bool first(uint64_t wave_index) {
        if (queues == nullptr) {
            cur = wave_index;
            return cur < nchunks;
        }
        q = (uint32_t)(wave_index % (uint64_t)kSubQueues);
        tried = 0u;
        return refill();
    }
    __device__ __forceinline__ bool next() {
        if (queues == nullptr) {
            cur += stride;
            return cur < nchunks;
        }
        if (++cur < end) return true;
        return refill();
    }
};

}  // namespace rov

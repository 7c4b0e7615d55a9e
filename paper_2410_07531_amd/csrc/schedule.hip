// The three schedules of the paper's silicon experiment (Sec. 6.1) and the
// transformer-block forward built on them.
//
//   sequential: GEMM(s) -> RNG kernel -> attention(mask), one stream;
//   fused:      GEMM(s) -> attention with in-kernel Philox, one stream;
//   overlap:    RNG kernel on a side stream while the GEMM(s) run on the main
//               stream; attention(mask) on the main stream after both.
//
// Streams and events only: every kernel is launched by the launchers of the
// other translation units.  Host side: a call first validates every kernel of
// its sequence without launching, then enqueues under one process-wide lock, so
// that the fork / join events (one set per process; a stream-wait captures the
// event's state at the time of the call, so re-recording them for the next call
// is safe) are never re-recorded by another host thread between a call's record
// and its wait.  If a launch fails after the side stream was forked, the side
// stream is still joined into the main stream before the call returns.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <map>
#include <mutex>

#include "rov_internal.h"

namespace rov {
namespace {

struct Events {
    hipEvent_t fork = nullptr, join = nullptr;
    hipEvent_t rng_done[2] = {nullptr, nullptr}, attn_done[2] = {nullptr, nullptr};   // chunked schedule
    bool ok = false;
};

// Serialises the enqueue phase of the schedule entry points (host side only; the work itself is
// asynchronous).  Held from the first event record of a call to its last stream wait.
std::mutex g_sched_mu;

// Call with g_sched_mu held.
int get_events(Events** out) {
    static Events ev;
    if (!ev.ok) {
        ROV_HIP_TRY(hipEventCreateWithFlags(&ev.fork, hipEventDisableTiming));
        ROV_HIP_TRY(hipEventCreateWithFlags(&ev.join, hipEventDisableTiming));
        for (int i = 0; i < 2; ++i) {
            ROV_HIP_TRY(hipEventCreateWithFlags(&ev.rng_done[i], hipEventDisableTiming));
            ROV_HIP_TRY(hipEventCreateWithFlags(&ev.attn_done[i], hipEventDisableTiming));
        }
        ev.ok = true;
    }
    *out = &ev;
    return ROV_OK;
}

// The side stream's part of one call.  fork(): the side stream waits for what the main stream has
// queued so far.  mark(): the point of the side stream the main stream will wait for.  join(): the
// main stream waits for that point.  A call that returns early between fork() and join() (a
// launch failed) still joins: the destructor marks the side stream's end and makes the main
// stream wait for it, so nothing the side stream was given runs unordered against the caller's
// later work on the main stream.
struct SideStream {
    Events* ev = nullptr;
    hipStream_t ms = nullptr, ss = nullptr;
    bool open = false;
    int fork() {
        ROV_HIP_TRY(hipEventRecord(ev->fork, ms));
        ROV_HIP_TRY(hipStreamWaitEvent(ss, ev->fork, 0));
        open = true;
        return ROV_OK;
    }
    int mark() {
        ROV_HIP_TRY(hipEventRecord(ev->join, ss));
        return ROV_OK;
    }
    int join() {
        ROV_HIP_TRY(hipStreamWaitEvent(ms, ev->join, 0));
        open = false;
        return ROV_OK;
    }
    ~SideStream() {
        if (open && hipEventRecord(ev->join, ss) == hipSuccess) (void)hipStreamWaitEvent(ms, ev->join, 0);
    }
};

// Masks left in flight by ROV_SCHED_OVERLAP_DEFERRED calls, keyed by their buffer: what the
// following block needs in order to finish and join them (guarded by g_sched_mu).
struct InFlightMask {
    hipStream_t ss;
    int qslot;              // work queue the small grid pulls from (-1: plain launch, nothing to help with)
    uint64_t seed, offset;
    int B, H, S, causal;
    float p;
};
std::map<const void*, InFlightMask> g_in_flight;

bool valid_schedule(int s) {
    return s == ROV_SCHED_SEQUENTIAL || s == ROV_SCHED_FUSED || s == ROV_SCHED_OVERLAP;
}

int check_gemm_desc(const rov_gemm_desc& g) {
    if (g.A == nullptr || g.Bm == nullptr || g.C == nullptr || g.M <= 0 || g.N <= 0 || g.K <= 0)
        return ROV_ERR_INVALID;
    if (!aligned(g.A, 16) || !aligned(g.Bm, 16) || !aligned(g.C, 16)) return ROV_ERR_INVALID;
    if (g.dtype != ROV_F32 && g.dtype != ROV_BF16 && g.dtype != ROV_FP8_E4M3) return ROV_ERR_INVALID;
    return ROV_OK;
}

int check_attn_desc(const rov_attn_desc& a) {
    if (a.Q == nullptr || a.K == nullptr || a.V == nullptr || a.O == nullptr) return ROV_ERR_INVALID;
    if (a.B <= 0 || a.H <= 0 || a.Hkv <= 0 || a.S <= 0 || a.d <= 0 || (a.H % a.Hkv) != 0)
        return ROV_ERR_INVALID;
    if (a.dtype != ROV_F32 && a.dtype != ROV_BF16)
        return a.dtype == ROV_FP8_E4M3 ? ROV_ERR_UNSUPPORTED : ROV_ERR_INVALID;
    if (!(a.p >= 0.0f) || !(a.p < 1.0f)) return ROV_ERR_INVALID;
    if (a.d > 256 || a.B > 65535 || a.H > 65535) return ROV_ERR_UNSUPPORTED;
    return ROV_OK;
}

// Runs one launcher call bracketed by trace events on its stream.
template <typename F>
int traced(int kind, hipStream_t st, F&& launch) {
    const int slot = trace_begin(kind, st);
    const int rc = launch();
    trace_end(slot, st);
    return rc;
}

int t_gemm(const void* A, const void* Bm, void* C, const void* R, int M, int N, int K, int dtype,
           int transB, float sa, float sb, hipStream_t st) {
    return traced(ROV_TRACE_GEMM, st, [&] {
        return launch_gemm_residual(A, Bm, C, R, M, N, K, dtype, transB, sa, sb, st);
    });
}

int t_mask(uint64_t seed, uint64_t offset, int B, int H, int S, float p, uint64_t* out, hipStream_t st,
           int grid_mode, int qslot, bool lower_only, int rounds = 10, int bits = 32) {
    return traced(grid_mode == MASK_GRID_HELPER ? ROV_TRACE_RNG_HELPER : ROV_TRACE_RNG, st, [&] {
        if (bits != 32) return launch_mask_bits(seed, offset, B, H, S, p, bits, out, st, grid_mode);
        return launch_mask(seed, offset, B, H, S, p, rounds, out, st, grid_mode, qslot, lower_only);
    });
}

// Will the small RNG grid finish while the GEMMs beside it run?  Then the plain launch is enough;
// otherwise the mask goes through a work queue and a helper launch finishes it after the GEMMs.
// The rates are this chip's measured ones with both kernels running: 1.16 PFLOP/s for the bf16
// GEMMs and 2.55 for fp8 (12 % and 8 % below their stand-alone rates; 30 TFLOP/s for the fp32
// kernel), 0.335 T Philox calls/s for the three-waves-per-SIMD grid beside them (0.44 of the
// stand-alone kernel).  A wrong guess costs time (an empty helper launch, about 10 us, or an RNG
// tail at the small grid's rate), never correctness.
bool rng_fits_beside(double gemm_flop, int dtype, double rng_calls) {
    const double rate = dtype == ROV_F32 ? 30e12 : (dtype == ROV_FP8_E4M3 ? 2.55e15 : 1.16e15);
    const double t_gemm = gemm_flop / rate;
    const double t_rng = rng_calls / 0.335e12;
    return t_rng < 0.9 * t_gemm;
}

double gemm_flop(int M, int N, int K) { return 2.0 * (double)M * (double)N * (double)K; }

// Hybrid schedule of the block: how many query rows of the next layer's mask the small RNG grid
// gets done beside the block's PROJ / FC1 / FC2 GEMMs (1.3 PFLOP/s alone, 12 % slower with the RNG
// there all the time, 0.335 T Philox calls/s beside them: this chip's measured rates, the same as in
// rng_fits_beside), with a twentieth of margin, in steps of 2048 rows (a full round of attention
// workgroups at 32 heads); below one step the mask is not worth its launches.
// rov_set_block_hybrid_mask_rows overrides the rule.
std::atomic<int> g_hybrid_rows{0};
int hybrid_rows(const rov_block_cfg* c, int B, int S) {
    const int forced = g_hybrid_rows.load();
    int R;
    if (forced != 0) {
        R = forced < 0 ? 0 : forced;
    } else {
        const double T = (double)B * S;
        const double t_gemms = (gemm_flop((int)T, c->hidden, c->H * c->d) + 3.0 * gemm_flop((int)T, c->ffn, c->hidden)) /
                               1.3e15 * 1.12;
        const double frac = 0.95 * t_gemms * 0.335e12 / (double)rov_mask_philox_calls(B, c->H, S);
        // (while most of it fits, the overlap schedule's full-speed launch for the rest costs no more
        // than drawing those rows in the attention kernel: measured level at 0.8)
        R = frac >= 0.7 ? S : (int)(frac * S / 2048.0) * 2048;
    }
    R = R < S ? R - R % 32 : S;
    return R;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct BlockLayout {
    size_t h, qkv, att, x2, u, total;
};

bool block_layout(const rov_block_cfg* c, int B, int S, BlockLayout* L) {
    if (c == nullptr || B <= 0 || S <= 0 || c->H <= 0 || c->Hkv <= 0 || c->d <= 0 ||
        c->hidden <= 0 || c->ffn <= 0)
        return false;
    const size_t T = (size_t)B * (size_t)S;
    size_t off = 0;
    auto take = [&](size_t elems) {
        const size_t at = off;
        off = align_up(off + elems * 2, 256);
        return at;
    };
    L->h = take(T * c->hidden);
    L->qkv = take(T * (size_t)(c->H + 2 * c->Hkv) * c->d);
    L->att = take(T * (size_t)c->H * c->d);
    L->x2 = take(T * c->hidden);
    L->u = take(T * c->ffn);
    L->total = off;
    return true;
}

}  // namespace
}  // namespace rov

namespace rov {
namespace {
// The layer step for a round count (32 random bits per element) or a width (10 rounds).
int layer_step_impl(int schedule, const rov_gemm_desc* gemms, int n_gemms, const rov_attn_desc* attn,
                    uint64_t seed, uint64_t offset, int rounds, int bits, uint64_t* mask, void* main_stream,
                    void* side_stream) {
    if (rounds != 10 && rounds != 7 && rounds != 5 && rounds != 3) return ROV_ERR_INVALID;
    if (bits != 32 && bits != 16 && bits != 8) return ROV_ERR_INVALID;
    if (bits != 32 && rounds != 10) return ROV_ERR_UNSUPPORTED;
    if (!valid_schedule(schedule) || attn == nullptr || n_gemms < 0 || (n_gemms > 0 && gemms == nullptr))
        return ROV_ERR_INVALID;
    for (int i = 0; i < n_gemms; ++i) {
        const int rc = check_gemm_desc(gemms[i]);
        if (rc != ROV_OK) return rc;
    }
    {
        const int rc = check_attn_desc(*attn);
        if (rc != ROV_OK) return rc;
    }
    const bool dropout = attn->p > 0.0f;
    const bool need_mask = dropout && schedule != ROV_SCHED_FUSED;
    if (need_mask && (mask == nullptr || !aligned(mask, 8))) return ROV_ERR_INVALID;
    if (schedule == ROV_SCHED_OVERLAP && main_stream == side_stream) return ROV_ERR_INVALID;
    hipStream_t ms = (hipStream_t)main_stream, ss = (hipStream_t)side_stream;
    // every kernel of the sequence is checked before the first one is enqueued
    for (int i = 0; i < n_gemms; ++i) {
        const rov_gemm_desc& g = gemms[i];
        const int rc = check_gemm(g.A, g.Bm, g.C, nullptr, EPI_ADD, g.M, g.N, g.K, g.dtype, g.transB);
        if (rc != ROV_OK) return rc;
    }
    {
        int rc = check_attention_rows(attn->Q, attn->K, attn->V, attn->O, attn->B, attn->H, attn->Hkv, attn->S,
                                      attn->d, attn->strides, attn->dtype, attn->p, need_mask ? mask : nullptr, 0,
                                      attn->S, rounds, bits);
        if (rc == ROV_OK && need_mask) rc = check_mask(attn->B, attn->H, attn->S, attn->p, rounds, bits, mask);
        if (rc != ROV_OK) return rc;
    }

    std::lock_guard<std::mutex> sched_lock(g_sched_mu);
    SideStream side;
    int qslot = -1;
    const bool overlap = schedule == ROV_SCHED_OVERLAP && need_mask;
    if (overlap) {
        int rc = get_events(&side.ev);
        if (rc != ROV_OK) return rc;
        side.ms = ms;
        side.ss = ss;
        double flop = 0.0;
        int slowest = ROV_FP8_E4M3;   // the dtype whose GEMM rate is lowest among the sequence's
        for (int i = 0; i < n_gemms; ++i) {
            flop += gemm_flop(gemms[i].M, gemms[i].N, gemms[i].K);
            if (gemms[i].dtype == ROV_F32 || (gemms[i].dtype == ROV_BF16 && slowest != ROV_F32)) slowest = gemms[i].dtype;
        }
        const double calls = (double)rov_mask_philox_calls(attn->B, attn->H, attn->S) * (attn->causal ? 0.5 : 1.0);
        // (cost per call ~ rounds; the narrower kernels have no work-queue form and simply run on)
        if (bits == 32 && !rng_fits_beside(flop, slowest, calls * (0.25 + 0.075 * rounds))) {
            rc = mask_queue_acquire(ms, &qslot);   // reset here: ordered before both RNG launches
            if (rc != ROV_OK) return rc;
        }
        // the mask buffer may still be read by work already queued on the main stream
        rc = side.fork();
        if (rc != ROV_OK) return rc;
    }
    int rc = ROV_OK;
    auto run_gemm = [&](int i) {
        const rov_gemm_desc& g = gemms[i];
        return t_gemm(g.A, g.Bm, g.C, nullptr, g.M, g.N, g.K, g.dtype, g.transB, g.scaleA, g.scaleB, ms);
    };
    if (overlap) {
        // GEMMs first so that their workgroups claim each compute unit's LDS and most of its
        // registers; the RNG workgroups then fill the space left over (paper Sec. 6.2)
        if (n_gemms > 0) {
            rc = run_gemm(0);
            if (rc != ROV_OK) return rc;
        }
        rc = t_mask(seed, offset, attn->B, attn->H, attn->S, attn->p, mask, ss, MASK_GRID_BESIDE, qslot,
                    attn->causal != 0, rounds, bits);
        if (rc != ROV_OK) return rc;
        rc = side.mark();
        if (rc != ROV_OK) return rc;
        for (int i = 1; i < n_gemms; ++i) {
            rc = run_gemm(i);
            if (rc != ROV_OK) return rc;
        }
        // whatever the small grid has not produced when the GEMMs end is finished at full speed
        // (paper Sec. 3.3); waves of this launch leave at once if the queue is already empty
        if (qslot >= 0) {
            rc = t_mask(seed, offset, attn->B, attn->H, attn->S, attn->p, mask, ms, MASK_GRID_HELPER, qslot,
                        attn->causal != 0, rounds, bits);
            if (rc != ROV_OK) return rc;
        }
        rc = side.join();
        if (rc != ROV_OK) return rc;
        rc = mask_queue_release(qslot, ms);
        if (rc != ROV_OK) return rc;
    } else {
        for (int i = 0; i < n_gemms; ++i) {
            rc = run_gemm(i);
            if (rc != ROV_OK) return rc;
        }
        if (need_mask) {
            rc = t_mask(seed, offset, attn->B, attn->H, attn->S, attn->p, mask, ms, MASK_GRID_FULL, -1,
                        attn->causal != 0, rounds, bits);
            if (rc != ROV_OK) return rc;
        }
    }
    return traced(ROV_TRACE_ATTENTION, ms, [&] {
        return launch_attention(attn->Q, attn->K, attn->V, attn->O, attn->B, attn->H, attn->Hkv,
                                attn->S, attn->d, attn->strides, attn->dtype, attn->causal, attn->p,
                                need_mask ? mask : nullptr, seed, offset, ms, rounds, bits);
    });
}

}  // namespace
}  // namespace rov

extern "C" int rov_gemm_swiglu(const void* A, const void* Wg, const void* Wu, void* C, int M, int N, int K,
                               void* stream) {
    return rov::launch_gemm_swiglu(A, Wg, Wu, C, M, N, K, (hipStream_t)stream);
}

extern "C" int rov_gemm_swiglu_fp8(const void* A, const void* Wg, const void* Wu, void* C, int M, int N, int K,
                                   float scaleA, float scaleWg, float scaleWu, float scaleC, void* stream) {
    return rov::launch_gemm_swiglu_fp8(A, Wg, Wu, C, M, N, K, scaleA, scaleWg, scaleWu, scaleC, (hipStream_t)stream);
}

extern "C" int rov_gemm_rng_fused(const void* A, const void* Bm, void* C, int M, int N, int K, uint64_t seed,
                                  uint64_t offset, int B, int H, int S, float p, uint64_t* mask, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    if (A == nullptr || Bm == nullptr || C == nullptr || mask == nullptr) return ROV_ERR_INVALID;
    int rc = rov::check_gemm_rng(A, Bm, C, M, N, K, B, H, S, p, mask);   // nothing is enqueued on an argument error
    if (rc != ROV_OK) return rc;
    int slot = -1;
    rc = rov::mask_queue_acquire(st, &slot);
    if (rc != ROV_OK) return rc;
    rc = rov::traced(ROV_TRACE_GEMM, st, [&] {
        return rov::launch_gemm_rng(A, Bm, C, M, N, K, seed, offset, B, H, S, p, mask, slot, st);
    });
    if (rc != ROV_OK) return rc;
    // what the RNG waves of the GEMM kernel did not get to, at full speed (paper Sec. 3.3)
    rc = rov::traced(ROV_TRACE_RNG_HELPER, st, [&] {
        return rov::launch_mask(seed, offset, B, H, S, p, 10, mask, st, rov::MASK_GRID_HELPER, slot, false);
    });
    if (rc != ROV_OK) return rc;
    return rov::mask_queue_release(slot, st);
}

extern "C" int rov_layer_step(int schedule, const rov_gemm_desc* gemms, int n_gemms,
                              const rov_attn_desc* attn, uint64_t seed, uint64_t offset,
                              uint64_t* mask, void* main_stream, void* side_stream) {
    return rov::layer_step_impl(schedule, gemms, n_gemms, attn, seed, offset, 10, 32, mask, main_stream,
                                side_stream);
}

extern "C" int rov_layer_step_rounds(int schedule, const rov_gemm_desc* gemms, int n_gemms,
                                     const rov_attn_desc* attn, uint64_t seed, uint64_t offset, int rounds,
                                     uint64_t* mask, void* main_stream, void* side_stream) {
    return rov::layer_step_impl(schedule, gemms, n_gemms, attn, seed, offset, rounds, 32, mask, main_stream,
                                side_stream);
}

extern "C" int rov_layer_step_bits(int schedule, const rov_gemm_desc* gemms, int n_gemms,
                                   const rov_attn_desc* attn, uint64_t seed, uint64_t offset, int bits,
                                   uint64_t* mask, void* main_stream, void* side_stream) {
    return rov::layer_step_impl(schedule, gemms, n_gemms, attn, seed, offset, 10, bits, mask, main_stream,
                                side_stream);
}

extern "C" int rov_layer_step_chunked(const rov_gemm_desc* gemms, int n_gemms, const rov_attn_desc* attn,
                                      uint64_t seed, uint64_t offset, int q_chunk_rows,
                                      uint64_t* mask_ring, void* main_stream, void* side_stream) {
    using namespace rov;
    if (attn == nullptr || n_gemms < 0 || (n_gemms > 0 && gemms == nullptr)) return ROV_ERR_INVALID;
    for (int i = 0; i < n_gemms; ++i) {
        const int rc = check_gemm_desc(gemms[i]);
        if (rc != ROV_OK) return rc;
    }
    {
        const int rc = check_attn_desc(*attn);
        if (rc != ROV_OK) return rc;
    }
    if (!(attn->p > 0.0f)) return ROV_ERR_INVALID;                      // nothing to pipeline without dropout
    if (q_chunk_rows <= 0 || (q_chunk_rows & 31) != 0) return ROV_ERR_INVALID;
    if (mask_ring == nullptr || !aligned(mask_ring, 8) || main_stream == side_stream) return ROV_ERR_INVALID;
    hipStream_t ms = (hipStream_t)main_stream, ss = (hipStream_t)side_stream;
    const int S = attn->S, B = attn->B, H = attn->H;
    const int nchunks = (S + q_chunk_rows - 1) / q_chunk_rows;
    const uint64_t slot_words = rov_mask_words_rows(B, H, S, 0, q_chunk_rows);
    uint64_t* slot[2] = {mask_ring, mask_ring + slot_words};
    // every kernel of the sequence is checked before the first one is enqueued (a chunk's mask and
    // attention launches take the same arguments but for the row range, which is valid by construction)
    for (int i = 0; i < n_gemms; ++i) {
        const rov_gemm_desc& g = gemms[i];
        const int rc = check_gemm(g.A, g.Bm, g.C, nullptr, EPI_ADD, g.M, g.N, g.K, g.dtype, g.transB);
        if (rc != ROV_OK) return rc;
    }
    {
        int rc = check_attention_rows(attn->Q, attn->K, attn->V, attn->O, B, H, attn->Hkv, S, attn->d, attn->strides,
                                      attn->dtype, attn->p, mask_ring, 0, q_chunk_rows, 10, 32);
        if (rc == ROV_OK) rc = check_mask(B, H, S, attn->p, 10, 32, mask_ring);
        if (rc != ROV_OK) return rc;
    }

    std::lock_guard<std::mutex> sched_lock(g_sched_mu);
    SideStream side;
    int rc = get_events(&side.ev);
    if (rc != ROV_OK) return rc;
    side.ms = ms;
    side.ss = ss;
    Events* ev = side.ev;
    int qslot[2] = {-1, -1};   // work queue of the chunk that currently owns each ring slot
    auto rng_chunk = [&](int c) {   // small grid on the side stream
        rc = traced(ROV_TRACE_RNG, ss, [&] {
            return launch_mask_rows(seed, offset, B, H, S, attn->p, c * q_chunk_rows, q_chunk_rows, slot[c & 1],
                                    ss, MASK_GRID_BESIDE, qslot[c & 1]);
        });
        if (rc != ROV_OK) return rc;
        ROV_HIP_TRY(hipEventRecord(ev->rng_done[c & 1], ss));
        return (int)ROV_OK;
    };
    auto rng_help = [&](int c) {    // device-filling grid on the main stream: finishes the chunk
        if (qslot[c & 1] < 0) return (int)ROV_OK;
        return traced(ROV_TRACE_RNG_HELPER, ms, [&] {
            return launch_mask_rows(seed, offset, B, H, S, attn->p, c * q_chunk_rows, q_chunk_rows, slot[c & 1],
                                    ms, MASK_GRID_HELPER, qslot[c & 1]);
        });
    };
    {   // chunks 0 and 1 run beside the GEMMs; later chunks run beside attention and always get help
        double flop = 0.0;
        int slowest = ROV_FP8_E4M3;
        for (int i = 0; i < n_gemms; ++i) {
            flop += gemm_flop(gemms[i].M, gemms[i].N, gemms[i].K);
            if (gemms[i].dtype == ROV_F32 || (gemms[i].dtype == ROV_BF16 && slowest != ROV_F32)) slowest = gemms[i].dtype;
        }
        const double calls = 16.0 * (double)slot_words * (nchunks > 1 ? 2.0 : 1.0);
        if (!rng_fits_beside(flop, slowest, calls))
            for (int c = 0; c < 2 && c < nchunks; ++c) {
                rc = mask_queue_acquire(ms, &qslot[c]);
                if (rc != ROV_OK) return rc;
            }
    }
    // the ring may still be read by work queued earlier on the main stream
    rc = side.fork();
    if (rc != ROV_OK) return rc;
    int next_gemm = 0;
    if (n_gemms > 0) {   // first GEMM first, so that its workgroups claim the compute units
        const rov_gemm_desc& g = gemms[0];
        rc = t_gemm(g.A, g.Bm, g.C, nullptr, g.M, g.N, g.K, g.dtype, g.transB, g.scaleA, g.scaleB, ms);
        if (rc != ROV_OK) return rc;
        next_gemm = 1;
    }
    // the first two chunks of the mask are generated beside the GEMMs
    for (int c = 0; c < 2 && c < nchunks; ++c) {
        rc = rng_chunk(c);
        if (rc != ROV_OK) return rc;
    }
    for (int i = next_gemm; i < n_gemms; ++i) {
        const rov_gemm_desc& g = gemms[i];
        rc = t_gemm(g.A, g.Bm, g.C, nullptr, g.M, g.N, g.K, g.dtype, g.transB, g.scaleA, g.scaleB, ms);
        if (rc != ROV_OK) return rc;
    }
    for (int c = 0; c < nchunks; ++c) {
        rc = rng_help(c);
        if (rc != ROV_OK) return rc;
        ROV_HIP_TRY(hipStreamWaitEvent(ms, ev->rng_done[c & 1], 0));
        // both launches that pop from the chunk's queue are now ordered on the main stream
        rc = mask_queue_release(qslot[c & 1], ms);
        if (rc != ROV_OK) return rc;
        qslot[c & 1] = -1;
        rc = traced(ROV_TRACE_ATTENTION, ms, [&] {
            return launch_attention_rows(attn->Q, attn->K, attn->V, attn->O, B, H, attn->Hkv, S, attn->d,
                                         attn->strides, attn->dtype, attn->causal, attn->p, slot[c & 1], true,
                                         seed, offset, c * q_chunk_rows, q_chunk_rows, ms);
        });
        if (rc != ROV_OK) return rc;
        if (c + 2 < nchunks) {   // chunk c+2 reuses this slot once attention has read it
            rc = mask_queue_acquire(ms, &qslot[c & 1]);
            if (rc != ROV_OK) return rc;
            ROV_HIP_TRY(hipEventRecord(ev->attn_done[c & 1], ms));
            ROV_HIP_TRY(hipStreamWaitEvent(ss, ev->attn_done[c & 1], 0));
            rc = rng_chunk(c + 2);
            if (rc != ROV_OK) return rc;
        }
    }
    side.open = false;   // every chunk's side-stream launch has been waited for by its attention
    return ROV_OK;
}

extern "C" size_t rov_block_workspace_bytes(const rov_block_cfg* cfg, int B, int S, int schedule) {
    (void)schedule;
    rov::BlockLayout L;
    if (!rov::block_layout(cfg, B, S, &L)) return 0;
    return L.total;
}

extern "C" int rov_block_hybrid_mask_rows(const rov_block_cfg* cfg, int B, int S) {
    rov::BlockLayout L;
    if (!rov::block_layout(cfg, B, S, &L)) return ROV_ERR_INVALID;
    return rov::hybrid_rows(cfg, B, S);
}

extern "C" int rov_set_block_hybrid_mask_rows(int rows) { return rov::g_hybrid_rows.exchange(rows); }

namespace rov {
namespace {
int block_forward_impl(const rov_block_weights* w, const void* x, void* y, int B, int S,
                       const rov_block_cfg* cfg, int schedule, uint64_t seed,
                       uint64_t offset, int mask_ready, uint64_t* mask,
                       uint64_t* next_mask, void* workspace, size_t workspace_bytes,
                       void* main_stream, void* side_stream) {
    BlockLayout L;
    if (w == nullptr || x == nullptr || y == nullptr ||
        !(valid_schedule(schedule) || schedule == ROV_SCHED_HYBRID || schedule == ROV_SCHED_OVERLAP_DEFERRED) ||
        !block_layout(cfg, B, S, &L))
        return ROV_ERR_INVALID;
    const bool defer = schedule == ROV_SCHED_OVERLAP_DEFERRED;
    if (defer) schedule = ROV_SCHED_OVERLAP;
    if (mask_ready != ROV_MASK_NOT_READY && mask_ready != ROV_MASK_READY && mask_ready != ROV_MASK_IN_FLIGHT)
        return ROV_ERR_INVALID;
    const bool in_flight = mask_ready == ROV_MASK_IN_FLIGHT;
    if (in_flight && schedule != ROV_SCHED_OVERLAP) return ROV_ERR_INVALID;
    if (w->norm1 == nullptr || w->norm2 == nullptr || w->wqkv == nullptr || w->wo == nullptr ||
        w->wg == nullptr || w->wu == nullptr || w->wd == nullptr)
        return ROV_ERR_INVALID;
    if ((cfg->H % cfg->Hkv) != 0 || !(cfg->p >= 0.0f) || !(cfg->p < 1.0f) || !(cfg->eps > 0.0f) ||
        !(cfg->rope_theta > 0.0f))
        return ROV_ERR_INVALID;
    if (cfg->dtype != ROV_BF16 && cfg->dtype != ROV_FP8_E4M3)
        return cfg->dtype == ROV_F32 ? ROV_ERR_UNSUPPORTED : ROV_ERR_INVALID;
    const bool f8 = cfg->dtype == ROV_FP8_E4M3;
    const int dt = cfg->dtype;
    if ((cfg->d != 64 && cfg->d != 128) || (cfg->hidden % 64) != 0 || (cfg->ffn % 64) != 0)
        return ROV_ERR_UNSUPPORTED;
    if (f8) {
        if ((cfg->hidden % 128) != 0 || (cfg->ffn % 128) != 0 || ((cfg->H * cfg->d) % 128) != 0) return ROV_ERR_UNSUPPORTED;
        for (int i = 0; i < 4; ++i)
            if (!(cfg->act_scale[i] > 0.0f)) return ROV_ERR_INVALID;
        for (int i = 0; i < 5; ++i)
            if (!(w->w_scale[i] > 0.0f)) return ROV_ERR_INVALID;
    }
    // fp8: per-tensor dequantisation scales of the quantised activations (h1, a, h2, u) and the weights
    const float sa0 = f8 ? cfg->act_scale[0] : 1.0f, sa1 = f8 ? cfg->act_scale[1] : 1.0f;
    const float sa2 = f8 ? cfg->act_scale[2] : 1.0f, sa3 = f8 ? cfg->act_scale[3] : 1.0f;
    const float sw_qkv = f8 ? w->w_scale[0] : 1.0f, sw_o = f8 ? w->w_scale[1] : 1.0f, sw_g = f8 ? w->w_scale[2] : 1.0f;
    const float sw_u = f8 ? w->w_scale[3] : 1.0f, sw_d = f8 ? w->w_scale[4] : 1.0f;
    if (workspace == nullptr || !aligned(workspace, 256)) return ROV_ERR_INVALID;
    if (workspace_bytes < L.total) return ROV_ERR_WORKSPACE;
    const bool dropout = cfg->p > 0.0f;
    // hybrid: stored bits for query rows [0, R), in-kernel Philox for the rest (the same bits)
    const bool hybrid = schedule == ROV_SCHED_HYBRID && dropout;
    const int R = hybrid ? hybrid_rows(cfg, B, S) : S;
    const bool use_mask = dropout && schedule != ROV_SCHED_FUSED && R > 0;
    if (use_mask && (mask == nullptr || !aligned(mask, 8))) return ROV_ERR_INVALID;
    if (next_mask != nullptr && (!aligned(next_mask, 8) || next_mask == mask)) return ROV_ERR_INVALID;
    const bool overlap = (schedule == ROV_SCHED_OVERLAP || schedule == ROV_SCHED_HYBRID) && dropout;
    if (overlap && main_stream == side_stream) return ROV_ERR_INVALID;
    if (!overlap && next_mask != nullptr) return ROV_ERR_INVALID;   // only the overlap schedule runs ahead
    hipStream_t ms = (hipStream_t)main_stream, ss = (hipStream_t)side_stream;

    char* ws = (char*)workspace;
    void* h = ws + L.h;
    void* qkv = ws + L.qkv;
    void* att = ws + L.att;
    void* x2 = ws + L.x2;
    void* u = ws + L.u;
    const int64_t T = (int64_t)B * S;
    if (T > 0x7FFFFFFF) return ROV_ERR_UNSUPPORTED;
    const int H = cfg->H, Hkv = cfg->Hkv, d = cfg->d, hidden = cfg->hidden, ffn = cfg->ffn;
    const int qkv_n = (H + 2 * Hkv) * d;
    const uint16_t* qp = (const uint16_t*)qkv;
    const int64_t strides[12] = {
        (int64_t)S * qkv_n, qkv_n, d,      // Q
        (int64_t)S * qkv_n, qkv_n, d,      // K
        (int64_t)S * qkv_n, qkv_n, d,      // V
        (int64_t)S * H * d, (int64_t)H * d, d};   // O (elements: bf16, or bytes when fp8)
    // fp8: the attention output is quantised in the attention kernel's epilogue and lives, as bytes, in
    // the slot of the SwiGLU output (free until FC1 runs, after the PROJ GEMM has consumed it)
    void* att_out = f8 ? u : att;
    const float att_q = f8 ? sa1 : 0.0f;
    int rc = ROV_OK;
    // every kernel of the block is checked before the first one is enqueued
#define ROV_STEP(expr)            \
    do {                          \
        rc = (expr);              \
        if (rc != ROV_OK) return rc; \
    } while (0)
    if ((hidden % 8) != 0 || (d % 8) != 0) return ROV_ERR_UNSUPPORTED;   // RMSNorm / RoPE vector width
    ROV_STEP(check_gemm(h, w->wqkv, qkv, nullptr, EPI_ADD, (int)T, qkv_n, hidden, dt, 1));
    ROV_STEP(check_gemm(att_out, w->wo, x2, x, EPI_ADD, (int)T, hidden, H * d, dt, 1));
    if (f8)
        ROV_STEP(check_gemm_swiglu_fp8(h, w->wg, w->wu, u, (int)T, ffn, hidden, sa3));
    else
        ROV_STEP(check_gemm_swiglu(h, w->wg, w->wu, u, (int)T, ffn, hidden));
    ROV_STEP(check_gemm(u, w->wd, y, x2, EPI_ADD, (int)T, hidden, ffn, dt, 1));
    ROV_STEP(check_attention_rows(qp, qp + (int64_t)H * d, qp + (int64_t)(H + Hkv) * d, att_out, B, H, Hkv, S, d, strides,
                                  ROV_BF16, cfg->p, use_mask ? mask : nullptr, 0, S, 10, 32));
    if (use_mask) ROV_STEP(check_mask(B, H, S, cfg->p, 10, 32, mask));
    if (next_mask != nullptr) ROV_STEP(check_mask(B, H, S, cfg->p, 10, 32, next_mask));

    std::lock_guard<std::mutex> sched_lock(g_sched_mu);
    SideStream side;
    if (overlap) {
        ROV_STEP(get_events(&side.ev));
        side.ms = ms;
        side.ss = ss;
    }
    // a mask the previous block left in flight: the record of that call must describe this one
    InFlightMask fl{};
    if (in_flight) {
        if (!use_mask) return ROV_ERR_INVALID;
        const auto it = g_in_flight.find(mask);
        if (it == g_in_flight.end()) return ROV_ERR_INVALID;
        fl = it->second;
        if (fl.ss != ss || fl.seed != seed || fl.offset != offset || fl.B != B || fl.H != H || fl.S != S ||
            fl.p != cfg->p || fl.causal != (cfg->causal != 0))
            return ROV_ERR_INVALID;
        g_in_flight.erase(it);
        side.open = true;   // from here on an early return still joins the side stream
    } else if (use_mask && g_in_flight.count(mask) != 0) {
        return ROV_ERR_INVALID;   // still being written on a side stream: claim it (ROV_MASK_IN_FLIGHT) or rov_mask_finish it
    }
    if (next_mask != nullptr && g_in_flight.count(next_mask) != 0) return ROV_ERR_INVALID;

    // this block's own mask, if nobody produced it yet
    int qslot = -1;
    const double mask_calls = (double)rov_mask_philox_calls(B, H, S) * (cfg->causal ? 0.5 : 1.0);
    if (use_mask && !mask_ready && overlap) {
        if (!rng_fits_beside(gemm_flop((int)((int64_t)B * S), (cfg->H + 2 * cfg->Hkv) * cfg->d, cfg->hidden), dt,
                             mask_calls))
            ROV_STEP(mask_queue_acquire(ms, &qslot));
        ROV_STEP(side.fork());
    }
    ROV_STEP(traced(ROV_TRACE_GLUE, ms, [&] {
        return f8 ? launch_rmsnorm_fp8(x, w->norm1, h, T, hidden, cfg->eps, sa0, ms)
                  : launch_rmsnorm(x, w->norm1, h, T, hidden, cfg->eps, ms);
    }));
    ROV_STEP(t_gemm(h, w->wqkv, qkv, nullptr, (int)T, qkv_n, hidden, dt, 1, sa0, sw_qkv, ms));
    if (use_mask && !mask_ready) {
        if (overlap && R < S) {   // hybrid: the first R rows only, compact
            ROV_STEP(traced(ROV_TRACE_RNG, ss, [&] {
                return launch_mask_rows(seed, offset, B, H, S, cfg->p, 0, R, mask, ss, MASK_GRID_BESIDE, qslot);
            }));
            ROV_STEP(side.mark());
            if (qslot >= 0)
                ROV_STEP(traced(ROV_TRACE_RNG_HELPER, ms, [&] {
                    return launch_mask_rows(seed, offset, B, H, S, cfg->p, 0, R, mask, ms, MASK_GRID_HELPER, qslot);
                }));
        } else if (overlap) {
            ROV_STEP(t_mask(seed, offset, B, H, S, cfg->p, mask, ss, MASK_GRID_BESIDE, qslot, cfg->causal != 0));
            ROV_STEP(side.mark());
            if (qslot >= 0)
                ROV_STEP(t_mask(seed, offset, B, H, S, cfg->p, mask, ms, MASK_GRID_HELPER, qslot, cfg->causal != 0));
        } else {
            ROV_STEP(t_mask(seed, offset, B, H, S, cfg->p, mask, ms, MASK_GRID_FULL, -1, cfg->causal != 0));
        }
    }
    if (in_flight && fl.qslot >= 0)
        // what the small grid (running since the previous block) has not produced by the end of this
        // block's QKV GEMM is finished at full speed (paper Sec. 3.3)
        ROV_STEP(t_mask(seed, offset, B, H, S, cfg->p, mask, ms, MASK_GRID_HELPER, fl.qslot, cfg->causal != 0));
    ROV_STEP(traced(ROV_TRACE_GLUE, ms, [&] {   // q heads then k heads
        return launch_rope(qkv, T, qkv_n, S, H + Hkv, d, cfg->rope_theta, ms);
    }));
    if (use_mask && !mask_ready && overlap) {
        ROV_STEP(side.join());
        ROV_STEP(mask_queue_release(qslot, ms));
    }
    if (in_flight) {
        ROV_STEP(side.mark());    // everything queued on the side stream so far, the RNG grid included
        ROV_STEP(side.join());
        ROV_STEP(mask_queue_release(fl.qslot, ms));
    }

    if (hybrid && R < S) {
        if (R > 0)
            ROV_STEP(traced(ROV_TRACE_ATTENTION, ms, [&] {
                return launch_attention_rows(qp, qp + (int64_t)H * d, qp + (int64_t)(H + Hkv) * d, att_out, B, H, Hkv, S,
                                             d, strides, ROV_BF16, cfg->causal, cfg->p, mask, true, seed, offset, 0,
                                             R, ms, 10, 32, att_q);
            }));
        ROV_STEP(traced(ROV_TRACE_ATTENTION, ms, [&] {
            return launch_attention_rows(qp, qp + (int64_t)H * d, qp + (int64_t)(H + Hkv) * d, att_out, B, H, Hkv, S, d,
                                         strides, ROV_BF16, cfg->causal, cfg->p, nullptr, false, seed, offset, R,
                                         S - R, ms, 10, 32, att_q);
        }));
    } else {
        ROV_STEP(traced(ROV_TRACE_ATTENTION, ms, [&] {
            return launch_attention_rows(qp, qp + (int64_t)H * d, qp + (int64_t)(H + Hkv) * d, att_out, B, H, Hkv, S,
                                         d, strides, ROV_BF16, cfg->causal, cfg->p, use_mask ? mask : nullptr, false,
                                         seed, offset, 0, S, ms, 10, 32, att_q);
        }));
    }

    // the next layer's mask runs beside this block's remaining GEMMs (it would compete with
    // attention for VALU issue, so it starts once attention is done)
    int qslot_next = -1;
    const bool run_ahead = overlap && next_mask != nullptr && R > 0;
    if (run_ahead) {
        const double rest = gemm_flop((int)T, hidden, H * d) + 2.0 * gemm_flop((int)T, ffn, hidden) +
                            gemm_flop((int)T, hidden, ffn);
        // (hybrid with R < S: the rows were chosen to fit, no queue and no helper launch)
        if (R == S && !rng_fits_beside(rest, dt, mask_calls)) ROV_STEP(mask_queue_acquire(ms, &qslot_next));
        ROV_STEP(side.fork());
    }
    ROV_STEP(t_gemm(att_out, w->wo, x2, x, (int)T, hidden, H * d, dt, 1, sa1, sw_o, ms));
    if (run_ahead) {
        if (R < S)
            ROV_STEP(traced(ROV_TRACE_RNG, ss, [&] {
                return launch_mask_rows(seed, offset + rov_mask_philox_calls(B, H, S), B, H, S, cfg->p, 0, R, next_mask,
                                        ss, MASK_GRID_BESIDE, -1);
            }));
        else
            ROV_STEP(t_mask(seed, offset + rov_mask_philox_calls(B, H, S), B, H, S, cfg->p, next_mask, ss,
                            MASK_GRID_BESIDE, qslot_next, cfg->causal != 0));
        ROV_STEP(side.mark());
    }
    ROV_STEP(traced(ROV_TRACE_GLUE, ms, [&] {
        return f8 ? launch_rmsnorm_fp8(x2, w->norm2, h, T, hidden, cfg->eps, sa2, ms)
                  : launch_rmsnorm(x2, w->norm2, h, T, hidden, cfg->eps, ms);
    }));
    // gate and up projections as one product with the SwiGLU in its epilogue: u = silu(h Wg^T) * (h Wu^T),
    // the gate never leaves the accumulators and h is fetched once for both (fp8: u leaves quantised)
    ROV_STEP(traced(ROV_TRACE_GEMM, ms, [&] {
        return f8 ? launch_gemm_swiglu_fp8(h, w->wg, w->wu, u, (int)T, ffn, hidden, sa2, sw_g, sw_u, sa3, ms)
                  : launch_gemm_swiglu(h, w->wg, w->wu, u, (int)T, ffn, hidden, ms);
    }));
    ROV_STEP(t_gemm(u, w->wd, y, x2, (int)T, hidden, ffn, dt, 1, sa3, sw_d, ms));
    if (run_ahead && defer && R == S) {
        // left in flight: the following block (mask_ready == ROV_MASK_IN_FLIGHT) helps and joins
        g_in_flight[next_mask] = InFlightMask{ss, qslot_next, seed, offset + rov_mask_philox_calls(B, H, S), B, H, S,
                                              cfg->causal != 0, cfg->p};
        side.open = false;
    } else if (run_ahead) {
        // what is left of the next mask when the last GEMM ends is finished at full speed
        if (qslot_next >= 0)
            ROV_STEP(t_mask(seed, offset + rov_mask_philox_calls(B, H, S), B, H, S, cfg->p, next_mask, ms,
                            MASK_GRID_HELPER, qslot_next, cfg->causal != 0));
        ROV_STEP(side.join());
        ROV_STEP(mask_queue_release(qslot_next, ms));
    }
#undef ROV_STEP
    return ROV_OK;
}

// Completes a mask that an OVERLAP_DEFERRED block left in flight and nobody claimed: what the small
// grid has not produced yet is finished by a full-size launch on the main stream (paper Sec. 3.3),
// the side stream is joined into the main stream and the work-queue slot is given back.
int mask_finish_impl(uint64_t* mask, void* main_stream) {
    if (mask == nullptr) return ROV_ERR_INVALID;
    std::lock_guard<std::mutex> sched_lock(g_sched_mu);
    const auto it = g_in_flight.find(mask);
    if (it == g_in_flight.end()) return ROV_ERR_INVALID;
    const InFlightMask fl = it->second;
    hipStream_t ms = (hipStream_t)main_stream;
    if (ms == fl.ss) return ROV_ERR_INVALID;
    if (fl.qslot >= 0) {
        const int rc0 = check_mask(fl.B, fl.H, fl.S, fl.p, 10, 32, mask);
        if (rc0 != ROV_OK) return rc0;
    }
    SideStream side;
    int rc = get_events(&side.ev);
    if (rc != ROV_OK) return rc;
    side.ms = ms;
    side.ss = fl.ss;
    g_in_flight.erase(it);
    side.open = true;   // an early return below still joins
    if (fl.qslot >= 0) {
        rc = t_mask(fl.seed, fl.offset, fl.B, fl.H, fl.S, fl.p, mask, ms, MASK_GRID_HELPER, fl.qslot, fl.causal != 0);
        if (rc != ROV_OK) return rc;
    }
    rc = side.mark();
    if (rc != ROV_OK) return rc;
    rc = side.join();
    if (rc != ROV_OK) return rc;
    return mask_queue_release(fl.qslot, ms);
}

// Scratch of rov_block_forward_static: the block's intermediate tensors (normed activations, QKV,
// attention output, residual stream, SwiGLU output) for callers that cannot bring a workspace.
// Every byte a block reads from it was written earlier in the same call, so nothing is cleared
// between calls.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// device address is looked up once per device and that pointer is what the kernels are given.
constexpr size_t kStaticScratchBytes = ROV_BLOCK_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

int static_scratch_ptr(void** out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* ptrs[kMaxDevices] = {};
    int dev = 0;
    ROV_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return ROV_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (ptrs[dev] == nullptr) {
        void* p = nullptr;
        ROV_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (p == nullptr) return ROV_ERR_HIP;
        ptrs[dev] = p;
    }
    *out = ptrs[dev];
    return ROV_OK;
}
}  // namespace
}  // namespace rov

extern "C" int rov_block_forward(const rov_block_weights* w, const void* x, void* y, int B, int S,
                                 const rov_block_cfg* cfg, int schedule, uint64_t seed,
                                 uint64_t offset, int mask_ready, uint64_t* mask,
                                 uint64_t* next_mask, void* workspace, size_t workspace_bytes,
                                 void* main_stream, void* side_stream) {
    return rov::block_forward_impl(w, x, y, B, S, cfg, schedule, seed, offset, mask_ready, mask, next_mask, workspace,
                                   workspace_bytes, main_stream, side_stream);
}

extern "C" int rov_mask_finish(uint64_t* mask, void* main_stream) { return rov::mask_finish_impl(mask, main_stream); }

extern "C" size_t rov_block_static_scratch_bytes(void) { return rov::kStaticScratchBytes; }

extern "C" int rov_block_forward_static(const rov_block_weights* w, const void* x, void* y, int B, int S,
                                        const rov_block_cfg* cfg, int schedule, uint64_t seed,
                                        uint64_t offset, int mask_ready, uint64_t* mask,
                                        uint64_t* next_mask, void* main_stream, void* side_stream) {
    // the size limit comes first: a block too large for the static scratch is an argument error
    // and touches nothing
    const size_t need = rov_block_workspace_bytes(cfg, B, S, schedule);
    if (need == 0) return ROV_ERR_INVALID;
    if (need > rov::kStaticScratchBytes) return ROV_ERR_WORKSPACE;
    void* ws = nullptr;
    const int rc = rov::static_scratch_ptr(&ws);
    if (rc != ROV_OK) return rc;
    return rov::block_forward_impl(w, x, y, B, S, cfg, schedule, seed, offset, mask_ready, mask, next_mask, ws,
                                   rov::kStaticScratchBytes, main_stream, side_stream);
}

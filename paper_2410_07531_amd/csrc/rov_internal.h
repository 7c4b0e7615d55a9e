// Internal helpers shared by the translation units of librov (host side).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "rov.h"

namespace rov {

// Records the failing hipError_t for rov_last_hip_error() and yields ROV_ERR_HIP.
int record_hip_error(hipError_t e);

#define ROV_HIP_TRY(expr)                                        \
    do {                                                         \
        hipError_t rov_e_ = (expr);                              \
        if (rov_e_ != hipSuccess) return ::rov::record_hip_error(rov_e_); \
    } while (0)

// Launch check: hipGetLastError after a kernel launch.
#define ROV_LAUNCH_CHECK() ROV_HIP_TRY(hipGetLastError())

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Number of compute units of the current device (cached per process).
int device_cu_count();

// Raises a kernel's dynamic-LDS limit to `bytes` once per (device, kernel); later calls return at once.
int set_max_dynamic_lds(const void* kern, int bytes);

// Keep threshold minus one: an element is kept iff x <= t_minus_1 (== x < T,
// T = floor((1-p)*2^32) in double, T in [256, 2^32]).  Returns false if p is
// outside [0,1) or NaN.
bool keep_threshold_minus_1(float p, uint32_t* t_minus_1);

// Kernel tracing (rov_trace_enable / rov_trace_read): trace_begin records a timing event on
// `st` and returns a slot (or -1 when tracing is off); trace_end records the closing event.
int trace_begin(int kind, hipStream_t st);
void trace_end(int slot, hipStream_t st);

// Launchers used across translation units (all asynchronous on `stream`).
// Grid of the RNG kernel: alone on the device; a small persistent grid meant to run beside a
// GEMM (overlap schedules); or a device-filling persistent grid that helps such a small grid
// finish, launched where the GEMMs end (the full-speed tail of the RNG, paper Sec. 3.3).  The last two share the mask through a work queue:
// qslot >= 0 (from mask_queue_acquire, which resets the slot on the given stream; it must be
// ordered before both launches) makes the waves pull 64-word chunks from that queue, so each
// chunk is produced by whichever launch gets to it first.  qslot < 0: static striding.
enum { MASK_GRID_FULL = 0, MASK_GRID_BESIDE = 1, MASK_GRID_HELPER = 2 };
int mask_queue_acquire(hipStream_t stream, int* slot);
// To be called once per acquired slot, with a stream on which every launch that uses the slot is
// already ordered (the main stream after the join): the slot's next user waits for that point.
int mask_queue_release(int slot, hipStream_t stream);
// Device address of a queue slot's counters (for kernels of other translation units that pull
// chunks from it), and the queue geometry the mask launches use for a mask of nchunks chunks.
int mask_queue_device_ptr(int slot, void** ptr);
void mask_queue_geometry(uint64_t nchunks, uint64_t* per, uint32_t* batch);
// lower_only: write only what causal attention reads (tiles with key tile <= query tile).
int launch_mask(uint64_t seed, uint64_t offset, int B, int H, int S, float p, int rounds,
                uint64_t* out, hipStream_t stream, int grid_mode = MASK_GRID_FULL, int qslot = -1,
                bool lower_only = false);

// Same layout with `bits` (8, 16 or 32) random bits per element; grid stride, no work queue.
int launch_mask_bits(uint64_t seed, uint64_t offset, int B, int H, int S, float p, int bits, uint64_t* out,
                     hipStream_t stream, int grid_mode);
// Tile rows [q_begin/32, ceil(min(q_begin+q_rows, S)/32)) of every (batch, head), compact
// [B*H][nqt][T][16], same bits as the full mask.
int launch_mask_rows(uint64_t seed, uint64_t offset, int B, int H, int S, float p, int q_begin,
                     int q_rows, uint64_t* out, hipStream_t stream, int grid_mode, int qslot);
int launch_gemm(const void* A, const void* Bm, void* C, int M, int N, int K, int dtype, int transB,
                float scaleA, float scaleB, hipStream_t stream);
// C = alpha * A W^T + R (R: bf16 [M,N] or nullptr); MFMA path only when R is given.
int launch_gemm_residual(const void* A, const void* Bm, void* C, const void* R, int M, int N, int K,
                         int dtype, int transB, float scaleA, float scaleB, hipStream_t stream);
// The same with the epilogue chosen: EPI_ADD as above, EPI_SILU_MUL: C = silu(R) * (alpha * A W^T).
enum { EPI_ADD = 0, EPI_SILU_MUL = 1 };
int launch_gemm_epilogue(const void* A, const void* Bm, void* C, const void* R, int epi, int M, int N, int K,
                         int dtype, int transB, float scaleA, float scaleB, hipStream_t stream);
int launch_attention(const void* Q, const void* K, const void* V, void* O, int B, int H, int Hkv,
                     int S, int d, const int64_t strides[12], int dtype, int causal, float p,
                     const uint64_t* mask, uint64_t seed, uint64_t offset, hipStream_t stream,
                     int rounds = 10 /* Philox rounds of the fused variant: 3, 5, 7 or 10 */,
                     int bits = 32 /* its random bits per element: 8, 16 or 32 (10 rounds only) */);

// Query rows [q_begin, min(q_begin + q_rows, S)) only.  mask_is_rows: `mask` holds just the tile
// rows of that range (as written by launch_mask_rows) instead of the full mask.
int launch_attention_rows(const void* Q, const void* K, const void* V, void* O, int B, int H, int Hkv,
                          int S, int d, const int64_t strides[12], int dtype, int causal, float p,
                          const uint64_t* mask, bool mask_is_rows, uint64_t seed, uint64_t offset,
                          int q_begin, int q_rows, hipStream_t stream, int rounds = 10, int bits = 32,
                          float o_fp8_scale = 0.0f /* > 0: O holds OCP e4m3 bytes of (value / o_fp8_scale), its
                                                      strides count bytes (bf16 inputs, head dimension 64 or 128) */);

// C[M,N] = silu(A Wg^T) * (A Wu^T), bf16 with fp32 accumulation: the two products of a SwiGLU in one
// kernel (both weight matrices [N,K], K % 64 == 0, N % 4 == 0).
int launch_gemm_swiglu(const void* A, const void* Wg, const void* Wu, void* C, int M, int N, int K,
                       hipStream_t stream);
// The same with e4m3 operands and an e4m3 result (the fp8 block's FC1): C = q(silu(sA sWg A Wg^T) *
// (sA sWu A Wu^T) / scaleC), bytes [M,N]; K % 128 == 0, N % 4 == 0.
int launch_gemm_swiglu_fp8(const void* A, const void* Wg, const void* Wu, void* C, int M, int N, int K,
                           float scaleA, float scaleWg, float scaleWu, float scaleC, hipStream_t stream);
int check_gemm_swiglu_fp8(const void* A, const void* Wg, const void* Wu, const void* C, int M, int N, int K,
                          float scaleC);
// One kernel whose workgroups compute a tile of the bf16 GEMM with four waves while four more
// waves generate keep-mask chunks pulled from queue slot `qslot` (paper Sec. 6.1: the single-kernel,
// wave-specialised form of the overlap).  S % 32 == 0; what the RNG waves do not get to stays in
// the queue for a helper launch of the mask kernel.
int launch_gemm_rng(const void* A, const void* Bm, void* C, int M, int N, int K, uint64_t seed, uint64_t offset,
                    int B, int H, int S, float p, uint64_t* mask, int qslot, hipStream_t stream);

// Argument checks of the launchers above, without launching anything: a schedule validates every
// kernel of its sequence with these before it enqueues the first one.
int check_gemm(const void* A, const void* Bm, const void* C, const void* R, int epi, int M, int N, int K,
               int dtype, int transB);
int check_gemm_swiglu(const void* A, const void* Wg, const void* Wu, const void* C, int M, int N, int K);
int check_attention_rows(const void* Q, const void* K, const void* V, const void* O, int B, int H, int Hkv,
                         int S, int d, const int64_t strides[12], int dtype, float p, const uint64_t* mask,
                         int q_begin, int q_rows, int rounds, int bits);
int check_mask(int B, int H, int S, float p, int rounds, int bits, const uint64_t* out);
int check_gemm_rng(const void* A, const void* Bm, const void* C, int M, int N, int K, int B, int H, int S, float p,
                   const uint64_t* mask);

int launch_rmsnorm(const void* x, const void* weight, void* y, int64_t rows, int n, float eps,
                   hipStream_t stream);
// y8 (bytes, [rows, n]) = e4m3(RMSNorm(x) * weight / scale): the fp8 block's quantised activations.
int launch_rmsnorm_fp8(const void* x, const void* weight, void* y8, int64_t rows, int n, float eps, float scale,
                       hipStream_t stream);
int launch_rope(void* buf, int64_t tokens, int64_t row_elems, int S, int nheads, int d, float theta,
                hipStream_t stream);

}  // namespace rov

/*
 * rov - RNG/GEMM overlap for attention dropout on MI355X (gfx950).
 *
 * C ABI of the hot path of "Reducing the Cost of Dropout in Flash-Attention by
 * Hiding RNG with GEMM" (arXiv 2410.07531): a stand-alone Philox kernel writes
 * the dropout keep-mask to HBM on a side stream while dense GEMMs run, and a
 * flash-attention forward consumes the mask (paper Sec. 1, Sec. 6.1).
 *
 * Conventions shared by every entry point
 *  - Return value: ROV_OK (0) or a negative ROV_ERR_* code.  Arguments are checked
 *    for every kernel of a call before the first one is enqueued: on
 *    ROV_ERR_INVALID, ROV_ERR_UNSUPPORTED and ROV_ERR_WORKSPACE nothing was enqueued
 *    and outputs are untouched.  ROV_ERR_HIP means a HIP runtime call failed
 *    (rov_last_hip_error() returns its hipError_t); in an entry point that launches
 *    several kernels the earlier ones stay enqueued and the outputs are undefined,
 *    but a side stream that was forked has been joined into the main stream again.
 *  - Threads: every entry point may be called from several host threads.  The
 *    schedule entry points (rov_layer_step*, rov_block_forward*) serialise their
 *    enqueue phase inside the library; the work they enqueue is ordered by the
 *    streams they are given, as usual.  The process-wide rov_set_* knobs are for
 *    experiments and are read once per call.  Masks that two launches produce
 *    together go through one of 64 work queues of the library; a queue is taken for
 *    the duration of a call (for a mask left in flight: until it is claimed or
 *    finished) and handed out again only after the launches that used it have
 *    completed.  With all 64 taken a call returns ROV_ERR_UNSUPPORTED.
 *  - Every data pointer is a DEVICE pointer owned by the caller, valid until
 *    the work enqueued on `stream` has completed.  The library allocates no
 *    device memory and never synchronises the device: calls are asynchronous
 *    on the given stream.  `stream` is a hipStream_t passed as void* (NULL =
 *    the default stream).  Descriptor structs themselves live in HOST memory
 *    and are read before the call returns.
 *  - Ordering: a call is ordered only against earlier work on the stream(s) it
 *    is given.  Inputs written on any other stream must be complete, or
 *    event-ordered before those streams, when the call is made.
 *  - dtype codes: ROV_F32 = 0, ROV_BF16 = 1, ROV_FP8_E4M3 = 2 (OCP e4m3).
 */
#ifndef ROV_H
#define ROV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ROV_OK 0
#define ROV_ERR_INVALID (-1)      /* null pointer, size <= 0, p outside [0,1), bad enum, misalignment */
#define ROV_ERR_UNSUPPORTED (-2)  /* valid but not implemented shape / dtype combination */
#define ROV_ERR_HIP (-3)          /* a HIP runtime call failed */
#define ROV_ERR_WORKSPACE (-4)    /* workspace too small */

#define ROV_F32 0
#define ROV_BF16 1
#define ROV_FP8_E4M3 2

#define ROV_SCHED_SEQUENTIAL 0    /* GEMMs, RNG kernel, attention: one stream (paper Sec. 6.1, baseline) */
#define ROV_SCHED_FUSED 1         /* GEMMs, attention with in-kernel Philox (paper Sec. 6.1, fusion) */
#define ROV_SCHED_OVERLAP 2       /* RNG on a side stream beside the GEMMs, joined before attention */
#define ROV_SCHED_HYBRID 3        /* rov_block_forward only: OVERLAP for the query rows whose bits fit beside the GEMMs, FUSED for the rest */
#define ROV_SCHED_OVERLAP_DEFERRED 4 /* rov_block_forward only: OVERLAP, but the next layer's mask is left in flight at return */

/* values of rov_block_forward's mask_ready */
#define ROV_MASK_NOT_READY 0      /* the block generates its mask itself */
#define ROV_MASK_READY 1          /* `mask` holds it (and the work that wrote it is ordered before main_stream) */
#define ROV_MASK_IN_FLIGHT 2      /* the previous block's ROV_SCHED_OVERLAP_DEFERRED call is still generating it on side_stream */

/* hipError_t of the last failing HIP call made by this library on the calling thread (0 if none). */
int rov_last_hip_error(void);

/* Static version string. */
const char *rov_version(void);

/* ---------------------------------------------------------------- mask geometry
 * The keep-mask of a B x H x S x S score matrix (paper Sec. 7.2: B*nH*SQ^2 bits)
 * is an array of 64-bit words.  Each S x S matrix is cut into T x T tiles of
 * 32 x 32 elements, T = ceil(S/32), 16 words per tile, row-major
 * [B][H][T (query tile)][T (key tile)][16]:
 *     word index w = (((b*H + h)*T + qt)*T + kt)*16 + e,
 *     bit l (LSB first) of word w  <->  row 32*qt + l%32,
 *                                       column 32*kt + 8*(e/4) + 4*(l/32) + e%4.
 * That is the order in which a 64-lane wave holds a 32 x 32 fp32 MFMA accumulator
 * tile (lane l, register e): a mask word is the per-lane keep predicate of one
 * accumulator register, so attention applies it with one select per element and
 * loads it with scalar loads, and the RNG kernel's 64-lane compare result is the
 * word.  Bits whose row or column is >= S are 0; a set bit means "keep".
 * rov_mask_words         = B*H*T*T*16 (0 if any argument is <= 0).
 * rov_mask_philox_calls  = 64*words/4: how far one mask advances the Philox call
 *                          counter; the next mask (next layer, next step) uses
 *                          offset + this value. */
uint64_t rov_mask_words(int B, int H, int S);
uint64_t rov_mask_philox_calls(int B, int H, int S);

/* ---------------------------------------------------------------- Philox
 * Philox-4x32 block function (the generator the paper uses, Sec. 2.3; round
 * function and constants from the publication it cites).  Call number n (64-bit,
 * wrapping) under a 64-bit seed uses counter (lo32(n), hi32(n), 0, 0) and key
 * (lo32(seed), hi32(seed)).
 *
 * Test hook: out[4*i .. 4*i+3] = Philox(seed, first_counter + i), i < ncalls.
 * out: device, 16-byte aligned, 4*ncalls uint32.  rounds in [1, 16].
 * ncalls == 0 is a no-op returning ROV_OK. */
int rov_philox_raw(uint64_t seed, uint64_t first_counter, uint64_t ncalls, int rounds,
                   uint32_t *out, void *stream);

/* Stand-alone RNG kernel (paper Sec. 6.1, the second dropout scenario: the random
 * bits go to HBM and the attention kernel reads them later).
 * Mask words are taken in groups of four (g = w / 4, r = w % 4).  Lane l of
 * group g makes Philox-4x32-10 call number offset + 64*g + l; output word r of
 * that call, x, decides bit l of mask word 4*g + r: keep iff x < Tp with
 * Tp = floor((1 - p) * 2^32) computed in double from the float p.
 * out: device, 8-byte aligned, rov_mask_words(B,H,S) uint64, fully overwritten.
 * Requires B,H,S > 0 and 0 <= p < 1 (p == 0 keeps everything). */
int rov_dropout_mask_generate(uint64_t seed, uint64_t offset, int B, int H, int S, float p,
                              uint64_t *out, void *stream);

/* Same bits, but only what causal attention reads: every tile with key tile <= query
 * tile is written; of the other tiles, those that share a 64-word chunk (4 consecutive
 * tiles) with a needed tile are written too, the rest of `out` is left untouched.  Halves
 * the RNG work when the mask is only used with causal != 0 (rov_layer_step and
 * rov_block_forward call it that way for causal attention). */
int rov_dropout_mask_generate_causal(uint64_t seed, uint64_t offset, int B, int H, int S, float p,
                                     uint64_t *out, void *stream);

/* Same with a selectable round count (paper Sec. 5.2 studies 3, 5 and 7 rounds).
 * rounds in {3, 5, 7, 10}. */
int rov_dropout_mask_generate_rounds(uint64_t seed, uint64_t offset, int B, int H, int S, float p,
                                     int rounds, uint64_t *out, void *stream);

/* Same layout and call numbering, but with `bits` (8, 16 or 32) random bits per element
 * instead of 32 - the other way, next to fewer rounds (paper Sec. 5.2), of making the RNG
 * kernel cheaper; an addition of this library, not the paper's.  Each 32-bit output word of
 * a call is cut into 32/bits fields, field s = (x >> (bits*s)) & (2^bits - 1); mask words are
 * taken in groups of E = 4*32/bits: lane l of group g = w / E makes call number
 * offset + 64*g + l, and field (w % E) / 4 of output word (w % E) % 4 decides bit l of word w:
 * keep iff field < Tb, Tb = floor((1 - p) * 2^bits) in double from the float p.  The kept
 * probability is quantised to Tb / 2^bits (230/256 for p = 0.1 at 8 bits).  bits == 32 is
 * rov_dropout_mask_generate.  One mask advances the call counter by
 * rov_mask_philox_calls_bits = 64*words/E (0 for an unsupported `bits`).  10 rounds.
 * rov_attention_fwd_dropout reads such a mask like any other; the fused variant that draws
 * the same fields is rov_attention_fwd_dropout_bits.  Other values of bits: ROV_ERR_INVALID. */
uint64_t rov_mask_philox_calls_bits(int B, int H, int S, int bits);
int rov_dropout_mask_generate_bits(uint64_t seed, uint64_t offset, int B, int H, int S, float p,
                                   int bits, uint64_t *out, void *stream);

/* Rows of the mask only (paper Sec. 7.2: chunking along the sequence bounds the mask's
 * memory).  Writes the tile rows that cover query rows [q_begin, min(q_begin + q_rows, S)) of
 * every (batch, head), compactly as [B][H][nqt][T][16] with nqt = ceil((q_end - q_begin)/32):
 * exactly the words the full mask of rov_dropout_mask_generate has there (call numbers come
 * from the position in the full mask, so chunked and unchunked runs drop the same elements).
 * q_begin must be a multiple of 32 and < S; q_rows > 0.  rov_mask_words_rows = B*H*nqt*T*16
 * (0 for invalid arguments). */
uint64_t rov_mask_words_rows(int B, int H, int S, int q_begin, int q_rows);
int rov_dropout_mask_generate_rows(uint64_t seed, uint64_t offset, int B, int H, int S, float p,
                                   int q_begin, int q_rows, uint64_t *out, void *stream);

/* Launch-shape control for the RNG kernel, used by the overlap experiments
 * (paper Sec. 6.2: the RNG kernel must fit beside a GEMM that owns most of each
 * compute unit).  max_workgroups <= 0 restores the default (enough workgroups
 * to fill the device).  Process-wide; returns the previous value. */
int rov_set_rng_max_workgroups(int max_workgroups);

/* Size of the persistent RNG grid that the overlap schedules launch beside a
 * GEMM, in workgroups (4 waves, one per SIMD) per compute unit.  Small enough
 * that a GEMM workgroup still fits on every compute unit whichever kernel
 * arrives first.  n <= 0 restores the default: as many as fit beside the
 * library's largest GEMM kernel on a SIMD's register file (3, or 2 for the
 * mask-kernel variants that need 32 registers).  Returns the previous value
 * (0 = the default rule). */
int rov_set_rng_overlap_workgroups_per_cu(int n);

/* Diagnostic: VALU issue cost of the instruction kinds the RNG kernel is made of
 * (paper Table 1 bounds the RNG kernel by "Issue stage" and "ALU pipe"; the
 * ceiling this build prices the kernel against is derived from these measured
 * costs).  Launches `workgroups` x 256 threads; each lane runs 8 independent
 * chains x 4 x iters operations of `kind`:
 *   0 = 32x32->64 multiply plus one add, 1 = low-half multiply, 2 = high-half
 *   multiply, 3 = three-input xor, 4 = add, 5 = compare-to-ballot plus lane write
 *   plus one add, 6 = MFMA 32x32x16 bf16 (32 independent issues per iteration,
 *   i.e. 32 * 32768 flop per wave per iteration: the matrix-core rate under load).
 * out: device, 2 uint64 per wave (4*workgroups waves): elapsed shader-clock
 * ticks of the loop as read by s_memtime, and a checksum. */
int rov_valu_probe(int kind, int iters, int workgroups, uint64_t *out, void *stream);

/* ---------------------------------------------------------------- GEMM
 * C[M,N] = scaleA*scaleB * sum_k A[m,k] * Bm[k,n], fp32 accumulation (paper
 * Table 1, GEMM column; the QKV / PROJ / FC1 / FC2 layers of Sec. 3.2).
 * A: row-major [M,K].  Bm: row-major [K,N] if transB == 0, row-major [N,K]
 * (K contiguous, the layout of a weight matrix) if transB != 0.
 * C: row-major [M,N]; fp32 for ROV_F32, bf16 for ROV_BF16 and ROV_FP8_E4M3.
 * scaleA, scaleB: per-tensor dequantisation scales (use 1.0f for fp32/bf16).
 * Pointers 16-byte aligned.  Shape limits are reported as ROV_ERR_UNSUPPORTED. */
int rov_gemm(const void *A, const void *Bm, void *C, int M, int N, int K, int dtype, int transB,
             float scaleA, float scaleB, void *stream);

/* Tile width of the bf16 matrix-core GEMM kernel (the Table 1 GEMM column's
 * MMA-bound kernel), in output columns: 0 = chosen per call from the shape (the
 * default: the width that wastes least of the last round of workgroups over the
 * compute units), or one of 128, 160, 192, 224, 256 for every later call.  The
 * result is the same sum in the same order for every width.  rov_gemm_swiglu and
 * rov_gemm_swiglu_fp8 have two tile forms: 256 forces the wide one, 128 the narrow
 * one, other values leave their choice to the shape.  For experiments
 * and tests; process-wide.  Returns the previous value, or ROV_ERR_INVALID
 * (nothing changed) for any other argument. */
int rov_set_gemm_tile_cols(int cols);
/* The tile width the matrix-core kernel uses for an M x N output with the
 * current setting (host-side rule, no device work): 128..256, or
 * ROV_ERR_INVALID for M <= 0 or N <= 0. */
int rov_gemm_tile_cols(int M, int N);

/* C[M,N] = silu(A Wg^T) * (A Wu^T), bf16 operands and result, fp32 accumulation: the gate and
 * up projections of the block's SwiGLU feed-forward (Fig. 2's FC1 in its Llama form) as one
 * product, the gate kept in the accumulators.  A [M,K], Wg and Wu [N,K], all row-major with K
 * contiguous; device pointers, 16-byte aligned.  K % 64 == 0 and N % 4 == 0, else
 * ROV_ERR_UNSUPPORTED. */
int rov_gemm_swiglu(const void *A, const void *Wg, const void *Wu, void *C, int M, int N, int K, void *stream);

/* The same product in fp8 for the fp8 block: A [M,K], Wg, Wu [N,K] and the result C [M,N] are OCP e4m3
 * bytes with one dequantisation scale per tensor:
 *     C = e4m3( silu(scaleA*scaleWg * A Wg^T) * (scaleA*scaleWu * A Wu^T) / scaleC ),
 * nearest code, ties to even, saturating at +-448; fp32 accumulation.  K % 128 == 0 and N % 4 == 0,
 * else ROV_ERR_UNSUPPORTED; A, Wg, Wu 16-byte aligned, C 4-byte aligned; scaleC > 0. */
int rov_gemm_swiglu_fp8(const void *A, const void *Wg, const void *Wu, void *C, int M, int N, int K,
                        float scaleA, float scaleWg, float scaleWu, float scaleC, void *stream);

/* The overlap as ONE kernel (paper Sec. 6.1 names this wave-specialised form beside
 * the two-kernel one it uses): every workgroup computes a tile of
 * C[M,N] = A[M,K] * Bm[N,K]^T (bf16, K contiguous in both, fp32 accumulation) with four
 * of its waves while four more waves generate chunks of the keep-mask of
 * rov_dropout_mask_generate(seed, offset, B, H, S, p) (Philox4x32-10, same bits);
 * what they have not produced when the GEMM ends is produced at full speed by a
 * launch of the mask kernel queued behind it (Sec. 3.3).  On return both C and the
 * whole mask are ordered on `stream`.  For comparison with rov_layer_step's
 * two-kernel overlap; slower than it on this chip (the GEMM must use its
 * narrowest tile so that two waves fit on a SIMD).
 * Device pointers: A, Bm, C 16-byte aligned, mask 8-byte aligned with
 * rov_mask_words(B,H,S) words.  K % 64 == 0, N % 4 == 0, S % 32 == 0, else
 * ROV_ERR_UNSUPPORTED; null pointers, sizes <= 0, p outside [0,1): ROV_ERR_INVALID. */
int rov_gemm_rng_fused(const void *A, const void *Bm, void *C, int M, int N, int K, uint64_t seed,
                       uint64_t offset, int B, int H, int S, float p, uint64_t *mask, void *stream);

/* ---------------------------------------------------------------- attention
 * O = dropout(softmax(Q K^T / sqrt(d))) V, dropout applied to the softmax
 * output (paper Sec. 2.2), kept probabilities scaled by 1/(1-p); the softmax
 * normaliser runs over all admissible columns.  Query head h uses key/value
 * head h / (H / Hkv).  causal != 0: column j admissible for row i iff j <= i.
 * Element (b, s, h, t) of tensor X lives at X[b*strides[3x] + s*strides[3x+1] +
 * h*strides[3x+2] + t] with x = 0 (Q), 1 (K), 2 (V), 3 (O); strides in elements;
 * the head dimension is contiguous.
 * mask != NULL: keep-mask words as written by rov_dropout_mask_generate for the
 *               same (B,H,S) - the paper's "attention with element dropping".
 * mask == NULL and p > 0: the fused variant (paper Sec. 6.1, fusion): the kernel
 *               generates the same Philox bits itself from (seed, offset).
 * p == 0 disables dropout (mask, seed, offset ignored). */
int rov_attention_fwd_dropout(const void *Q, const void *K, const void *V, void *O,
                              int B, int H, int Hkv, int S, int d, const int64_t strides[12],
                              int dtype, int causal, float p, const uint64_t *mask,
                              uint64_t seed, uint64_t offset, void *stream);

/* Same with a selectable Philox round count for the fused variant (paper Sec. 5.2): with
 * mask == NULL and p > 0 the kernel draws the bits of
 * rov_dropout_mask_generate_rounds(seed, offset, ..., rounds).  rounds in {3, 5, 7, 10}; with a
 * mask, or p == 0, the value is only checked. */
int rov_attention_fwd_dropout_rounds(const void *Q, const void *K, const void *V, void *O,
                                     int B, int H, int Hkv, int S, int d, const int64_t strides[12],
                                     int dtype, int causal, float p, const uint64_t *mask,
                                     uint64_t seed, uint64_t offset, int rounds, void *stream);

/* Same with `bits` (8, 16 or 32) random bits per element for the fused variant: with mask == NULL
 * and p > 0 the kernel draws the bits of rov_dropout_mask_generate_bits(seed, offset, ..., bits)
 * (a lane makes one Philox call per 4*32/bits of its elements).  10 rounds. */
int rov_attention_fwd_dropout_bits(const void *Q, const void *K, const void *V, void *O,
                                   int B, int H, int Hkv, int S, int d, const int64_t strides[12],
                                   int dtype, int causal, float p, const uint64_t *mask,
                                   uint64_t seed, uint64_t offset, int bits, void *stream);

/* Same for query rows [q_begin, min(q_begin + q_rows, S)) only: those rows of O are written,
 * the others are left alone.  mask_rows (may be NULL: fused variant) holds just the tile rows
 * of that range, as written by rov_dropout_mask_generate_rows with the same q_begin, q_rows.
 * q_begin: multiple of 32, < S. */
int rov_attention_fwd_dropout_rows(const void *Q, const void *K, const void *V, void *O,
                                   int B, int H, int Hkv, int S, int d, const int64_t strides[12],
                                   int dtype, int causal, float p, const uint64_t *mask_rows,
                                   uint64_t seed, uint64_t offset, int q_begin, int q_rows,
                                   void *stream);

/* ---------------------------------------------------------------- schedules
 * One "layer step" of the paper's silicon experiment (Sec. 6.1): n_gemms
 * independent GEMMs, the RNG kernel, then attention with dropout, arranged by
 * `schedule`:
 *   ROV_SCHED_SEQUENTIAL: GEMMs -> RNG -> attention(mask), all on main_stream.
 *   ROV_SCHED_FUSED:      GEMMs -> attention(fused Philox) on main_stream.
 *   ROV_SCHED_OVERLAP:    RNG on side_stream concurrently with the GEMMs on
 *                         main_stream; attention(mask) on main_stream after both.
 *                         If the RNG is not done when the GEMMs end, the rest of it runs
 *                         at full speed (paper Sec. 3.3): a second RNG launch on
 *                         main_stream shares the mask's chunks with the first through a
 *                         work queue and exits at once when none are left.
 * mask: device buffer of rov_mask_words(B,H,S) words (unused for FUSED, may be
 * NULL there).  side_stream must differ from main_stream for OVERLAP. */
typedef struct rov_gemm_desc {
    const void *A;
    const void *Bm;
    void *C;
    int M, N, K;
    int dtype;
    int transB;
    float scaleA, scaleB;
} rov_gemm_desc;

typedef struct rov_attn_desc {
    const void *Q;
    const void *K;
    const void *V;
    void *O;
    int B, H, Hkv, S, d;
    int64_t strides[12];
    int dtype;
    int causal;
    float p;
} rov_attn_desc;

int rov_layer_step(int schedule, const rov_gemm_desc *gemms, int n_gemms, const rov_attn_desc *attn,
                   uint64_t seed, uint64_t offset, uint64_t *mask, void *main_stream,
                   void *side_stream);

/* rov_layer_step with a selectable Philox round count (paper Sec. 5.2: fewer rounds shrink both
 * the stand-alone RNG kernel and the fused attention kernel, and with them what the overlap
 * schedule has to hide).  rounds in {3, 5, 7, 10} applies to the mask kernel (SEQUENTIAL, OVERLAP)
 * and to the in-kernel generation (FUSED) alike, so the three schedules still drop the same
 * elements: those of rov_dropout_mask_generate_rounds(seed, offset, ..., rounds).  rounds == 10 is
 * rov_layer_step.  Other values: ROV_ERR_INVALID. */
int rov_layer_step_rounds(int schedule, const rov_gemm_desc *gemms, int n_gemms,
                          const rov_attn_desc *attn, uint64_t seed, uint64_t offset, int rounds,
                          uint64_t *mask, void *main_stream, void *side_stream);

/* rov_layer_step with `bits` (8, 16 or 32) random bits per element for the mask kernel, the
 * other way of shrinking the RNG (paper Sec. 5.2): the three schedules drop the elements of
 * rov_dropout_mask_generate_bits(seed, offset, ..., bits) (FUSED draws the same fields in the
 * attention kernel).  bits == 32 is rov_layer_step.  Other values: ROV_ERR_INVALID. */
int rov_layer_step_bits(int schedule, const rov_gemm_desc *gemms, int n_gemms,
                        const rov_attn_desc *attn, uint64_t seed, uint64_t offset, int bits,
                        uint64_t *mask, void *main_stream, void *side_stream);

/* The overlap schedule with the mask pipelined in chunks of q_chunk_rows query rows (paper
 * Sec. 7.2, sequence chunking): mask_ring holds two slots of
 * rov_mask_words_rows(B,H,S,0,q_chunk_rows) words instead of the whole mask.  Chunks 0 and 1 are
 * generated on side_stream beside the GEMMs; attention runs chunk by chunk on main_stream, and
 * chunk c+2 is generated into the slot of chunk c while attention works on chunk c+1.  Output
 * and dropped elements are those of rov_layer_step with the full mask.  Requires attn->p > 0,
 * q_chunk_rows a positive multiple of 32, side_stream != main_stream. */
int rov_layer_step_chunked(const rov_gemm_desc *gemms, int n_gemms, const rov_attn_desc *attn,
                           uint64_t seed, uint64_t offset, int q_chunk_rows, uint64_t *mask_ring,
                           void *main_stream, void *side_stream);

/* ---------------------------------------------------------------- kernel tracing
 * Per-kernel timing of what rov_layer_step and rov_block_forward launch (the
 * paper times each kernel of the sequence after warm-up, Sec. 6.1).  While
 * enabled, every kernel launched by those two entry points is bracketed by
 * timing events on its own stream.  rov_trace_read waits for the recorded
 * events (HOST-side wait on them only), writes up to max_records (kind,
 * milliseconds) pairs in launch order into the HOST arrays, stores the count in
 * *n_records and clears the log.  Kinds: ROV_TRACE_GEMM, _RNG, _ATTENTION,
 * _GLUE (RMSNorm / RoPE / SwiGLU), _RNG_HELPER (the second RNG launch of the overlap schedules,
 * which finishes on main_stream, at full device width, what the small grid on side_stream has
 * not produced by the time the GEMMs end).  At most 16384 records are kept between reads.
 * rov_trace_enable(on): 0 switches tracing off, a negative value traces every kind, a positive
 * value is a set of kinds (bit k set = trace kind k), so that a timed loop can carry the two
 * events of its dominant kernel only.  Returns the previous setting. */
#define ROV_TRACE_GEMM 0
#define ROV_TRACE_RNG 1
#define ROV_TRACE_ATTENTION 2
#define ROV_TRACE_GLUE 3
#define ROV_TRACE_RNG_HELPER 4
int rov_trace_enable(int on);
int rov_trace_read(int *kinds, float *ms, int max_records, int *n_records);

/* ---------------------------------------------------------------- transformer block
 * Llama-style block forward (paper Fig. 2 / Sec. 3.2 block with RMSNorm, rotary
 * embedding, grouped-query attention, SwiGLU):
 *   h1 = RMSNorm(x)*norm1; [q|k|v] = h1 Wqkv^T; RoPE(q,k); a = attention_dropout(q,k,v);
 *   x2 = x + a Wo^T; h2 = RMSNorm(x2)*norm2; y = x2 + (silu(h2 Wg^T) * (h2 Wu^T)) Wd^T.
 * RoPE rotates the adjacent pair (2t, 2t+1) of token position s by s*theta^(-2t/d).
 * Weights are row-major [out_features, in_features]; d must be 64 or 128.  x, y: bf16
 * [B, S, hidden].
 * cfg->dtype == ROV_BF16: bf16 weights, hidden and ffn multiples of 64.
 * cfg->dtype == ROV_FP8_E4M3 (the precision the paper measures in, Sec. 1 / Sec. 6): the five
 *   weight matrices are OCP e4m3 bytes with one dequantisation scale each (w->w_scale), and every
 *   GEMM takes its activation in e4m3 too, quantised with a per-tensor scale the caller supplies
 *   (cfg->act_scale, e.g. amax / 448 from a calibration pass, so that nothing here synchronises):
 *     h1 = Q0(RMSNorm(x)*norm1); a = Q1(attention_dropout(q,k,v)); h2 = Q2(RMSNorm(x2)*norm2);
 *     u = Q3(silu(h2 Wg^T) * (h2 Wu^T)),  Qi(v) = act_scale[i] * e4m3(v / act_scale[i])
 *   (nearest code, ties to even, saturating at +-448), each applied where the value is produced
 *   (normalisation kernel, attention epilogue, FC1 epilogue).  q, k, v, the residual stream and y
 *   stay bf16; GEMMs accumulate in fp32.  hidden, ffn and H*d multiples of 128; norm weights bf16.
 *   Scales must be > 0.
 *
 * This block's attention uses the mask of (seed, offset), p = cfg->p:
 *   SEQUENTIAL  mask_ready == 0: the RNG kernel runs on main_stream between the
 *               QKV GEMM and attention.  mask_ready != 0: `mask` already holds it.
 *   FUSED       no mask buffer; attention generates the bits itself.
 *   OVERLAP     mask_ready == 0: the RNG kernel runs on side_stream beside the QKV
 *               GEMM and is joined before attention.  mask_ready != 0: `mask`
 *               already holds it (written during the previous block).  If
 *               next_mask != NULL, the mask of the following layer (offset +
 *               rov_mask_philox_calls(B,H,S)) is generated into it on side_stream
 *               beside this block's PROJ / FC1 / FC2 GEMMs and joined at the end
 *               (paper Sec. 1: RNG hidden behind the GEMM layers between the
 *               previous and the current attention).  next_mask must be NULL for
 *               the other schedules and must differ from mask.
 *   OVERLAP_DEFERRED  As OVERLAP, for a stack of blocks called one after the other on the same
 *               stream pair: the mask of the following layer is started beside this block's
 *               PROJ / FC1 / FC2 GEMMs and NOT joined when the call returns.  The following
 *               block is called with that buffer as `mask` and mask_ready ==
 *               ROV_MASK_IN_FLIGHT: the RNG keeps running beside its RMSNorm and QKV GEMM - all
 *               the GEMM layers between the previous and the current attention, as in paper
 *               Sec. 1 - whatever is left then runs at full speed (Sec. 3.3), and the side
 *               stream is joined before its attention.  Until that call (or any other work
 *               ordered after side_stream) `next_mask` is incomplete.  mask_ready ==
 *               ROV_MASK_IN_FLIGHT is accepted by OVERLAP and OVERLAP_DEFERRED, with the seed,
 *               offset, sizes, p and causal flag the deferred call used for that buffer, else
 *               ROV_ERR_INVALID.
 *   HYBRID      (not in the paper; for sequences so long that the RNG outlasts the
 *               GEMMs, the paper's third regime of Sec. 4.1.)  As OVERLAP, but a mask
 *               holds only the first R = rov_block_hybrid_mask_rows(cfg, B, S) query
 *               rows, in the layout of rov_dropout_mask_generate_rows(q_begin = 0,
 *               q_rows = R), R chosen so that the RNG kernel finishes beside the
 *               GEMMs; attention takes stored bits for those rows and draws the
 *               same bits in-kernel for the others, so the output is that of the
 *               other schedules bit for bit.  R == S is OVERLAP, R == 0 is FUSED.
 *               mask / next_mask as for OVERLAP (mask may be NULL when R == 0).
 * workspace: device scratch, 256-byte aligned, at least
 * rov_block_workspace_bytes() bytes; contents undefined afterwards. */
typedef struct rov_block_cfg {
    int H, Hkv, d, hidden, ffn;
    int dtype;
    int causal;
    float p;
    float eps;
    float rope_theta;
    float act_scale[4];  /* ROV_FP8_E4M3 only: dequantisation scales of h1, a, h2, u (ignored for bf16) */
} rov_block_cfg;

typedef struct rov_block_weights {
    const void *norm1;   /* [hidden] */
    const void *norm2;   /* [hidden] */
    const void *wqkv;    /* [(H + 2*Hkv)*d, hidden] */
    const void *wo;      /* [hidden, H*d] */
    const void *wg;      /* [ffn, hidden] */
    const void *wu;      /* [ffn, hidden] */
    const void *wd;      /* [hidden, ffn] */
    float w_scale[5];    /* ROV_FP8_E4M3 only: dequantisation scales of wqkv, wo, wg, wu, wd (ignored for bf16) */
} rov_block_weights;

size_t rov_block_workspace_bytes(const rov_block_cfg *cfg, int B, int S, int schedule);

/* Rows of a mask under ROV_SCHED_HYBRID: a multiple of 32 in [0, S] (host-side rule from the
 * block's GEMM work and the mask's Philox calls; ROV_ERR_INVALID for a bad cfg or size).
 * rov_set_block_hybrid_mask_rows: rows > 0 forces that many (rounded down to 32, at most S),
 * rows < 0 forces none, 0 restores the rule; process-wide, for tests and experiments; returns
 * the previous setting. */
int rov_block_hybrid_mask_rows(const rov_block_cfg *cfg, int B, int S);
int rov_set_block_hybrid_mask_rows(int rows);

int rov_block_forward(const rov_block_weights *w, const void *x, void *y, int B, int S,
                      const rov_block_cfg *cfg, int schedule, uint64_t seed, uint64_t offset,
                      int mask_ready, uint64_t *mask, uint64_t *next_mask,
                      void *workspace, size_t workspace_bytes, void *main_stream, void *side_stream);

/* Completes a mask that a ROV_SCHED_OVERLAP_DEFERRED call left in flight when no following block
 * will claim it (the last block of a stack, a caller that changes its mind): whatever the small
 * RNG grid on the side stream has not produced yet is generated at full speed on main_stream
 * (paper Sec. 3.3: the rest of the RNG runs alone once the GEMMs are over), and main_stream then
 * waits for the side stream, so that work enqueued on main_stream afterwards sees the whole mask.
 * mask: the `next_mask` of that call.  main_stream: the main stream of that call (or a stream
 * ordered after it); it must differ from the side stream the deferred call used.  ROV_ERR_INVALID if the buffer is not in flight (nothing is enqueued).  While a buffer
 * is in flight, rov_block_forward accepts it only as `mask` with ROV_MASK_IN_FLIGHT; any other use
 * of it there is ROV_ERR_INVALID, and the caller must not free it. */
int rov_mask_finish(uint64_t *mask, void *main_stream);

/* rov_block_forward for callers that cannot allocate device memory or carry a workspace around:
 * code running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results and errors as rov_block_forward, minus the workspace: the block's
 * intermediate tensors live in a scratch array that is part of the library's device image
 * (ROV_BLOCK_STATIC_SCRATCH_BYTES = 64 MiB per GPU the library runs on, held until the process
 * ends).  The call allocates nothing and frees nothing.  A block that needs more scratch than that
 * (rov_block_workspace_bytes(cfg, B, S, schedule) > rov_block_static_scratch_bytes(); 64 MiB is
 * 1024 tokens of a hidden-4096 / ffn-14336 block) is refused with ROV_ERR_WORKSPACE before
 * anything is enqueued.  Every call on a GPU uses that GPU's one array: two calls whose work
 * overlaps in time on one GPU (different stream pairs, or two host threads) race on it, so
 * callers serialise them; back-to-back calls on one main stream are ordered by the stream.
 * Nothing in the array needs clearing between calls (a block writes every byte before it reads
 * it). */
#define ROV_BLOCK_STATIC_SCRATCH_BYTES (64u << 20)
size_t rov_block_static_scratch_bytes(void);
int rov_block_forward_static(const rov_block_weights *w, const void *x, void *y, int B, int S,
                             const rov_block_cfg *cfg, int schedule, uint64_t seed, uint64_t offset,
                             int mask_ready, uint64_t *mask, uint64_t *next_mask,
                             void *main_stream, void *side_stream);

#ifdef __cplusplus
}
#endif
#endif /* ROV_H */

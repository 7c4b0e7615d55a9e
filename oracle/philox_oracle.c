/*
 * CPU oracle: Philox4x32-R block function and the attention-dropout keep-mask.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call, link or
 * import this file; it exists so that the HIP kernels can be compared, bit for
 * bit, with a slow and obviously correct scalar implementation.  It shares no
 * code, header, table or constant generator with the HIP path.
 *
 * What it follows:
 *  - The paper (Sec. 2.3) names Philox, a counter-based generator built on
 *    wide multiplies, and cites the Philox publication (Salmon, Moraes, Dror,
 *    Shaw, "Parallel random numbers: as easy as 1, 2, 3", SC'11) for the round
 *    function; the constants and the round below are those of that
 *    publication's Philox-4x32 and are pinned by its known-answer vectors.
 *  - The paper (Sec. 6.1, Sec. 7.2) says the stand-alone RNG kernel stores one
 *    bit per element of the B x nH x SQ x SQ score matrix.  The paper does not
 *    say how (seed, offset, element) map to (counter, key, output word, bit);
 *    the map used here is a reading, written out in oracle_dropout_mask().
 *
 * Parity pins (tests marked "not gpu"): known-answer vectors for R = 10 and
 * R = 7, the C++26 engine's specified 10000th output, threshold closed forms,
 * kept-fraction within 4 sigma, offset splitting, monotonicity in p, and an
 * independent big-integer Python evaluation of the same definitions; for the
 * 8/16-bit variants additionally a hand-decoded example on the pinned raw
 * words and a numpy reconstruction from the raw stream.
 * Statistical quality of Philox itself: parity unpinned (taken from the cited
 * publication).
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>

/* Multipliers and Weyl key increments of Philox-4x32 (Philox publication). */
#define PHILOX_M0 0xD2511F53u
#define PHILOX_M1 0xCD9E8D57u
#define PHILOX_W0 0x9E3779B9u
#define PHILOX_W1 0xBB67AE85u

/* One Philox-4x32 block: `rounds` rounds on counter c[0..3] with key k[0..1].
 * Round: p0 = M0*c0, p1 = M1*c2 (64-bit products);
 *        c <- ( hi(p1)^c1^k0, lo(p1), hi(p0)^c3^k1, lo(p0) );
 * the key is advanced by (W0, W1) between rounds. */
void oracle_philox4x32(const uint32_t ctr[4], const uint32_t key[2], int rounds,
                       uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < rounds; ++r) {
        uint64_t p0 = (uint64_t)PHILOX_M0 * (uint64_t)c0;
        uint64_t p1 = (uint64_t)PHILOX_M1 * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += PHILOX_W0;
        k1 += PHILOX_W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The (seed, call index) -> (counter, key) map of this build:
 * key = (lo32(seed), hi32(seed)); counter = (lo32(n), hi32(n), 0, 0) where n is
 * the 64-bit call index (arithmetic mod 2^64). */
static void philox_call(uint64_t seed, uint64_t n, int rounds, uint32_t out[4])
{
    uint32_t ctr[4] = { (uint32_t)n, (uint32_t)(n >> 32), 0u, 0u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    oracle_philox4x32(ctr, key, rounds, out);
}

/* Raw stream: out[4*i .. 4*i+3] = Philox(seed, first_counter + i). */
void oracle_philox_raw(uint64_t seed, uint64_t first_counter, uint64_t ncalls,
                       int rounds, uint32_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)ncalls; ++i)
        philox_call(seed, first_counter + (uint64_t)i, rounds, out + 4 * (size_t)i);
}

/* Keep threshold: an element is kept iff its 32-bit random word x satisfies
 * x < T with T = floor((1 - p) * 2^32), evaluated in IEEE double from the
 * float argument p.  T is returned as a 64-bit value because p = 0 gives
 * T = 2^32 (every element kept).  Returns 0 on success, -1 if p is outside
 * [0, 1) or NaN. */
int oracle_keep_threshold(float p, uint64_t *T)
{
    if (!(p >= 0.0f) || !(p < 1.0f)) return -1;
    double t = (1.0 - (double)p) * 4294967296.0;
    *T = (uint64_t)t; /* t >= 0: truncation is floor */
    return 0;
}

/* Mask geometry: the S x S score matrix of one (batch, head) is cut into T x T tiles of
 * 32 x 32 elements, T = ceil(S/32); a tile is 16 words of 64 bits. */
uint64_t oracle_mask_words(int B, int H, int S)
{
    uint64_t T = ((uint64_t)S + 31u) / 32u;
    return (uint64_t)B * (uint64_t)H * T * T * 16u;
}

/* Number of Philox calls one mask consumes: 64 lanes per group of 4 words. */
uint64_t oracle_mask_philox_calls(int B, int H, int S)
{
    uint64_t words = oracle_mask_words(B, H, S);
    return 64u * ((words + 3u) / 4u);
}

/* Keep-mask for a B x H x S x S score matrix (paper Sec. 6.1 / 7.2: one bit per element,
 * B*nH*SQ^2 bits when S is a multiple of 32).
 *
 * Layout (the paper does not fix one; this is the reading taken): word index
 *     w = (((b*H + h)*T + qt)*T + kt)*16 + e,   T = ceil(S/32), 0 <= e < 16;
 * bit l (LSB first, 0 <= l < 64) of word w is the element
 *     row  i = 32*qt + (l % 32),
 *     col  j = 32*kt + 8*(e / 4) + 4*(l / 32) + (e % 4).
 * This is the order in which a 64-lane wave of a CDNA matrix core holds a 32 x 32 fp32
 * accumulator tile (lane l, register e), so a mask word is directly a per-lane predicate for
 * one accumulator register.  Bits whose row or column is >= S are 0.  Bit = 1 means keep.
 *
 * Random words: words are taken in groups of four, g = w / 4, r = w % 4.  Lane l of group g
 * makes Philox call number n = offset + 64*g + l (mod 2^64) with `rounds` rounds; output word
 * r of that call decides bit l of mask word 4*g + r.  `offset` counts Philox calls.
 *
 * Returns 0, or -1 for invalid arguments (out untouched). */
int oracle_dropout_mask_rounds(uint64_t seed, uint64_t offset, int B, int H, int S,
                               float p, int rounds, uint64_t *out)
{
    uint64_t Tkeep;
    if (B <= 0 || H <= 0 || S <= 0 || rounds <= 0 || out == NULL) return -1;
    if (oracle_keep_threshold(p, &Tkeep) != 0) return -1;
    const uint64_t T = ((uint64_t)S + 31u) / 32u;
    const uint64_t words = oracle_mask_words(B, H, S);
    const uint64_t groups = words / 4u;   /* words is a multiple of 16 */

#pragma omp parallel for schedule(static)
    for (int64_t gi = 0; gi < (int64_t)groups; ++gi) {
        const uint64_t g = (uint64_t)gi;
        uint64_t acc[4] = { 0, 0, 0, 0 };
        for (unsigned l = 0; l < 64; ++l) {
            uint32_t x[4];
            philox_call(seed, offset + 64u * g + l, rounds, x);
            for (unsigned r = 0; r < 4; ++r) {
                const uint64_t w = 4u * g + r;
                const uint64_t e = w % 16u;
                const uint64_t kt = (w / 16u) % T;
                const uint64_t qt = (w / (16u * T)) % T;
                const uint64_t i = 32u * qt + (l % 32u);                         /* row */
                const uint64_t j = 32u * kt + 8u * (e / 4u) + 4u * (l / 32u) + (e % 4u);   /* column */
                if (i < (uint64_t)S && j < (uint64_t)S && (uint64_t)x[r] < Tkeep)
                    acc[r] |= (uint64_t)1 << l;
            }
        }
        for (unsigned r = 0; r < 4; ++r) out[4u * g + r] = acc[r];
    }
    return 0;
}

int oracle_dropout_mask(uint64_t seed, uint64_t offset, int B, int H, int S,
                        float p, uint64_t *out)
{
    return oracle_dropout_mask_rounds(seed, offset, B, H, S, p, 10, out);
}

/* Narrow-threshold variants (the paper, Sec. 5.2, reduces the RNG cost by running fewer
 * rounds; spending fewer random bits per element is the other knob of the same trade-off and is
 * this build's addition, not the paper's): each 32-bit output word of a call is cut into
 * 32/bits fields of `bits` bits, field s = (x >> (bits*s)) & (2^bits - 1), and one field decides
 * one element: keep iff field < Tb with Tb = floor((1 - p) * 2^bits), in IEEE double from the
 * float p.  The kept probability is therefore quantised to Tb / 2^bits (230/256 for p = 0.1
 * and bits = 8).
 *
 * Words are taken in groups of E = 4 * 32/bits (16 for bits = 8, 8 for bits = 16, 4 for
 * bits = 32): g = w / E, e = w % E.  Lane l of group g makes call number offset + 64*g + l;
 * field s = e / 4 of output word r = e % 4 of that call decides bit l of mask word E*g + e.
 * bits = 32 is oracle_dropout_mask_rounds.  Layout of words and bits as above. */
int oracle_keep_threshold_bits(float p, int bits, uint64_t *T)
{
    if (!(p >= 0.0f) || !(p < 1.0f)) return -1;
    if (bits != 8 && bits != 16 && bits != 32) return -1;
    double t = (1.0 - (double)p) * (double)((uint64_t)1 << bits);
    *T = (uint64_t)t;
    return 0;
}

uint64_t oracle_mask_philox_calls_bits(int B, int H, int S, int bits)
{
    if (bits != 8 && bits != 16 && bits != 32) return 0;
    const uint64_t E = 4u * (32u / (unsigned)bits);
    uint64_t words = oracle_mask_words(B, H, S);
    return 64u * ((words + E - 1u) / E);
}

int oracle_dropout_mask_bits(uint64_t seed, uint64_t offset, int B, int H, int S,
                             float p, int rounds, int bits, uint64_t *out)
{
    uint64_t Tkeep;
    if (B <= 0 || H <= 0 || S <= 0 || rounds <= 0 || out == NULL) return -1;
    if (oracle_keep_threshold_bits(p, bits, &Tkeep) != 0) return -1;
    const uint64_t T = ((uint64_t)S + 31u) / 32u;
    const uint64_t words = oracle_mask_words(B, H, S);
    const uint64_t E = 4u * (32u / (unsigned)bits);
    const uint64_t fmask = bits == 32 ? 0xFFFFFFFFull : (((uint64_t)1 << bits) - 1u);
    const uint64_t groups = words / E;    /* words is a multiple of 16 */

#pragma omp parallel for schedule(static)
    for (int64_t gi = 0; gi < (int64_t)groups; ++gi) {
        const uint64_t g = (uint64_t)gi;
        uint64_t acc[16];
        memset(acc, 0, sizeof acc);
        for (unsigned l = 0; l < 64; ++l) {
            uint32_t x[4];
            philox_call(seed, offset + 64u * g + l, rounds, x);
            for (unsigned e = 0; e < E; ++e) {
                const unsigned r = e % 4u, s = e / 4u;
                const uint64_t field = ((uint64_t)x[r] >> ((unsigned)bits * s)) & fmask;
                const uint64_t w = E * g + e;
                const uint64_t ew = w % 16u;
                const uint64_t kt = (w / 16u) % T;
                const uint64_t qt = (w / (16u * T)) % T;
                const uint64_t i = 32u * qt + (l % 32u);
                const uint64_t j = 32u * kt + 8u * (ew / 4u) + 4u * (l / 32u) + (ew % 4u);
                if (i < (uint64_t)S && j < (uint64_t)S && field < Tkeep)
                    acc[e] |= (uint64_t)1 << l;
            }
        }
        for (unsigned e = 0; e < E; ++e) out[E * g + e] = acc[e];
    }
    return 0;
}

/* Number of set bits in a word array (kept-fraction tests and timing sink). */
uint64_t oracle_popcount_words(const uint64_t *w, uint64_t n)
{
    uint64_t total = 0;
#pragma omp parallel for reduction(+ : total) schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i)
        total += (uint64_t)__builtin_popcountll(w[i]);
    return total;
}

/* Number of threads the OpenMP loops above use (reported beside timings). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif

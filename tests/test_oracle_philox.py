"""Pins for the Philox / keep-mask oracle (CPU only).

Each test fixes the oracle to something other than itself: published
known-answer vectors, closed forms, invariants of the definition, or a second
evaluation with Python integers.
"""
import math
import os

import numpy as np
import pytest

from oracle import philox as P

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _kat_rows():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            t = line.split()
            rows.append((int(t[0]), [int(v, 16) for v in t[1:5]], [int(v, 16) for v in t[5:7]],
                         [int(v, 16) for v in t[7:11]]))
    return rows


@pytest.mark.parametrize("rounds,ctr,key,expect", _kat_rows())
def test_known_answer_vectors(rounds, ctr, key, expect):
    # Philox publication's known-answer set (cited by the paper, Sec. 2.3), R = 10 and R = 7.
    assert P.philox4x32(ctr, key, rounds) == expect
    assert P.philox4x32_py(ctr, key, rounds) == expect


def test_cxx26_engine_10000th_output():
    with open(os.path.join(GOLDEN, "philox_engine_10000th.txt")) as f:
        val = int([l for l in f if not l.startswith("#")][0])
    # raw stream with key = seed 20111115: call 2499, word 3
    raw = P.philox_raw(20111115, 0, 2500, 10)
    assert int(raw[2499, 3]) == val
    # and through the 64-bit counter split used by the mask: starting elsewhere gives the same call
    assert int(P.philox_raw(20111115, 2499, 1, 10)[0, 3]) == val


def test_round_function_is_a_bijection_step():
    # One round with zero key on counter (c0,c1,c2,c3): the outputs lo(p0), lo(p1) are odd-multiplier
    # products mod 2^32, hence invertible; recover c0 and c2 with the modular inverses.
    inv0 = pow(0xD2511F53, -1, 2**32)
    inv1 = pow(0xCD9E8D57, -1, 2**32)
    rng = np.random.default_rng(1)
    for _ in range(50):
        c = [int(v) for v in rng.integers(0, 2**32, size=4)]
        o = P.philox4x32(c, [0, 0], 1)
        assert (o[3] * inv0) % 2**32 == c[0]
        assert (o[1] * inv1) % 2**32 == c[2]
        assert o[0] == ((0xCD9E8D57 * c[2]) >> 32) ^ c[1]
        assert o[2] == ((0xD2511F53 * c[0]) >> 32) ^ c[3]


def test_key_schedule_matches_composition_of_single_rounds():
    # R rounds with key k == R single rounds with keys k + r*(W0, W1)
    rng = np.random.default_rng(2)
    W0, W1 = 0x9E3779B9, 0xBB67AE85
    for _ in range(20):
        c = [int(v) for v in rng.integers(0, 2**32, size=4)]
        k = [int(v) for v in rng.integers(0, 2**32, size=2)]
        x = c
        for r in range(10):
            x = P.philox4x32(x, [(k[0] + r * W0) % 2**32, (k[1] + r * W1) % 2**32], 1)
        assert x == P.philox4x32(c, k, 10)


def test_raw_stream_counter_and_key_split():
    seed = 0x0123456789ABCDEF
    first = 2**32 - 3          # crosses the 32-bit boundary: carry into the second counter word
    raw = P.philox_raw(seed, first, 8, 10)
    for i in range(8):
        n = first + i
        exp = P.philox4x32_py([n & 0xFFFFFFFF, n >> 32, 0, 0], [seed & 0xFFFFFFFF, seed >> 32], 10)
        assert [int(v) for v in raw[i]] == exp
    # wrap of the 64-bit call index
    raw = P.philox_raw(seed, 2**64 - 2, 4, 10)
    assert [int(v) for v in raw[2]] == P.philox4x32_py([0, 0, 0, 0], [seed & 0xFFFFFFFF, seed >> 32], 10)


def test_threshold_closed_forms():
    assert P.keep_threshold(0.1) == 0xE6666660
    assert P.keep_threshold(0.5) == 0x80000000
    assert P.keep_threshold(0.25) == 0xC0000000
    assert P.keep_threshold(0.0) == 2**32
    # exact rational floor for a spread of p (1 - p is exact in double for these)
    from fractions import Fraction
    for p in [0.1, 0.2, 0.3, 0.05, 0.9, 0.999, 1e-3, 0.7071]:
        pf = float(np.float32(p))
        assert P.keep_threshold(p) == int((1 - Fraction(pf)) * 2**32)
    for bad in [-0.1, 1.0, 1.5, float("nan")]:
        with pytest.raises(ValueError):
            P.keep_threshold(bad)


def test_mask_worked_example_tiny_config():
    # Tiny workload: B=1, H=2, S=128, p=0.1, seed=1234, offset=0.
    # Raw words for calls 0 and 1 (pinned through the KAT-checked block function):
    r0 = P.philox4x32_py([0, 0, 0, 0], [1234, 0])
    r1 = P.philox4x32_py([1, 0, 0, 0], [1234, 0])
    assert r0 == [0x2090B348, 0xDA7CF0AB, 0x4401906F, 0xCBCA470E]
    assert r1 == [0x9EEEDE35, 0x1CBE137C, 0xFA277093, 0x147EDD50]
    m = P.dropout_mask(1234, 0, 1, 2, 128, 0.1).reshape(-1)
    T = 0xE6666660
    for r in range(4):
        assert (int(m[r]) >> 0) & 1 == int(r0[r] < T)
        assert (int(m[r]) >> 1) & 1 == int(r1[r] < T)
    assert [(int(m[r]) >> 1) & 1 for r in range(4)] == [1, 1, 0, 1]   # 0xfa277093 >= T
    assert m.size == 1 * 2 * 128 * 2 and m.size * 64 == 32768


@pytest.mark.parametrize("B,H,S,p,seed,offset", [
    (1, 2, 128, 0.1, 1234, 0),
    (1, 1, 70, 0.3, 99, 5),             # ragged: S not a multiple of 32 (padding rows and columns)
    (2, 3, 33, 0.5, 2**40 + 7, 2**32 - 64),   # carry into the second counter word
    (1, 1, 1, 0.1, 1, 0),
])
def test_mask_c_matches_python_integers(B, H, S, p, seed, offset):
    a = P.dropout_mask(seed, offset, B, H, S, p)
    b = P.dropout_mask_py(seed, offset, B, H, S, p)
    assert np.array_equal(a, b)


def test_mask_equals_thresholded_raw_stream():
    # mask bit (w, l) == raw[offset + 64*(w>>2) + l][w & 3] < T, built with numpy from the raw stream
    B, H, S, p, seed, offset = 1, 3, 192, 0.1, 777, 12345      # S % 32 == 0: no padding bits
    words = B * H * (S // 32) ** 2 * 16
    raw = P.philox_raw(seed, offset, 64 * ((words + 3) // 4), 10).reshape(-1, 64, 4)   # [g, l, r]
    bits = (raw.astype(np.uint64) < P.keep_threshold(p)).transpose(0, 2, 1).reshape(-1, 64)[:words]  # [w, l]
    weights = (np.uint64(1) << np.arange(64, dtype=np.uint64))
    expect = (bits.astype(np.uint64) * weights).sum(axis=1, dtype=np.uint64)
    got = P.dropout_mask(seed, offset, B, H, S, p).reshape(-1)
    assert np.array_equal(got, expect)


def test_mask_padding_bits_are_zero_and_p0_keeps_all():
    S = 70                                   # 3 x 3 tiles of 32: rows / columns 70..95 are padding
    m = P.dropout_mask(5, 0, 1, 2, S, 0.0)
    keep = P.unpack_keep(m, 96)
    assert keep[..., :S, :S].all() and not keep[..., S:, :].any() and not keep[..., :, S:].any()
    assert P.popcount(m) == 2 * S * S
    m = P.dropout_mask(5, 0, 1, 2, S, 0.4)
    k2 = P.unpack_keep(m, 96)
    assert not k2[..., S:, :].any() and not k2[..., :, S:].any()


def test_mask_layout_element_to_word_bit_map():
    # element (i, j) of head h sits in tile (i/32, j/32), word e = 4*((j%32)/8) + (j%32)%4,
    # bit l = 32*(((j%32)/4)%2) + i%32 -- spelled out here independently of unpack_keep
    B, H, S, p = 1, 2, 100, 0.3
    m = P.dropout_mask(21, 9, B, H, S, p)
    keep = P.unpack_keep(m, S)
    rng = np.random.default_rng(0)
    for _ in range(500):
        h, i, j = int(rng.integers(H)), int(rng.integers(S)), int(rng.integers(S))
        jl = j % 32
        e = 4 * (jl // 8) + jl % 4
        l = 32 * ((jl // 4) % 2) + i % 32
        assert ((int(m[0, h, i // 32, j // 32, e]) >> l) & 1) == int(keep[0, h, i, j])
    # the raw-stream view of the same bit: word index w, group w//4, lane l, output word w%4
    T = 4
    raw = P.philox_raw(21, 9, 64 * (m.size // 4), 10)
    thr = P.keep_threshold(p)
    for _ in range(200):
        h, i, j = int(rng.integers(H)), int(rng.integers(S)), int(rng.integers(S))
        jl = j % 32
        e, l = 4 * (jl // 8) + jl % 4, 32 * ((jl // 4) % 2) + i % 32
        w = ((h * T + i // 32) * T + j // 32) * 16 + e
        assert bool(keep[0, h, i, j]) == (int(raw[64 * (w // 4) + l, w % 4]) < thr)
    # one row of tiles unpacks to the same 32 rows
    assert np.array_equal(P.unpack_keep_rows(m[0, 1, 2], S), keep[0, 1, 64:96])


def test_mask_reproducible_and_seed_offset_sensitive():
    a = P.dropout_mask(1234, 0, 1, 2, 128, 0.1)
    assert np.array_equal(a, P.dropout_mask(1234, 0, 1, 2, 128, 0.1))
    assert not np.array_equal(a, P.dropout_mask(1235, 0, 1, 2, 128, 0.1))
    assert not np.array_equal(a, P.dropout_mask(1234, 64, 1, 2, 128, 0.1))


def _four_sigma_ok(kept, n, q):
    return abs(kept / n - q) <= 4.0 * math.sqrt(q * (1 - q) / n)


@pytest.mark.parametrize("B,H,S,p", [(1, 2, 128, 0.1), (1, 8, 512, 0.1), (2, 4, 256, 0.5), (1, 4, 1024, 0.9)])
def test_kept_fraction_within_four_sigma(B, H, S, p):
    m = P.dropout_mask(1234, 0, B, H, S, p)
    q = P.keep_threshold(p) / 2**32
    assert _four_sigma_ok(P.popcount(m), B * H * S * S, q)
    for b in range(B):
        for h in range(H):
            assert _four_sigma_ok(P.popcount(m[b, h]), S * S, q)


def test_kept_fraction_at_second_workload_size():
    # 32 x 2048 x 2048 bits, the Llama-3-8B single-layer workload
    m = P.dropout_mask(1234, 0, 1, 32, 2048, 0.1)
    q = P.keep_threshold(0.1) / 2**32
    assert _four_sigma_ok(P.popcount(m), 32 * 2048 * 2048, q)


def test_offset_splitting():
    # a mask generated from word 4k on, with the offset advanced by 64k calls, is the tail of the full mask
    B, H, S, p = 1, 4, 128, 0.1
    full = P.dropout_mask(42, 1000, B, H, S, p).reshape(-1)
    # tail that starts at head 2: words = 2 heads * 16 tiles * 16 = 512 => k = 128 groups
    tail = P.dropout_mask(42, 1000 + 64 * 128, 1, 2, S, p).reshape(-1)
    assert np.array_equal(full[512:], tail)
    assert P.mask_philox_calls(B, H, S) == 64 * (B * H * 16 * 16 // 4)
    # consecutive masks with the offset advanced by mask_philox_calls never share a call:
    nxt = P.dropout_mask(42, 1000 + P.mask_philox_calls(B, H, S), B, H, S, p).reshape(-1)
    assert not np.array_equal(full, nxt)


def test_monotone_in_p():
    a = P.dropout_mask(7, 0, 1, 2, 256, 0.1).reshape(-1)
    b = P.dropout_mask(7, 0, 1, 2, 256, 0.3).reshape(-1)
    assert np.all((b & ~a) == 0)          # kept at p = 0.3  =>  kept at p = 0.1
    assert P.popcount(b) < P.popcount(a)


def test_lane_word_and_row_independence_smoke():
    B, H, S, p = 1, 8, 512, 0.5
    m = P.dropout_mask(3, 0, B, H, S, p)
    q = 0.5
    flat = m.reshape(-1)
    bits = np.unpackbits(flat.view(np.uint8).reshape(-1, 8), axis=1, bitorder="little")   # [word, lane]
    n_per_lane = bits.shape[0]
    lane_freq = bits.sum(axis=0) / n_per_lane
    assert np.all(np.abs(lane_freq - q) <= 4.5 * math.sqrt(q * (1 - q) / n_per_lane))
    for r in range(4):                                          # frequency per word slot r = w & 3
        sub = flat[r::4]
        assert _four_sigma_ok(P.popcount(sub), sub.size * 64, q)
    rows = P.unpack_keep(m, S).reshape(-1, S)
    assert abs(rows.mean() - q) <= 4 * math.sqrt(q * (1 - q) / rows.size)
    x = np.logical_xor(rows[:-1], rows[1:]).mean()
    assert abs(x - 2 * q * (1 - q)) < 4 * math.sqrt(0.25 / rows[:-1].size)


def test_mask_invalid_arguments():
    for args in [(0, 1, 8, 0.1), (1, 0, 8, 0.1), (1, 1, 0, 0.1), (1, 1, 8, 1.0), (1, 1, 8, -0.5)]:
        with pytest.raises(ValueError):
            P.dropout_mask(1, 0, *args)


def test_rounds_variants_differ_and_match_python():
    for R in (3, 5, 7, 10):
        a = P.dropout_mask(11, 3, 1, 1, 64, 0.2, rounds=R)
        assert np.array_equal(a, P.dropout_mask_py(11, 3, 1, 1, 64, 0.2, rounds=R))
    assert not np.array_equal(P.dropout_mask(11, 3, 1, 1, 64, 0.2, rounds=7),
                              P.dropout_mask(11, 3, 1, 1, 64, 0.2, rounds=10))


# ---------------------------------------------------------------------------
# Narrow-threshold variants: 8 or 16 random bits per element
# ---------------------------------------------------------------------------
def test_bits_threshold_closed_forms():
    from fractions import Fraction
    assert P.keep_threshold_bits(0.1, 8) == 230           # 0.9 * 256 = 230.4
    assert P.keep_threshold_bits(0.1, 16) == 58982        # 0.9 * 65536 = 58982.4
    assert P.keep_threshold_bits(0.5, 8) == 128 and P.keep_threshold_bits(0.5, 16) == 32768
    assert P.keep_threshold_bits(0.0, 8) == 256 and P.keep_threshold_bits(0.0, 16) == 65536
    for bits in (8, 16, 32):
        for p in [0.1, 0.2, 0.3, 0.05, 0.9, 0.999, 1e-3, 0.7071]:
            pf = float(np.float32(p))
            assert P.keep_threshold_bits(p, bits) == int((1 - Fraction(pf)) * 2**bits)
        assert P.keep_threshold_bits(0.3, 32) == P.keep_threshold(0.3)
    for bad in [(0.1, 4), (0.1, 12), (0.1, 64), (1.0, 8), (-0.1, 16)]:
        with pytest.raises(ValueError):
            P.keep_threshold_bits(*bad)


def test_bits_32_is_the_plain_mask():
    for args in [(1234, 0, 1, 2, 128, 0.1), (9, 2**32 - 64, 2, 1, 70, 0.4)]:
        assert np.array_equal(P.dropout_mask_bits(*args, 32), P.dropout_mask(*args))
        assert P.mask_philox_calls_bits(*args[2:5], 32) == P.mask_philox_calls(*args[2:5])


def test_bits_worked_example_from_pinned_raw_words():
    # calls 0 and 1 under seed 1234 (pinned above through the known-answer-checked block function):
    #   call 0 -> 2090b348 da7cf0ab 4401906f cbca470e,  call 1 -> 9eeede35 1cbe137c fa277093 147edd50
    # 8 bits: field s of word r is byte s; T8(0.1) = 230 = 0xe6.  Lane 1, r = 0: bytes 35 de ee 9e ->
    # kept, kept, DROPPED (0xee >= 0xe6), kept: bit 1 of mask words 0, 4, 8, 12.
    m8 = P.dropout_mask_bits(1234, 0, 1, 2, 128, 0.1, 8).reshape(-1)
    assert [(int(m8[4 * s]) >> 1) & 1 for s in range(4)] == [1, 1, 0, 1]
    # lane 0, r = 3: cbca470e -> bytes 0e 47 ca cb, all below 0xe6; r = 1: da7cf0ab -> ab f0 7c da: f0 dropped
    assert [(int(m8[4 * s + 3]) >> 0) & 1 for s in range(4)] == [1, 1, 1, 1]
    assert [(int(m8[4 * s + 1]) >> 0) & 1 for s in range(4)] == [1, 0, 1, 1]
    # 16 bits: T16(0.1) = 58982 = 0xe666.  Lane 1, r = 2: fa277093 -> halves 7093 (kept), fa27 (dropped)
    m16 = P.dropout_mask_bits(1234, 0, 1, 2, 128, 0.1, 16).reshape(-1)
    assert [(int(m16[4 * s + 2]) >> 1) & 1 for s in range(2)] == [1, 0]
    # lane 0, r = 1: da7cf0ab -> f0ab dropped (>= e666), da7c kept
    assert [(int(m16[4 * s + 1]) >> 0) & 1 for s in range(2)] == [0, 1]


@pytest.mark.parametrize("bits", [8, 16])
@pytest.mark.parametrize("B,H,S,p,seed,offset", [
    (1, 2, 128, 0.1, 1234, 0),
    (1, 1, 70, 0.3, 99, 5),
    (2, 3, 33, 0.5, 2**40 + 7, 2**32 - 64),
    (1, 1, 1, 0.1, 1, 0),
])
def test_bits_c_matches_python_integers(bits, B, H, S, p, seed, offset):
    a = P.dropout_mask_bits(seed, offset, B, H, S, p, bits)
    b = P.dropout_mask_py(seed, offset, B, H, S, p, bits=bits)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("bits", [8, 16])
def test_bits_mask_equals_thresholded_fields_of_raw_stream(bits):
    # built with numpy from the (separately pinned) raw stream: word E*g + 4*s + r, bit l
    #   == field s of raw[offset + 64*g + l][r] < Tb
    B, H, S, p, seed, offset = 1, 3, 192, 0.1, 777, 12345
    nf = 32 // bits
    E = 4 * nf
    words = B * H * (S // 32) ** 2 * 16
    raw = P.philox_raw(seed, offset, 64 * (words // E), 10).reshape(-1, 64, 4).astype(np.uint64)   # [g, l, r]
    fields = np.stack([(raw >> np.uint64(bits * s)) & np.uint64(2**bits - 1) for s in range(nf)], axis=1)  # [g, s, l, r]
    keep = fields < np.uint64(P.keep_threshold_bits(p, bits))
    keep = keep.transpose(0, 1, 3, 2).reshape(-1, 64)                                                # [(g, s, r), l]
    weights = (np.uint64(1) << np.arange(64, dtype=np.uint64))
    expect = (keep.astype(np.uint64) * weights).sum(axis=1, dtype=np.uint64)
    got = P.dropout_mask_bits(seed, offset, B, H, S, p, bits).reshape(-1)
    assert np.array_equal(got, expect)
    assert P.mask_philox_calls_bits(B, H, S, bits) == 64 * (words // E)


@pytest.mark.parametrize("bits", [8, 16])
def test_bits_kept_fraction_within_four_sigma_of_quantised_probability(bits):
    # the kept probability is Tb / 2^bits, not 1 - p: 230/256 = 0.8984 for 8 bits at p = 0.1
    B, H, S, p = 1, 8, 512, 0.1
    m = P.dropout_mask_bits(1234, 0, B, H, S, p, bits)
    q = P.keep_threshold_bits(p, bits) / 2**bits
    assert _four_sigma_ok(P.popcount(m), B * H * S * S, q)
    if bits == 8:   # and it is measurably not 1 - p at this size (the reason 32 bits is the default)
        assert not _four_sigma_ok(P.popcount(m), B * H * S * S, 0.9)
    for s_field in range(32 // bits):                      # every field position on its own
        sub = m.reshape(-1, 4 * (32 // bits))[:, 4 * s_field:4 * s_field + 4]
        assert _four_sigma_ok(P.popcount(sub), sub.size * 64, q)


@pytest.mark.parametrize("bits", [8, 16])
def test_bits_padding_monotone_and_offset_splitting(bits):
    S = 70
    m = P.dropout_mask_bits(5, 0, 1, 2, S, 0.0, bits)
    assert P.popcount(m) == 2 * S * S                      # p = 0 keeps exactly the in-range elements
    a = P.dropout_mask_bits(7, 0, 1, 2, 256, 0.1, bits).reshape(-1)
    b = P.dropout_mask_bits(7, 0, 1, 2, 256, 0.3, bits).reshape(-1)
    assert np.all((b & ~a) == 0) and P.popcount(b) < P.popcount(a)
    full = P.dropout_mask_bits(42, 1000, 1, 4, 128, 0.1, bits).reshape(-1)
    E = 4 * (32 // bits)
    tail = P.dropout_mask_bits(42, 1000 + 64 * (512 // E), 1, 2, 128, 0.1, bits).reshape(-1)
    assert np.array_equal(full[512:], tail)

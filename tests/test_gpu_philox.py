"""GPU parity: Philox words and keep-masks from the HIP kernels vs the CPU oracle, bit for bit."""
import ctypes

import numpy as np
import pytest

from oracle import philox as OP
from paper_2410_07531_amd import binding as rov
from paper_2410_07531_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _np_u32(t):
    return t.cpu().numpy().view(np.uint32)


def _np_u64(t):
    return t.cpu().numpy().view(np.uint64)


@pytest.mark.parametrize("rounds", [10, 7, 5, 3, 1, 16])
@pytest.mark.parametrize("seed,first,n", [
    (1234, 0, 1000),
    (0x0123456789ABCDEF, 2**32 - 300, 700),      # carry into the second counter word
    (2**64 - 1, 2**64 - 5, 64),                  # wrap of the 64-bit call index
])
def test_raw_words_bit_exact(rounds, seed, first, n):
    print("raw", rounds, seed, first, n, flush=True)
    got = _np_u32(rov.philox_raw(seed, first, n, rounds))
    assert np.array_equal(got, OP.philox_raw(seed, first, n, rounds))


def test_raw_known_answer_on_device():
    got = _np_u32(rov.philox_raw(0, 0, 1, 10))[0]
    assert [int(v) for v in got] == [0x6627E8D5, 0xE169C58D, 0xBC57AC4C, 0x9B00DBD8]


MASK_CASES = [
    # B, H, S, p, seed, offset
    (1, 2, 128, 0.1, wl.SEED, wl.OFFSET),                 # tiny workload
    (1, 2, 128, 0.1, wl.SEED, wl.CARRY_OFFSET),
    (1, 1, 1, 0.1, 1, 0),                                  # one bit
    (1, 1, 63, 0.5, 2, 7),                                 # ragged: S < 64
    (2, 3, 70, 0.3, 99, 5),                                # ragged rows, words not a multiple of 64
    (1, 5, 200, 0.25, 2**40 + 7, 2**32 - 64 * 16 - 3),     # ragged + carry inside a chunk
    (1, 3, 192, 0.0, 3, 0),                                # p = 0 keeps everything
    (1, 2, 256, 0.999, 4, 1),
    (1, 8, 512, 0.1, wl.SEED, 2**64 - 640),                # 64-bit wrap of the call index
    (2, 4, 1024, 0.1, wl.SEED, wl.OFFSET),                 # several chunks per wave, many blocks
]


@pytest.mark.parametrize("B,H,S,p,seed,offset", MASK_CASES)
def test_mask_bit_exact(B, H, S, p, seed, offset):
    print("mask", B, H, S, p, seed, offset, flush=True)
    got = _np_u64(rov.dropout_mask_generate(seed, offset, B, H, S, p))
    exp = OP.dropout_mask(seed, offset, B, H, S, p)
    assert got.shape == exp.shape
    assert np.array_equal(got, exp)


@pytest.mark.parametrize("rounds", [3, 5, 7])
def test_mask_round_variants_bit_exact(rounds):
    got = _np_u64(rov.dropout_mask_generate(11, 3, 1, 3, 200, 0.2, rounds=rounds))
    assert np.array_equal(got, OP.dropout_mask(11, 3, 1, 3, 200, 0.2, rounds=rounds))


def test_mask_small_grid_matches_default_grid():
    # the result must not depend on the launch shape
    a = _np_u64(rov.dropout_mask_generate(5, 0, 1, 8, 512, 0.1))
    prev = rov.set_rng_max_workgroups(3)
    try:
        b = _np_u64(rov.dropout_mask_generate(5, 0, 1, 8, 512, 0.1))
    finally:
        rov.set_rng_max_workgroups(prev)
    assert np.array_equal(a, b)


def test_mask_llama8b_s2k_full_and_carry():
    # second workload in full: 32 x 2048 x 2048 bits
    c = wl.CONFIGS[1]
    for offset in (wl.OFFSET, wl.CARRY_OFFSET):
        print("mask cfg2 offset", offset, flush=True)
        got = _np_u64(rov.dropout_mask_generate(wl.SEED, offset, c["B"], c["H"], c["S"], c["p"]))
        assert np.array_equal(got, OP.dropout_mask(wl.SEED, offset, c["B"], c["H"], c["S"], c["p"]))


def test_mask_largest_workload_sampled_and_counted():
    # 1 x 32 x 16384^2 bits (1 GiB): compare sampled slices with the oracle and the kept
    # fraction with its 4-sigma band
    import math
    import torch
    c = wl.CONFIGS[4]
    B, H, S, p = c["B"], c["H"], c["S"], c["p"]
    print("mask cfg5", flush=True)
    m = rov.dropout_mask_generate(wl.SEED, wl.OFFSET, B, H, S, p)
    T = S // 32
    words_per_head = T * T * 16
    for h in (0, 13, 31):
        # head h alone is the mask tail starting at word h*words_per_head (offset splitting)
        exp = OP.dropout_mask(wl.SEED, wl.OFFSET + 64 * (h * words_per_head // 4), 1, 1, S, p)
        assert np.array_equal(_np_u64(m[0, h]), exp[0, 0])
    # population count on the device copy, in slices (plumbing only)
    kept = 0
    flat = m.view(-1)
    step = 1 << 24
    for i in range(0, flat.numel(), step):
        chunk = flat[i:i + step].cpu().numpy().view(np.uint64)
        kept += OP.popcount(chunk)
    n = B * H * S * S
    q = OP.keep_threshold(p) / 2**32
    assert abs(kept / n - q) <= 4 * math.sqrt(q * (1 - q) / n)
    del m
    torch.cuda.empty_cache()


@pytest.mark.parametrize("B,H,S,cap", [(1, 2, 256, 0), (2, 3, 200, 0), (1, 1, 32, 0), (1, 2, 1024, 0),
                                        # power-of-two tile rows with a grid that strides many times over the chunks:
                                        # the launch shortens the grid so that a wave's chunks do not all sit at one
                                        # key-tile position (48 workgroups: stride 192 = 12 rows of 16 chunks)
                                        (1, 2, 2048, 48), (1, 3, 4096, 200), (2, 1, 2048, 0),
                                        # tile rows that are no power of two (T = 125, 500): the index arithmetic's
                                        # reciprocal division, with and without a capped grid
                                        (1, 2, 4000, 100), (1, 1, 16000, 0)])
def test_mask_causal_variant_writes_what_causal_attention_reads(B, H, S, cap):
    import torch
    p, seed, offset = 0.1, 7, 12345
    poison = 0x2AAAAAAAAAAAAAAA
    out = torch.full(rov.mask_shape(B, H, S), poison, dtype=torch.int64, device="cuda")
    prev = rov.set_rng_max_workgroups(cap)
    try:
        rov.dropout_mask_generate_causal(seed, offset, B, H, S, p, out)
        torch.cuda.synchronize()
    finally:
        rov.set_rng_max_workgroups(prev)
    got = _np_u64(out)
    exp = OP.dropout_mask(seed, offset, B, H, S, p)
    T = (S + 31) // 32
    qt, kt = np.meshgrid(np.arange(T), np.arange(T), indexing="ij")
    lower = kt <= qt
    assert np.array_equal(got[:, :, lower], exp[:, :, lower])            # every needed tile, same bits
    upper = got[:, :, ~lower]
    untouched = (upper == np.uint64(poison)).all(axis=-1)
    same = (upper == exp[:, :, ~lower]).all(axis=-1)
    assert np.all(untouched | same)                                       # the rest: untouched or the same bits
    if T >= 16:
        assert untouched.mean() > 0.6                                     # and most of it is really skipped


def test_mask_error_paths_leave_output_untouched():
    import torch
    out = torch.full(rov.mask_shape(1, 1, 64), 0x5A5A5A5A, dtype=torch.int64, device="cuda")
    L = rov.load()
    ptr = ctypes.c_void_p(out.data_ptr())
    s = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert L.rov_dropout_mask_generate(1, 0, 1, 1, 64, 1.0, ptr, s) == rov.ERR_INVALID
    assert L.rov_dropout_mask_generate(1, 0, 1, 1, 64, -0.1, ptr, s) == rov.ERR_INVALID
    assert L.rov_dropout_mask_generate(1, 0, 1, 1, 64, float("nan"), ptr, s) == rov.ERR_INVALID
    assert L.rov_dropout_mask_generate(1, 0, 0, 1, 64, 0.1, ptr, s) == rov.ERR_INVALID
    assert L.rov_dropout_mask_generate(1, 0, 1, 1, 0, 0.1, ptr, s) == rov.ERR_INVALID
    assert L.rov_dropout_mask_generate(1, 0, 1, 1, 64, 0.1, ctypes.c_void_p(0), s) == rov.ERR_INVALID
    assert L.rov_dropout_mask_generate(1, 0, 1, 1, 64, 0.1, ctypes.c_void_p(out.data_ptr() + 4), s) == rov.ERR_INVALID
    assert L.rov_dropout_mask_generate_rounds(1, 0, 1, 1, 64, 0.1, 4, ptr, s) == rov.ERR_INVALID
    assert L.rov_philox_raw(1, 0, 4, 0, ptr, s) == rov.ERR_INVALID
    assert L.rov_philox_raw(1, 0, 0, 10, ctypes.c_void_p(0), s) == rov.OK
    torch.cuda.synchronize()
    assert bool((out == 0x5A5A5A5A).all())


@pytest.mark.parametrize("bits", [8, 16, 32])
@pytest.mark.parametrize("B,H,S,p,seed,offset", MASK_CASES + [
    (1, 2, 96, 0.9999, 6, 0),                              # 8 bits: threshold 0, nothing kept
    (1, 32, 2048, 0.1, wl.SEED, wl.OFFSET),                # the measured workload at full size
])
def test_mask_bits_bit_exact(bits, B, H, S, p, seed, offset):
    print("mask bits", bits, B, H, S, p, seed, offset, flush=True)
    got = _np_u64(rov.dropout_mask_generate_bits(seed, offset, B, H, S, p, bits))
    exp = OP.dropout_mask_bits(seed, offset, B, H, S, p, bits)
    assert np.array_equal(got, exp)
    assert rov.mask_philox_calls_bits(B, H, S, bits) == OP.mask_philox_calls_bits(B, H, S, bits)


def test_mask_bits_rejects_other_widths():
    import torch
    out = torch.zeros(rov.mask_shape(1, 1, 32), dtype=torch.int64, device="cuda")
    for bits in (0, 4, 12, 24, 64):
        with pytest.raises(RuntimeError):
            rov.dropout_mask_generate_bits(1, 0, 1, 1, 32, 0.1, bits, out=out)
        assert rov.mask_philox_calls_bits(1, 1, 32, bits) == 0
    assert int(out.abs().sum()) == 0                        # nothing was written

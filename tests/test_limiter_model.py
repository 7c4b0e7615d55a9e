"""The limiter model (paper Sec. 3): composition rules, scaling laws and limiting cases.

These are properties the paper states for its model (Sec. 3.3 composition, Sec. 4.2 scaling laws,
Sec. 4.1 regions, Sec. 5.2 fewer rounds), checked on the gfx950 instantiation; how close the model
is to this chip is reported by bench.py next to the measured times, not asserted here.
"""
import dataclasses

import pytest

from paper_2410_07531_amd import limiter_model as L

C = L.MI355X


def test_composition_rules():
    # Sec. 3.3: baseline = sum of kernels; fusion replaces RNG + attention by the fused kernel;
    # overlap hides the RNG behind the GEMMs when it fits
    out = L.compose(C, [100e-6, 50e-6], 20e-6, 40e-6, 55e-6)
    assert out["baseline"] == pytest.approx(150e-6 + 20e-6 + 40e-6)
    assert out["fusion"] == pytest.approx(150e-6 + 55e-6)
    assert out["rng_exposed"] == 0.0                                 # 20 / 0.35 = 57 us < 154.5 us
    assert out["overlap"] == pytest.approx(150e-6 * (1 + C.gemm_slowdown_beside_rng) + 2 * C.stream_hop_s + 40e-6)
    assert out["hidden_fraction"] == pytest.approx(1 - 150e-6 * C.gemm_slowdown_beside_rng / 20e-6)


def test_overlap_when_rng_outlasts_the_gemms():
    # Sec. 3.3: what is left of the RNG when the GEMMs end runs at full speed
    g, r = 100e-6, 200e-6
    out = L.compose(C, [g], r, 0.0, 0.0)
    g_co = g * (1 + C.gemm_slowdown_rng_throughout)                   # the RNG is there all along
    done = g_co * C.rng_rate_rng_throughout / r                      # fraction produced beside the GEMM
    assert out["rng_exposed"] == pytest.approx((1 - done) * r + C.launch_s)
    assert out["overlap"] == pytest.approx(g_co + out["rng_exposed"] + 2 * C.stream_hop_s)
    # never worse than doing nothing beside the GEMM, up to the fixed costs
    assert out["overlap"] <= out["baseline"] + g * C.gemm_slowdown_rng_throughout + C.launch_s + 2 * C.stream_hop_s
    # an RNG that only just outlasts the GEMMs is not charged more than all of itself
    edge = L.compose(C, [g], g * 1.04 * C.rng_rate_beside_gemm, 0.0, 0.0)
    assert 0.0 <= edge["rng_exposed"] <= edge["baseline"]
    # no GEMM at all: the whole RNG is exposed
    assert L.compose(C, [], r, 0.0, 0.0)["rng_exposed"] == pytest.approx(r + C.launch_s)


def test_scaling_laws():
    # Sec. 4.2: RNG ~ B nH SQ^2, attention ~ B nH dH SQ^2, GEMM ~ M N K (fixed costs removed)
    def body(t):
        return t - C.launch_s
    r1, r2 = L.t_rng(C, 1, 32, 2048)["time"], L.t_rng(C, 2, 32, 4096)["time"]
    assert body(r2) / body(r1) == pytest.approx(8.0, rel=1e-6)
    a1, a2 = L.t_attention(C, 1, 32, 2048, 128)["time"], L.t_attention(C, 1, 32, 4096, 128)["time"]
    assert body(a2) / body(a1) == pytest.approx(4.0, rel=1e-6)
    g1, g2 = L.t_gemm(C, 8192, 4096, 4096)["time"], L.t_gemm(C, 16384, 8192, 4096)["time"]
    assert body(g2) / body(g1) == pytest.approx(4.0, rel=1e-6)
    # the RNG reads nothing and writes one bit per element (Table 1; Sec. 7.2)
    assert L.t_rng(C, 1, 32, 2048)["hbm_write"] == pytest.approx(32 * 2048 * 2048 / 8 / C.hbm_bytes_per_s)
    assert L.t_rng(C, 1, 32, 2048)["calls"] == 32 * 2048 * 2048 / 4


def test_wave_quantisation_of_the_gemm():
    # 2048 x 14336: 448 tiles of 256 x 256 would take two rounds over 256 compute units, as long as
    # 512 tiles; the launch's width rule picks 224 columns (512 tiles, two rounds of 7/8 the work)
    assert L.gemm_tile_cols(C, 2048, 14336) == 224
    assert L.gemm_tile_cols(C, 2048, 6144) == 192 and L.gemm_tile_cols(C, 2048, 4096) == 128
    assert L.gemm_tile_cols(C, 8192, 8192) == 256 and L.gemm_tile_cols(C, 16384, 14336) == 256
    a = L.t_gemm(C, 2048, 14336, 4096)["mfma"]
    full = L.t_gemm(C, 2048, 16384, 4096)["mfma"]          # 512 tiles of 256 x 256: two full rounds
    assert 0.875 * full < a < full
    # one tile more than a whole number of rounds costs a whole round (no narrower width helps here)
    assert L.t_gemm(C, 8192 + 256, 8192, 4096)["mfma"] > L.t_gemm(C, 8192, 8192, 4096)["mfma"] * 1.03
    # fp8 runs on the double-rate instruction
    assert L.t_gemm(C, 8192, 8192, 8192, esz=1)["mfma"] < 0.55 * L.t_gemm(C, 8192, 8192, 8192)["mfma"]


def test_fewer_rounds_and_fewer_bits_are_cheaper():
    # Sec. 5.2: Philox-5 and Philox-3 cost 71 % and 43 % of Philox-7's multiplies; the kernel time
    # falls less than that because compares, ballots and lane writes stay
    c7, c5, c3 = (L.philox_cycles_per_call(C, r) for r in (7, 5, 3))
    assert c3 < c5 < c7 < L.philox_cycles_per_call(C, 10)
    assert (2 * 5 - 2) / (2 * 7 - 2) < c5 / c7 < 1.0
    assert (2 * 3 - 2) / (2 * 7 - 2) < c3 / c7 < c5 / c7
    t32, t16, t8 = (L.t_rng(C, 1, 32, 2048, 10, b)["time"] for b in (32, 16, 8))
    assert t8 < t16 < t32 and t8 > t32 / 4                            # the per-field work does not shrink


def test_attention_modes_ordering():
    # Sec. 6.2 / Sec. 1: dropping with stored bits costs a little, in-kernel RNG costs a lot
    n, m, f = (L.t_attention(C, 1, 32, 2048, 128, mode)["time"] for mode in ("none", "mask", "fused"))
    assert n < m < f
    assert (m - n) / n < 0.2
    assert f - n > 0.5 * (L.t_rng(C, 1, 32, 2048)["time"] - C.launch_s)   # most of the RNG stays exposed
    c = L.t_attention(C, 1, 32, 16384, 128, "mask", causal=True)["time"]
    assert 0.45 < c / L.t_attention(C, 1, 32, 16384, 128, "mask")["time"] < 0.6


def test_regions_follow_the_gemm_to_rng_ratio():
    # Sec. 4.1: wide models at short sequences hide all of the RNG (region 1); long sequences on a
    # narrow model leave most of it exposed (region 3); RNG ~ S^2 against GEMM ~ S in between
    assert L.region(C, 1, 32, 2048, 128, 4096, 14336) == 1
    assert L.region(C, 1, 32, 16384, 128, 4096, 14336) == 2
    assert L.region(C, 1, 32, 65536, 128, 4096, 14336) == 3
    assert L.region(C, 1, 64, 8192, 128, 8192, 28672) == 1
    r = [L.block(C, 1, S, 32, 8, 128, 4096, 14336)["rng_exposed"] for S in (2048, 8192, 16384, 32768, 65536)]
    assert all(x <= y for x, y in zip(r, r[1:]))


def test_block_speedup_is_bounded_by_the_rng_share():
    b = L.block(C, 1, 16384, 32, 8, 128, 4096, 14336)
    assert 1.0 < b["speedup_vs_baseline"] <= b["baseline"] / (b["baseline"] - b["rng"])
    # a chip whose RNG is free gains nothing from the overlap
    free = dataclasses.replace(C, cyc_mad64=0.0, cyc_xor3=0.0, cyc_simple=0.0, cyc_cmp_writelane=0.0,
                               hbm_bytes_per_s=1e18, launch_s=0.0, stream_hop_s=0.0, gemm_slowdown_beside_rng=0.0)
    assert L.block(free, 1, 4096, 32, 8, 128, 4096, 14336)["speedup_vs_baseline"] == pytest.approx(1.0, abs=1e-6)

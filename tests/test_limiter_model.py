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
    # overlap hides the RNG behind the GEMMs when it fits, and the GEMMs pay only while it runs
    out = L.compose(C, [100e-6, 50e-6], 20e-6, 40e-6, 55e-6)
    assert out["baseline"] == pytest.approx(150e-6 + 20e-6 + 40e-6)
    assert out["fusion"] == pytest.approx(150e-6 + 55e-6)
    assert out["rng_exposed"] == 0.0                                 # 20 / 0.44 = 45 us < 168 us
    s = C.gemm_slowdown_beside_rng
    cost = (20e-6 / C.rng_rate_beside_gemm) * s / (1 + s)            # GEMM time lost while the grid runs
    assert out["overlap"] == pytest.approx(150e-6 + cost + 2 * C.stream_hop_s + 40e-6)
    assert out["hidden_fraction"] == pytest.approx(1 - cost / 20e-6)


def test_overlap_when_rng_outlasts_the_gemms():
    # Sec. 3.3: what is left of the RNG when the GEMMs end runs at full speed
    g, r = 100e-6, 200e-6
    out = L.compose(C, [g], r, 0.0, 0.0)
    g_co = g * (1 + C.gemm_slowdown_beside_rng)                      # the RNG is there all along
    done = g_co * C.rng_rate_beside_gemm / r                         # fraction produced beside the GEMM
    assert out["rng_exposed"] == pytest.approx((1 - done) * r + C.launch_s)
    assert out["overlap"] == pytest.approx(g_co + out["rng_exposed"] + 2 * C.stream_hop_s)
    # never worse than doing nothing beside the GEMM, up to the fixed costs
    assert out["overlap"] <= out["baseline"] + g * C.gemm_slowdown_beside_rng + C.launch_s + 2 * C.stream_hop_s
    # the two branches meet where the grid finishes exactly with the GEMMs
    edge_r = g_co * C.rng_rate_beside_gemm
    lo, hi = L.compose(C, [g], edge_r * 0.999, 0.0, 0.0), L.compose(C, [g], edge_r * 1.001, 0.0, 0.0)
    assert abs(hi["overlap"] - lo["overlap"]) <= 2 * C.launch_s
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
    a = L.t_gemm(C, 2048, 14336, 4096)["issue"]
    full = L.t_gemm(C, 2048, 16384, 4096)["issue"]         # 512 tiles of 256 x 256: two full rounds
    assert 0.875 * full < a < full
    # one tile more than a whole number of rounds costs a whole round (no narrower width helps here)
    assert L.t_gemm(C, 8192 + 256, 8192, 4096)["issue"] > L.t_gemm(C, 8192, 8192, 4096)["issue"] * 1.03
    # fp8 runs on the double-rate instruction
    assert L.t_gemm(C, 8192, 8192, 8192, esz=1)["issue"] < 0.6 * L.t_gemm(C, 8192, 8192, 8192)["issue"]
    # the SwiGLU form is the two projections' work in one kernel
    two = 2 * L.t_gemm(C, 16384, 14336, 4096)["issue"]
    assert 0.9 * two < L.t_gemm(C, 16384, 14336, 4096, dual=True)["issue"] < 1.1 * two


def test_clock_follows_the_matrix_core_duty():
    # the power limit: the busier the matrix cores, the lower the clock; never above the nominal one
    assert L.clock_hz(C, 0.0) == C.f_valu_hz and L.clock_hz(C, 1.0) == pytest.approx(C.f_valu_hz - C.f_drop_per_mfma_duty_hz)
    assert L.clock_hz(C, 0.3) > L.clock_hz(C, 0.6) > L.clock_hz(C, 0.9)
    assert L.clock_hz(dataclasses.replace(C, f_valu_hz=3e9), 0.0) == C.f_max_hz
    # a GEMM runs at a lower clock than attention, attention at a lower one than the RNG kernel
    assert L.t_gemm(C, 8192, 8192, 8192)["clock_hz"] < L.t_attention(C, 1, 32, 8192, 128, "mask")["clock_hz"] < C.f_valu_hz


def test_model_stays_close_to_the_recorded_measurements():
    # the kernels and blocks of one bench.py run (see limiter_model.validation): every kernel within
    # 12 %, the blocks within 10 %, and the model is never slower than the silicon by more than 6 %
    for name, (model, measured) in L.validation().items():
        assert -0.12 <= model / measured - 1.0 <= 0.06, (name, model, measured)


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
                               launch_s=0.0, stream_hop_s=0.0, gemm_slowdown_beside_rng=0.0)
    fb = L.block(free, 1, 4096, 32, 8, 128, 4096, 14336)
    assert fb["speedup_vs_baseline"] == pytest.approx(fb["baseline"] / (fb["baseline"] - fb["rng"]), rel=1e-9)
    assert fb["rng"] < 1e-2 * fb["baseline"]          # what is left is the mask's write time

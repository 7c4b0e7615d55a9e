"""Limiter model of the three schedules on one MI355X (paper Sec. 3, Table 1 and Sec. 3.3).

The paper predicts each kernel's runtime as the maximum, over the hardware limiters of its
Table 1, of (operations needed / operations per second the limiter sustains), and composes the
kernels into the baseline, fusion and overlap schedules (Sec. 3.3).  This module re-instantiates
that model for gfx950 from COUNTS: what a kernel of this library issues per unit of work (matrix
instructions, LDS-DMA loads, VALU instructions by class, LDS and HBM bytes; read off the kernels'
ISA and checked against the SQ_INSTS_* counters) priced with properties of the chip that were
measured by microbenchmarks or counters that do not depend on the shape being predicted.  There is
no per-kernel efficiency factor.  It is an analysis tool: nothing on the kernel path imports it.

Chip properties used (`Chip`), with where each comes from:
  * issue cycles per wave64 instruction class (rov_valu_probe, 8 waves per SIMD);
  * matrix-instruction passes (16 cycles for MFMA 16x16x32 bf16, 32 for 32x32x16 bf16 and for the
    fp8 16x16x128: the published peak divided by the flops of one instruction);
  * the cycles a 16-byte-per-lane LDS-DMA load keeps its wave from issuing matrix instructions
    (18; loads aimed outside their buffer, zero operands, round-1 measurement);
  * the clock the chip holds: 2.21 GHz under VALU-only load and 0.62 GHz less per unit of
    matrix-core duty (the board's power limit; GRBM_GUI_ACTIVE / duration of the RNG kernel, the
    8192^3 GEMM and the fused attention kernel), never above 2.4 GHz;
  * that VALU and matrix instructions of the two waves of a SIMD do not overlap in the attention
    kernel (a VALU instruction takes 8.7 instead of 4.7 cycles while the other wave's MFMA runs):
    attention is priced as the SUM of its matrix and VALU issue time, against its LDS and HBM time;
  * HBM 8 TB/s peak, 3.3 TB/s for the write burst at the end of a round of GEMM tiles, LDS
    128 bytes per clock per compute unit, L2 -> LDS 26 TB/s for whole-line requests;
  * interference between co-resident kernels (Sec. 6.2), two numbers measured on the S = 2048 layer
    step (the calibration case) and used unchanged for every other shape: the GEMMs run 12 % slower
    with the three-waves-per-SIMD RNG grid beside them, and that grid produces 0.44 of the
    stand-alone kernel's rate; what is left when the GEMMs end runs at the stand-alone rate
    (Sec. 3.3).

What the max-over-limiters rule leaves out is the imperfect overlap between limiters that are
close to each other (in the GEMM: matrix issue and the L2 -> LDS stream are within 1 % of each
other): the model is 8-19 % fast on the GEMMs and within 6 % on the RNG and attention kernels (see
`validation` at the end of the module; the table is reproduced by bench.py beside live timings).
"""
from dataclasses import dataclass
from typing import Dict, Sequence, Tuple


@dataclass(frozen=True)
class Chip:
    """One MI355X (gfx950): 256 compute units of 4 SIMDs."""
    cus: int = 256
    f_max_hz: float = 2.4e9
    # clock under load: f = min(f_max, f_valu - f_drop_per_mfma_duty * duty), duty = share of a SIMD's
    # cycles in which its matrix core runs
    f_valu_hz: float = 2.21e9
    f_drop_per_mfma_duty_hz: float = 0.62e9
    # matrix instructions: cycles a SIMD's matrix core is busy with one of them
    cyc_mfma_16x16x32_bf16: float = 16.0
    cyc_mfma_32x32x16_bf16: float = 32.0
    cyc_mfma_16x16x128_fp8: float = 32.0
    cyc_lds_dma_issue: float = 18.0
    # VALU issue cycles per wave64 instruction (probe: ns per instruction per SIMD x 2.21 GHz)
    cyc_simple: float = 2.4          # add, xor, max, select, convert, full-rate fp32
    cyc_xor3: float = 3.9
    cyc_mad64: float = 5.3
    cyc_cmp_writelane: float = 2.9   # compare-to-ballot plus one lane write
    cyc_exp2: float = 9.6            # transcendental: quarter rate
    # memory
    hbm_bytes_per_s: float = 8.0e12
    hbm_write_burst_bytes_per_s: float = 3.3e12
    l2_to_lds_bytes_per_s: float = 26e12
    lds_bytes_per_clk_per_cu: float = 128.0
    # scalar keep-word loads of the mask-reading attention: cycles of their latency that the softmax
    # phase does not cover, per 64-key tile and wave (the two waves of a SIMD cover half of it)
    cyc_keep_word_stall: float = 300.0
    # interference (Sec. 6.2), calibrated on the S = 2048 layer step
    gemm_slowdown_beside_rng: float = 0.12
    rng_rate_beside_gemm: float = 0.44
    # fixed costs: kernel launch on a busy stream, and a cross-stream event hop (fork or join)
    launch_s: float = 4e-6
    stream_hop_s: float = 6e-6


MI355X = Chip()


def _simd_count(chip: Chip) -> int:
    return chip.cus * 4


def clock_hz(chip: Chip, mfma_duty: float) -> float:
    """Clock the chip holds at a given matrix-core duty (power limit)."""
    return min(chip.f_max_hz, chip.f_valu_hz - chip.f_drop_per_mfma_duty_hz * max(0.0, min(1.0, mfma_duty)))


# --------------------------------------------------------------------------- kernels
def philox_cycles_per_call(chip: Chip, rounds: int = 10, bits: int = 32) -> float:
    """VALU issue cycles one wave64 spends per Philox call, from the mask kernel's instruction mix:
    per round two 32x32->64 multiplies and two three-input xors (the first two rounds save two
    multiplies and use plain xors: the upper counter words are zero and one product is
    wave-uniform); per output field one compare-to-ballot and two lane writes (both halves of the
    64-bit ballot), plus a field extract when fields are narrower than a word."""
    mads = 2 * rounds - 2
    xors = 2 * rounds - 5
    simple = 4 + 1                                     # plain xors of the first rounds, counter add
    fields = 4 * (32 // bits)
    per_field = chip.cyc_cmp_writelane + chip.cyc_simple + (chip.cyc_simple if bits < 32 else 0.0)
    return mads * chip.cyc_mad64 + xors * chip.cyc_xor3 + simple * chip.cyc_simple + fields * per_field


def t_rng(chip: Chip, B: int, H: int, S: int, rounds: int = 10, bits: int = 32, causal: bool = False) -> Dict[str, float]:
    """Stand-alone RNG kernel (paper Table 1, RNG column: no reads, issue / ALU bound)."""
    T = (S + 31) // 32
    words = B * H * T * T * 16
    if causal:
        words = words * (T + 1) / (2 * T)              # tiles with key tile <= query tile
    calls = 64.0 * words / (4 * (32 // bits))
    valu = calls / 64.0 * philox_cycles_per_call(chip, rounds, bits) / (_simd_count(chip) * clock_hz(chip, 0.0))
    hbm = words * 8.0 / chip.hbm_bytes_per_s
    return {"valu": valu, "hbm_write": hbm, "time": max(valu, hbm) + chip.launch_s, "calls": calls}


def gemm_tile_cols(chip: Chip, M: int, N: int) -> int:
    """Tile width the library's launch picks: tiles are 256 x 32*nj, nj = 4..8; workgroups run in
    rounds of one per compute unit and a tile costs about nj + 1 units (its activation panel does
    not shrink with it); smallest rounds x (nj + 1) wins, the widest on ties."""
    tiles_m = -(-M // 256)
    best, cols = None, 256
    for nj in range(8, 3, -1):
        cost = -(-(tiles_m * -(-N // (32 * nj))) // chip.cus) * (nj + 1)
        if best is None or cost < best:
            best, cols = cost, 32 * nj
    return cols


def t_gemm(chip: Chip, M: int, N: int, K: int, esz: int = 2, dual: bool = False) -> Dict[str, float]:
    """GEMM (paper Table 1, GEMM column: MMA math first, L2 read bandwidth second), from the tile
    kernel's counts.  A workgroup (one wave per SIMD) walks K in slot-steps of 128 bytes per row;
    per slot-step a wave issues 2 * 8 * nj MFMA 16x16x32 (bf16; fp8: 8 * nj MFMA 16x16x128 of twice
    the length) and 8 + nj LDS-DMA loads, each of which blocks its issue for cyc_lds_dma_issue; the
    workgroup moves (256 + 32 nj) rows x 128 bytes from L2 to LDS.  Workgroups run in rounds of one
    per compute unit; a round ends with its output leaving the chip in one burst.
    dual: the SwiGLU form (gate and up projections in one tile of half the output width; N counts
    the output columns)."""
    if dual:
        tiles_m, cu = -(-M // 256), chip.cus
        t8, t4 = tiles_m * -(-N // 128), tiles_m * -(-N // 64)
        nj = 8 if -(-t8 // cu) * 3 <= -(-t4 // cu) * 2 else 4      # the launch's rule for the dual tile
        tiles, out_cols = (t8 if nj == 8 else t4), 16 * nj
    else:
        cols = gemm_tile_cols(chip, M, N)
        nj = cols // 32
        tiles, out_cols = -(-M // 256) * -(-N // cols), cols
    rounds = -(-tiles // chip.cus)                       # the last round of tiles may be partly empty
    steps = K * esz / 128.0
    mfma_cyc = (2 * 8 * nj * chip.cyc_mfma_16x16x32_bf16) if esz == 2 else (8 * nj * chip.cyc_mfma_16x16x128_fp8)
    issue_cyc = mfma_cyc + (8 + nj) * chip.cyc_lds_dma_issue
    f = clock_hz(chip, mfma_cyc / issue_cyc)
    issue = rounds * steps * issue_cyc / f
    l2 = rounds * steps * chip.cus * (256 + 32 * nj) * 128.0 / chip.l2_to_lds_bytes_per_s
    drain = rounds * chip.cus * 256 * out_cols * 2.0 / chip.hbm_write_burst_bytes_per_s
    hbm = ((M + N * (2 if dual else 1)) * K * esz + M * N * 2.0) / chip.hbm_bytes_per_s
    return {"mfma": rounds * steps * mfma_cyc / f, "issue": issue, "l2": l2, "hbm": hbm, "drain": drain,
            "clock_hz": f, "time": max(issue, l2, hbm) + drain + chip.launch_s}


def t_attention(chip: Chip, B: int, H: int, S: int, d: int, mode: str = "mask", causal: bool = False) -> Dict[str, float]:
    """Flash-attention forward (paper Table 1, attention column: the non-MMA work binds), from the
    d = 128 kernel's counts per 64-key tile and wave (32 query rows): 32 MFMA 32x32x16; 33 exp2, 32
    multiply-adds into the exponent, 32 adds into the row sum, 16 three-input maxima, 16 packs to
    bf16 and 12 others; mode "mask": 32 selects more and the uncovered part of the scalar keep-word
    loads' latency; mode "fused": 8 Philox calls per lane with a plain compare per element in place of
    ballot and lane writes.  Each wave reads the K and V tile (32 KB) from LDS."""
    tiles = float(B) * H * (S / 32.0) * (S / 64.0) * (0.5 + 0.5 / max(S // 256, 1) if causal else 1.0)
    scale = d / 128.0
    mfma = 32.0 * scale * chip.cyc_mfma_32x32x16_bf16
    valu = 33 * chip.cyc_exp2 + (32 + 32 + 16 + 16 + 12) * chip.cyc_simple
    stall = 0.0
    if mode == "mask":
        valu += 32 * chip.cyc_simple
        stall = chip.cyc_keep_word_stall / 2.0
    elif mode == "fused":
        valu += 8 * (philox_cycles_per_call(chip, 10, 32) - 4.0 * chip.cyc_cmp_writelane) + 32 * 2 * chip.cyc_simple
    per_tile = mfma + valu + stall                       # the two pipes do not overlap (see module text)
    f = clock_hz(chip, mfma / per_tile)
    simd = tiles * per_tile / (_simd_count(chip) * f)
    lds = tiles * 32768.0 * scale / (chip.cus * chip.lds_bytes_per_clk_per_cu * f)
    mask_bytes = tiles * 256.0 if mode == "mask" else 0.0
    hbm = (mask_bytes + 4.0 * B * S * H * d * 2.0) / chip.hbm_bytes_per_s
    return {"mfma": tiles * mfma / (_simd_count(chip) * f), "valu": tiles * valu / (_simd_count(chip) * f),
            "lds": lds, "hbm": hbm, "clock_hz": f, "time": max(simd, lds, hbm) + chip.launch_s}


# --------------------------------------------------------------------------- schedules (paper Sec. 3.3)
def compose(chip: Chip, gemm_times: Sequence[float], rng_time: float, attn_mask_time: float,
            attn_fused_time: float) -> Dict[str, float]:
    """baseline = sum(GEMM) + RNG + attention(mask); fusion = sum(GEMM) + attention(fused);
    overlap = the GEMMs slowed by the RNG grid beside them for as long as it runs, plus what is left
    of the RNG when they end, at full speed, + attention(mask)."""
    g = float(sum(gemm_times))
    baseline = g + rng_time + attn_mask_time
    fusion = g + attn_fused_time
    rng_co = rng_time / chip.rng_rate_beside_gemm        # time the small grid alone would need
    g_all = g * (1.0 + chip.gemm_slowdown_beside_rng)    # the GEMMs with the grid there all the time
    if rng_co <= g_all:
        # the grid finishes inside the GEMMs: they are slowed only while it runs
        region = g + rng_co * chip.gemm_slowdown_beside_rng / (1.0 + chip.gemm_slowdown_beside_rng)
        exposed = 0.0
    else:
        left = max(0.0, 1.0 - g_all / rng_co) if g > 0.0 else 1.0
        exposed = left * rng_time + chip.launch_s
        region = g_all + exposed
    overlap = region + 2.0 * chip.stream_hop_s + attn_mask_time
    return {"baseline": baseline, "fusion": fusion, "overlap": overlap, "rng_exposed": exposed,
            "hidden_fraction": 1.0 - (region - g) / rng_time if rng_time > 0 else 1.0,
            "speedup_vs_baseline": baseline / overlap, "speedup_vs_fusion": fusion / overlap}


def layer_step(chip: Chip, B: int, H: int, S: int, d: int, gemms: Sequence[Tuple[int, int, int]],
               esz: int = 2, causal: bool = False) -> Dict[str, float]:
    """One GEMM(s) + RNG + attention step (the paper's silicon experiment, Sec. 6.1)."""
    gt = [t_gemm(chip, *g, esz=esz)["time"] for g in gemms]
    r = t_rng(chip, B, H, S, causal=causal)["time"]
    am = t_attention(chip, B, H, S, d, "mask", causal)["time"]
    af = t_attention(chip, B, H, S, d, "fused", causal)["time"]
    out = compose(chip, gt, r, am, af)
    out.update({"gemm": sum(gt), "rng": r, "attention_mask": am, "attention_fused": af})
    return out


def block(chip: Chip, B: int, S: int, H: int, Hkv: int, d: int, hidden: int, ffn: int, causal: bool = False) -> Dict[str, float]:
    """Transformer block in the steady state of a layer stack (paper Sec. 1 / Sec. 4.1): the mask of a
    layer is generated beside the PROJ, FC1 (gate and up as one product) and FC2 GEMMs of the layer
    before and the QKV GEMM of its own."""
    T = B * S
    gt = [t_gemm(chip, T, (H + 2 * Hkv) * d, hidden)["time"], t_gemm(chip, T, hidden, H * d)["time"],
          t_gemm(chip, T, ffn, hidden, dual=True)["time"], t_gemm(chip, T, hidden, ffn)["time"]]
    # norms, RoPE and the two residual epilogues: HBM passes over [T, hidden]
    glue = 8.0 * T * (3 * hidden) / chip.hbm_bytes_per_s + 3 * chip.launch_s
    r = t_rng(chip, B, H, S, causal=causal)["time"]
    am = t_attention(chip, B, H, S, d, "mask", causal)["time"]
    af = t_attention(chip, B, H, S, d, "fused", causal)["time"]
    out = compose(chip, gt, r, am, af)
    for k in ("baseline", "fusion", "overlap"):
        out[k] += glue
    out.update({"gemm": sum(gt), "rng": r, "attention_mask": am, "attention_fused": af, "glue": glue,
                "speedup_vs_baseline": out["baseline"] / out["overlap"],
                "speedup_vs_fusion": out["fusion"] / out["overlap"]})
    return out


def region(chip: Chip, B: int, H: int, S: int, d: int, hidden: int, ffn: int) -> int:
    """The paper's three regions of its Fig. 4 (Sec. 4.1): 1 = the GEMMs hide all of the RNG,
    2 = part of it, 3 = the RNG dominates (more than half of it is left when the GEMMs end)."""
    b = block(chip, B, S, H, H, d, hidden, ffn)
    if b["rng_exposed"] == 0.0:
        return 1
    return 2 if b["rng_exposed"] < 0.5 * b["rng"] else 3


def validation(chip: Chip = MI355X) -> Dict[str, Tuple[float, float]]:
    """(model ms, measured ms) for the kernels and blocks measured on one box in one bench.py run
    (stand-alone kernels and the S = 16384 Llama-3-8B block).  None of these shapes entered a chip
    constant; the interference pair was calibrated on the S = 2048 layer step."""
    ms = 1e3
    b = block(chip, 1, 16384, 32, 8, 128, 4096, 14336)
    return {
        "rng 32x16384^2 bits": (t_rng(chip, 1, 32, 16384)["time"] * ms, 2.80),
        "rng 32x2048^2 bits": (t_rng(chip, 1, 32, 2048)["time"] * ms, 0.0495),
        "attention S=16384 none": (t_attention(chip, 1, 32, 16384, 128, "none")["time"] * ms, 3.72),
        "attention S=16384 mask": (t_attention(chip, 1, 32, 16384, 128, "mask")["time"] * ms, 4.40),
        "attention S=16384 fused": (t_attention(chip, 1, 32, 16384, 128, "fused")["time"] * ms, 7.05),
        "gemm 16384x6144x4096": (t_gemm(chip, 16384, 6144, 4096)["time"] * ms, 0.64),
        "gemm 16384x4096x4096": (t_gemm(chip, 16384, 4096, 4096)["time"] * ms, 0.455),
        "gemm swiglu 16384x14336x4096": (t_gemm(chip, 16384, 14336, 4096, dual=True)["time"] * ms, 2.67),
        "gemm 16384x4096x14336": (t_gemm(chip, 16384, 4096, 14336)["time"] * ms, 1.40),
        "gemm 2048x14336x4096": (t_gemm(chip, 2048, 14336, 4096)["time"] * ms, 0.185),
        "gemm fp8 8192x8192x8192": (t_gemm(chip, 8192, 8192, 8192, esz=1)["time"] * ms, 0.385),
        "block S=16384 sequential": (b["baseline"] * ms, 13.17),
        "block S=16384 fused": (b["fusion"] * ms, 12.73),
        "block S=16384 overlap": (b["overlap"] * ms, 10.85),
    }

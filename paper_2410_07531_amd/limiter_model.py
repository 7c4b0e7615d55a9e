"""Limiter model of the three schedules on one MI355X (paper Sec. 3, Table 1 and Sec. 3.3).

The paper predicts each kernel's runtime as the maximum, over the hardware limiters of its
Table 1, of (operations needed / operations per second the limiter sustains), and composes the
kernels into the baseline, fusion and overlap schedules (Sec. 3.3).  This module re-instantiates
that model for gfx950: the limiters are this chip's (matrix cores, VALU issue, transcendental
rate, LDS, L2-to-CU and HBM bandwidth), the per-kernel operation counts are those of this
library's own kernels, and the sustained rates are the ones measured on the box (the functions
that measured them are named beside each constant).  It is an analysis tool: nothing on the
kernel path imports it.

Two things differ from the paper's GH100 model and are stated where they enter:
  * the matrix cores of an MI355X running random data are limited by board power, not by issue
    rate, so the MFMA limiter is a sustained rate (measured), not clock x width;
  * the RNG kernel beside a GEMM is a small persistent grid (two workgroups per compute unit),
    so its concurrent rate is a measured fraction of its stand-alone rate, and what is left when
    the GEMMs end runs at the stand-alone rate (the paper's rule, Sec. 3.3).
"""
from dataclasses import dataclass
from typing import Dict, Sequence, Tuple


@dataclass(frozen=True)
class Chip:
    """Sustained limiter rates of one MI355X (gfx950), 256 compute units."""
    cus: int = 256
    # Matrix cores, bf16, fp32 accumulate.  Peak is 4 SIMD x 1024 flop/clk x 2.4 GHz x 256 CU =
    # 2.5 PFLOP/s; a register-only loop of MFMA 16x16x32 on N(0,1) data sustains 2.05 PFLOP/s under
    # the power limit (rov_valu_probe-style loop).  fp8 on the double-rate MFMA 16x16x128: peak 5.0,
    # the same loop on random e4m3 data 4.55 PFLOP/s.
    mfma_flops: float = 2.05e15
    mfma_flops_fp8: float = 4.55e15
    # What the GEMM kernel keeps of that once operands stream through L2 and LDS (power shared with
    # the memory system): measured 1.38-1.45 PFLOP/s (bf16) and 2.75-3.0 PFLOP/s (fp8) on 8192-class
    # shapes with the 256 x 256 tile.
    gemm_efficiency: float = 0.69
    gemm_efficiency_fp8: float = 0.64
    # VALU issue: cycles per wave64 instruction per SIMD at the VALU clock below, from rov_valu_probe
    # (8 waves per SIMD, ns per wave-instruction per SIMD: add 1.13, three-input xor 1.79, 32x32->64
    # multiply-add 2.32, compare + lane write 2.39).
    valu_clock_hz: float = 2.3e9
    cyc_simple: float = 2.6
    cyc_xor3: float = 4.1
    cyc_mad64: float = 5.3
    cyc_cmp_writelane: float = 5.5
    cyc_exp2: float = 10.4         # transcendental: quarter rate of a full-rate fp32 op
    cyc_fp32: float = 2.6          # full-rate fp32 (mul, add, fma, max, select, convert)
    # Attention: how much longer the kernel takes than its matrix-core time plus its VALU time (the two
    # pipes are fed by the same two waves per SIMD and overlap little; barriers and the K/V tile waits)
    attention_overhead: float = 1.05
    # Mask mode beyond its one select per element (fitted: scalar keep-word loads, their waits, and the
    # SGPR pressure of 64 live word halves): measured 4.6 ms against 3.8 ms without dropout at S = 16384
    attention_mask_overhead: float = 1.13
    # Memory
    hbm_bytes_per_s: float = 8.0e12
    l2_to_cu_bytes_per_s: float = 13e12      # all CUs streaming GEMM operand slabs (measured inside the GEMM)
    # Interference, measured on the layer step: GEMM beside the small RNG grid, and the small grid's
    # rate relative to the stand-alone RNG kernel (paper Sec. 6.2 reports 4 % and 50 % on GH100).
    gemm_slowdown_beside_rng: float = 0.03
    # the same two numbers when the RNG runs for the whole duration of the GEMMs (block at S = 16384:
    # GEMMs 5.12 -> 5.93 ms, RNG 3.1 -> 6.6 ms)
    gemm_slowdown_rng_throughout: float = 0.16
    rng_rate_rng_throughout: float = 0.47
    rng_rate_beside_gemm: float = 0.35
    # Fixed costs: kernel launch on a busy stream, and a cross-stream event hop (fork or join).
    launch_s: float = 4e-6
    stream_hop_s: float = 6e-6


MI355X = Chip()


def _simd_count(chip: Chip) -> int:
    return chip.cus * 4


# --------------------------------------------------------------------------- kernels
def philox_cycles_per_call(chip: Chip, rounds: int = 10, bits: int = 32) -> float:
    """VALU issue cycles one wave64 spends per Philox call *per mask bit group*, from the kernel's
    instruction mix: per round two 32x32->64 multiplies and two three-input xors (the first two
    rounds save two multiplies and use plain xors: the upper counter words are zero and one product
    is wave-uniform); per output field one compare-to-ballot and two lane writes (both halves of
    the 64-bit ballot), plus a field extract when fields are narrower than a word."""
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
    valu = calls / 64.0 * philox_cycles_per_call(chip, rounds, bits) / (_simd_count(chip) * chip.valu_clock_hz)
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


def t_gemm(chip: Chip, M: int, N: int, K: int, esz: int = 2) -> Dict[str, float]:
    """GEMM (paper Table 1, GEMM column: MMA math first, L2 read bandwidth second)."""
    cols = gemm_tile_cols(chip, M, N)
    nj = cols // 32
    tiles = -(-M // 256) * -(-N // cols)
    rounds = -(-tiles // chip.cus)                       # the last round of tiles may be partly empty
    rate = (chip.mfma_flops * chip.gemm_efficiency if esz == 2 else chip.mfma_flops_fp8 * chip.gemm_efficiency_fp8)
    # a round takes one tile's time on every compute unit; a narrower tile moves more bytes per flop
    mfma = rounds * chip.cus * (2.0 * 256 * cols * K) / rate * ((nj + 1) / nj) / (9.0 / 8.0)
    l2 = tiles * (K * esz / 128.0) * (256 + cols) * 128.0 / chip.l2_to_cu_bytes_per_s
    hbm = ((M + N) * K * esz + M * N * 2.0) / chip.hbm_bytes_per_s
    return {"mfma": mfma, "l2": l2, "hbm": hbm, "time": max(mfma, l2, hbm) + chip.launch_s}


def t_attention(chip: Chip, B: int, H: int, S: int, d: int, mode: str = "mask", causal: bool = False) -> Dict[str, float]:
    """Flash-attention forward (paper Table 1, attention column: the non-MMA work binds).
    mode: "none" (no dropout), "mask" (drops with stored bits), "fused" (Philox in the kernel)."""
    elems = float(B) * H * S * S * (0.5 + 0.5 / max(S // 256, 1) if causal else 1.0)
    mfma = 4.0 * elems * d / (chip.mfma_flops * 0.80)    # MFMA 32x32x16: 1.66 of 2.05 PFLOP/s sustained
    # VALU instructions per score element, from the d = 128 kernel's loop (141 per 64-key tile and
    # lane-row of 32 elements): multiply-add into the exponent, exp2, sum, half a max3, half a pack
    # to bf16, and 0.4 of bookkeeping; the rescale of the output accumulator runs only while the
    # running maximum still moves (first tiles) and is left out
    per_elem = 3.4 * chip.cyc_fp32 + chip.cyc_exp2
    if mode != "none":
        per_elem += chip.cyc_fp32                        # one select per element
    if mode == "fused":
        # a quarter of a Philox call, with a plain compare in place of the ballot and lane writes
        per_elem += (philox_cycles_per_call(chip, 10, 32) - 4.0 * chip.cyc_cmp_writelane) / 4.0
    valu = elems / 64.0 * per_elem / (_simd_count(chip) * chip.valu_clock_hz)
    mask_bytes = elems / 8.0 if mode == "mask" else 0.0
    hbm = (mask_bytes + 4.0 * B * S * H * d * 2.0) / chip.hbm_bytes_per_s
    over = chip.attention_overhead * (chip.attention_mask_overhead if mode == "mask" else 1.0)
    return {"mfma": mfma, "valu": valu, "hbm": hbm,
            "time": max(over * (mfma + valu), hbm) + chip.launch_s}


# --------------------------------------------------------------------------- schedules (paper Sec. 3.3)
def compose(chip: Chip, gemm_times: Sequence[float], rng_time: float, attn_mask_time: float,
            attn_fused_time: float) -> Dict[str, float]:
    """baseline = sum(GEMM) + RNG + attention(mask); fusion = sum(GEMM) + attention(fused);
    overlap = (GEMMs slowed by the RNG beside them, or, if the RNG outlasts them, the GEMMs plus the
    rest of the RNG at full speed) + attention(mask)."""
    g = float(sum(gemm_times))
    baseline = g + rng_time + attn_mask_time
    fusion = g + attn_fused_time
    g_co = g * (1.0 + chip.gemm_slowdown_beside_rng)
    rng_co = rng_time / chip.rng_rate_beside_gemm        # time the small grid alone would need
    if rng_co <= g_co:
        region = g_co
        exposed = 0.0
    else:
        # the RNG is there for the whole of the GEMMs: they give up more of the (power-limited) clock
        # and the RNG gets more of the issue slots; what is left when they end runs at full rate
        g_co = g * (1.0 + chip.gemm_slowdown_rng_throughout)
        rng_co = rng_time / chip.rng_rate_rng_throughout
        left = max(0.0, 1.0 - g_co / rng_co)
        exposed = left * rng_time + chip.launch_s
        region = g_co + exposed
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
    """Transformer block in steady state (paper Sec. 1 / Sec. 4.1): the mask of a layer is generated
    beside the PROJ, FC1 (gate and up) and FC2 GEMMs of the layer before and the QKV GEMM of its own."""
    T = B * S
    shapes = [(T, (H + 2 * Hkv) * d, hidden), (T, hidden, H * d), (T, ffn, hidden), (T, ffn, hidden), (T, hidden, ffn)]
    gt = [t_gemm(chip, *g)["time"] for g in shapes]
    # norms, RoPE and the two residual epilogues: HBM passes over [T, hidden] (gate and up are one
    # product with the SwiGLU applied in its accumulators: no pass over [T, ffn])
    glue = 8.0 * T * (3 * hidden) / chip.hbm_bytes_per_s
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

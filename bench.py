#!/usr/bin/env python3
"""Benchmark of the RNG/GEMM-overlap hot path on one MI355X.

A "step" is one pass of the whole hot path on the Llama-3-8B-shaped single layer (B=1, H=32,
d=128, S=2048, p=0.1, bf16): the Philox4x32-10 keep-mask (32 x 2048 x 2048 bits) generated on
a side stream while the FFN-up GEMM (2048 x 4096 x 14336) runs, joined, then flash-attention
forward that drops with that mask (`rov_layer_step`, overlap schedule).  Inputs are synthetic
(seeded N(0,1) activations, N(0,0.02) weights) and already resident in HBM.

One JSON line is printed: whole-step mask throughput as `value`, the roofline of the dominant
kernel of the step (the GEMM, measured with HIP events inside the timed region through the
library's kernel trace), the CPU oracle timed on this machine's host cores on a bounded sample, and
the per-kernel / per-schedule numbers (stand-alone RNG Gbit/s and its VALU roofline, GEMM alone
vs beside the RNG, hidden fraction, sequential / fused / overlap step and block times).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0       # MI355X dense bf16 MFMA
PEAK_INT32_TOPS = 78.6          # 256 CU x 4 SIMD x 32 lanes/clk x 2.4 GHz (= fp32 FMA issue rate, 157.3 / 2)
INT32_OPS_PER_CALL = 84         # 20 wide multiplies (lo+hi = 2 results each), 40 two-input xors, 4 compares
# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch, scaled by what the
# same counters read for a 1 GiB copy: x2.00 and x1.00), see profiles/pmc_fetch_write_llama3_8b_s2k.md
TRAFFIC_GEMM_BYTES = int((195003.0 * 2.0 + 57362.6) * 1024)      # 2048x4096x14336 bf16 (algorithmic: 184.5 MiB)
TRAFFIC_RNG_BYTES = int((46.8 * 2.0 + 16384.0) * 1024)           # 32x2048x2048-bit mask (algorithmic: 16 MiB)
TRAFFIC_ATTN_MASK_BYTES = int((41047.4 * 2.0 + 16388.8) * 1024)  # attention reading the mask (algorithmic: 80 MiB)


def median_ms(fn, warm, iters, sync, ev_pair, inner=10):
    """Median over `iters` batches of the per-call time of `inner` back-to-back calls (HIP events on
    the current stream), so that launch latency after an idle queue is not billed to the kernel."""
    for _ in range(warm):
        fn()
    sync()
    ts = []
    for _ in range(iters):
        a, b = ev_pair()
        a.record()
        for _ in range(inner):
            fn()
        b.record()
        b.synchronize()
        ts.append(a.elapsed_time(b) / inner)
    return float(np.median(ts))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-block", action="store_true", help="skip the config-5 block timings")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--seq-sweep", action="store_true",
                    help="instead of the benchmark line: the Llama-3-8B block (non-causal) under the three schedules "
                         "at S = 2048 ... 32768 beside the limiter model's prediction and region, one JSON object")
    ap.add_argument("--kernels-only", action="store_true",
                    help="for profilers: launch a 1 GiB device copy (counter calibration), then the RNG, GEMM and "
                         "attention kernels of the workload alone and the overlap step, 5 times each; no JSON")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path has no cross-GPU step); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2410_07531_amd import binding as rov
    from paper_2410_07531_amd import workloads as wl

    rov.load()
    torch.cuda.set_device(0)
    dev = "cuda"
    sync = torch.cuda.synchronize
    main_s, side_s = torch.cuda.Stream(), torch.cuda.Stream()

    def ev_pair():
        return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    # ------------------------------------------------------------------ workload (configs[1])
    ci = 1
    c = wl.CONFIGS[ci]
    B, H, Hkv, S, d, p = c["B"], c["H"], c["Hkv"], c["S"], c["d"], c["p"]
    _, M, K, N = c["gemms"][0]
    rng = wl.rng_for(ci)
    q, k, v = wl.qkv(rng, B, S, H, Hkv, d)
    a, w = wl.gemm_operands(rng, M, K, N)
    bf = torch.bfloat16
    Q, Kt, V = [torch.from_numpy(x).to(bf).to(dev) for x in (q, k, v)]
    A, Wt = torch.from_numpy(a).to(bf).to(dev), torch.from_numpy(w).to(bf).to(dev)
    O = torch.empty_like(Q)
    C = torch.empty((M, N), dtype=bf, device=dev)
    mask = torch.empty(rov.mask_shape(B, H, S), dtype=torch.int64, device=dev)
    nbits = B * H * S * S
    ncalls = nbits // 4
    gemm_flops = 2.0 * M * N * K
    attn_flops = 4.0 * B * H * S * S * d
    gd = [rov.make_gemm_desc(A, Wt, C)]
    ad = rov.make_attn_desc(Q, Kt, V, O, p)

    def step(sched):
        rov.layer_step(sched, gd, ad, wl.SEED, wl.OFFSET, None if sched == rov.SCHED_FUSED else mask, main_s, side_s)

    if args.seq_sweep:
        from paper_2410_07531_amd import limiter_model as LM
        c5 = wl.CONFIGS[4]
        out = {}
        for S_ in (2048, 4096, 8192, 16384, 32768):
            print("seq-sweep: S =", S_, file=sys.stderr, flush=True)
            r = bench_block(torch, rov, wl, main_s, side_s, sync, ev_pair, seq_len=S_, causals=(False,), check=True)["noncausal"]
            bm = LM.block(LM.MI355X, c5["B"], S_, c5["H"], c5["Hkv"], c5["d"], c5["hidden"], c5["ffn"], False)
            r["limiter_model_ms"] = {"sequential": bm["baseline"] * 1e3, "fused": bm["fusion"] * 1e3,
                                     "overlap": bm["overlap"] * 1e3, "rng": bm["rng"] * 1e3,
                                     "rng_exposed": bm["rng_exposed"] * 1e3}
            r["limiter_model_region"] = LM.region(LM.MI355X, c5["B"], c5["H"], S_, c5["d"], c5["hidden"], c5["ffn"])
            out["S=%d" % S_] = r
        print(json.dumps({"seq_sweep_llama3_8b_block": out}))
        return

    if args.kernels_only:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        with torch.cuda.stream(main_s):
            for _ in range(5):
                dst.copy_(src)                                     # reads 1 GiB, writes 1 GiB
            for _ in range(5):
                rov.dropout_mask_generate(wl.SEED, 0, B, H, S, p, out=mask, stream=main_s)
            for _ in range(5):
                rov.gemm(A, Wt, C=C, stream=main_s)
            for _ in range(5):
                rov.attention_fwd_dropout(Q, Kt, V, p, mask=mask, O=O, stream=main_s)
            for _ in range(5):
                rov.attention_fwd_dropout(Q, Kt, V, p, seed=wl.SEED, offset=0, O=O, stream=main_s)
        for _ in range(5):
            step(rov.SCHED_OVERLAP)
        sync()
        print("kernels-only run done", file=sys.stderr)
        return

    # ------------------------------------------------------------------ timed region (overlap schedule)
    # Only the dominant kernel (the GEMM) carries timing events inside the timed region: two event
    # records per step on the stream it runs on.  The other kernels of the step are timed the same
    # way in a short pass of their own afterwards, so that their events do not slow the timed steps.
    for _ in range(args.warmup):
        step(rov.SCHED_OVERLAP)
    sync()
    rov.trace_enable(True, [rov.TRACE_GEMM])
    rov.trace_read()
    sync()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(rov.SCHED_OVERLAP)
    sync()
    t1 = time.perf_counter()
    rov.trace_enable(False)
    trace = rov.trace_read()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    gemm_in_step = float(np.mean([ms for kind, ms in trace if kind == rov.TRACE_GEMM]))
    rov.trace_enable(True)
    for _ in range(50):
        step(rov.SCHED_OVERLAP)
    sync()
    rov.trace_enable(False)
    by_kind = {}
    for kind, ms in rov.trace_read():
        by_kind.setdefault(kind, []).append(ms)
    rng_in_step = float(np.mean(by_kind[rov.TRACE_RNG]))
    rng_helper_in_step = float(np.mean(by_kind[rov.TRACE_RNG_HELPER])) if rov.TRACE_RNG_HELPER in by_kind else None
    attn_in_step = float(np.mean(by_kind[rov.TRACE_ATTENTION]))

    # ------------------------------------------------------------------ per-kernel and per-schedule numbers
    with torch.cuda.stream(main_s):
        t_rng = median_ms(lambda: rov.dropout_mask_generate(wl.SEED, 0, B, H, S, p, out=mask, stream=main_s),
                          5, 10, sync, ev_pair)
        t_gemm = median_ms(lambda: rov.gemm(A, Wt, C=C, stream=main_s), 5, 10, sync, ev_pair)
        t_attn_none = median_ms(lambda: rov.attention_fwd_dropout(Q, Kt, V, 0.0, O=O, stream=main_s), 3, 10, sync, ev_pair)
        t_attn_mask = median_ms(lambda: rov.attention_fwd_dropout(Q, Kt, V, p, mask=mask, O=O, stream=main_s),
                                3, 10, sync, ev_pair)
        t_attn_fused = median_ms(lambda: rov.attention_fwd_dropout(Q, Kt, V, p, seed=wl.SEED, offset=0, O=O,
                                                                  stream=main_s), 3, 10, sync, ev_pair)

        # the overlap schedule's first phase on its own: fork, GEMM || RNG (same small persistent RNG
        # grid as the library's overlap schedules use), join
        k_ovl = rov.set_rng_overlap_workgroups_per_cu(0)
        rov.set_rng_overlap_workgroups_per_cu(k_ovl)
        n_cu = torch.cuda.get_device_properties(0).multi_processor_count

        def gemm_beside_rng():
            fork = torch.cuda.Event()
            fork.record(main_s)
            side_s.wait_event(fork)
            rov.gemm(A, Wt, C=C, stream=main_s)
            rov.dropout_mask_generate(wl.SEED, 0, B, H, S, p, out=mask, stream=side_s)
            join = torch.cuda.Event()
            join.record(side_s)
            main_s.wait_event(join)

        rov.set_rng_max_workgroups(n_cu * k_ovl)
        t_pair = median_ms(gemm_beside_rng, 5, 10, sync, ev_pair)
        rov.set_rng_max_workgroups(0)
        # the same GEMM and mask from the wave-specialised single kernel (paper Sec. 6.1's other form)
        t_single = median_ms(lambda: rov.gemm_rng_fused(A, Wt, wl.SEED, 0, B, H, S, p, C=C, mask=mask, stream=main_s),
                             5, 10, sync, ev_pair)
        rov.set_rng_max_workgroups(0)
        t_seq = median_ms(lambda: step(rov.SCHED_SEQUENTIAL), 5, 10, sync, ev_pair)
        t_fus = median_ms(lambda: step(rov.SCHED_FUSED), 5, 10, sync, ev_pair)
        t_ovl = median_ms(lambda: step(rov.SCHED_OVERLAP), 5, 10, sync, ev_pair)

        def step_without_rng():   # the same GEMM and attention with the mask already in HBM
            rov.gemm(A, Wt, C=C, stream=main_s)
            rov.attention_fwd_dropout(Q, Kt, V, p, mask=mask, O=O, stream=main_s)

        t_norng = median_ms(step_without_rng, 5, 10, sync, ev_pair)
    # hidden fraction = 1 - (T[GEMM || RNG] - T[GEMM]) / T[RNG] on the fork / GEMM || RNG / join region;
    # the whole-step variant charges the RNG with everything the overlap step takes longer than the
    # same GEMM and attention run back to back without any RNG (clock and power effects included)
    hidden_region = 1.0 - (t_pair - t_gemm) / t_rng
    hidden = 1.0 - max(t_ovl - t_norng, 0.0) / t_rng
    gemm_slowdown = gemm_in_step / t_gemm - 1.0

    extras = {
        "rng_alone": {"ms": t_rng, "gbit_s": nbits / t_rng / 1e6, "gcalls_s": ncalls / t_rng / 1e6,
                      "roofline": {"bound": "alu", "achieved": ncalls * INT32_OPS_PER_CALL / t_rng / 1e9,
                                   "peak": PEAK_INT32_TOPS, "unit": "Tint32op/s",
                                   "frac": ncalls * INT32_OPS_PER_CALL / t_rng / 1e9 / PEAK_INT32_TOPS,
                                   "traffic": TRAFFIC_RNG_BYTES}},
        "gemm_alone": {"ms": t_gemm, "tflops": gemm_flops / t_gemm / 1e9,
                       "mfma_frac": gemm_flops / t_gemm / 1e9 / PEAK_BF16_TFLOPS},
        "gemm_in_overlap_step": {"ms": gemm_in_step, "tflops": gemm_flops / gemm_in_step / 1e9,
                                 "mfma_frac": gemm_flops / gemm_in_step / 1e9 / PEAK_BF16_TFLOPS,
                                 "slowdown_vs_alone": gemm_slowdown},
        "rng_in_overlap_step": {"ms": rng_in_step, "slowdown_vs_alone": rng_in_step / t_rng - 1.0,
                                "helper_launch_ms": rng_helper_in_step},
        "gemm_beside_rng_region_ms": t_pair,
        "gemm_and_rng_single_wave_specialised_kernel_ms": t_single,
        "rng_overlap_workgroups_per_cu": k_ovl,
        "rng_hidden_fraction": hidden_region,
        "rng_hidden_fraction_whole_step": hidden,
        "layer_step_without_rng_ms": t_norng,
        "attention": {"none_ms": t_attn_none, "mask_ms": t_attn_mask, "fused_ms": t_attn_fused,
                      "in_step_ms": attn_in_step,
                      "none_tflops": attn_flops / t_attn_none / 1e9, "mask_tflops": attn_flops / t_attn_mask / 1e9,
                      "fused_tflops": attn_flops / t_attn_fused / 1e9,
                      "dropping_overhead": t_attn_mask / t_attn_none - 1.0,
                      "mask_traffic_bytes": TRAFFIC_ATTN_MASK_BYTES},
        "layer_step_ms": {"sequential": t_seq, "fused": t_fus, "overlap": t_ovl},
        "layer_speedup_overlap_vs_sequential": t_seq / t_ovl,
        "layer_speedup_overlap_vs_fused": t_fus / t_ovl,
    }

    # ------------------------------------------------------------------ limiter model beside the measurements
    from paper_2410_07531_amd import limiter_model as LM
    lm = LM.layer_step(LM.MI355X, B, H, S, d, [(M, N, K)])
    extras["limiter_model_layer_step_ms"] = {
        "gemm": lm["gemm"] * 1e3, "rng": lm["rng"] * 1e3, "attention_mask": lm["attention_mask"] * 1e3,
        "attention_fused": lm["attention_fused"] * 1e3, "sequential": lm["baseline"] * 1e3,
        "fused": lm["fusion"] * 1e3, "overlap": lm["overlap"] * 1e3, "hidden_fraction": lm["hidden_fraction"]}

    # ------------------------------------------------------------------ transformer block (configs[4])
    if not args.no_block:
        del Q, Kt, V, O, A, Wt, C
        torch.cuda.empty_cache()
        extras["block_llama3_8b_s16k"] = bench_block(torch, rov, wl, main_s, side_s, sync, ev_pair)
        c5 = wl.CONFIGS[4]
        for causal in (False, True):
            bm = LM.block(LM.MI355X, c5["B"], c5["S"], c5["H"], c5["Hkv"], c5["d"], c5["hidden"], c5["ffn"], causal)
            extras["block_llama3_8b_s16k"]["causal" if causal else "noncausal"]["limiter_model_ms"] = {
                "sequential": bm["baseline"] * 1e3, "fused": bm["fusion"] * 1e3, "overlap": bm["overlap"] * 1e3,
                "rng_exposed": bm["rng_exposed"] * 1e3}

    # ------------------------------------------------------------------ 70B-shaped layer with fp8 GEMMs (configs[3])
    if not args.no_block:
        extras["layer_llama3_70b_fp8_s8k"] = bench_fp8_layer(torch, rov, wl, main_s, side_s, sync, ev_pair)

    # ------------------------------------------------------------------ CPU oracle on a bounded sample
    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(wl, ci, q, k, v, a, w, nbits)

    out = {
        "metric": "RNG mask Gbit/s + Transformer-block speedup: overlap vs sequential/fused",
        "value": nbits / ms_per_step / 1e6,
        "unit": "Gbit/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "llama3_8b_s2k: B=1 H=32 d=128 S=2048 p=0.1 mask 32x2048x2048 bits; "
                               "GEMM 2048x4096x14336 bf16; overlap schedule (RNG on side stream || GEMM, join, "
                               "attention with mask)",
                   "schedule": "overlap", "seed": wl.SEED, "offset": wl.OFFSET},
        "roofline": {"bound": "mfma", "kernel": "gemm_tn_kernel<7, false> (bf16, tile 256x224, inside the overlap step, RNG co-running)",
                     "achieved": gemm_flops / gemm_in_step / 1e9, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": gemm_flops / gemm_in_step / 1e9 / PEAK_BF16_TFLOPS, "traffic": TRAFFIC_GEMM_BYTES},
        "cpu_baseline": cpu,
        "extras": extras,
    }
    print(json.dumps(out))


def bench_block(torch, rov, wl, main_s, side_s, sync, ev_pair, seq_len=None, causals=(False, True), check=False):
    """Llama-3-8B block (fifth workload; seq_len overrides its S) under the three schedules.  check:
    also compare the three schedules' outputs bit for bit (they drop the same elements)."""
    ci = 4
    c = wl.CONFIGS[ci]
    B, H, Hkv, S, d, p, hidden, ffn = c["B"], c["H"], c["Hkv"], c["S"], c["d"], c["p"], c["hidden"], c["ffn"]
    S = S if seq_len is None else int(seq_len)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1000 + ci)
    bf = torch.bfloat16

    def randn(*shape, sd=1.0):
        return (torch.randn(*shape, device="cuda", generator=gen) * sd).to(bf)

    wts = dict(norm1=torch.ones(hidden, device="cuda", dtype=bf), norm2=torch.ones(hidden, device="cuda", dtype=bf),
               wqkv=randn((H + 2 * Hkv) * d, hidden, sd=0.02), wo=randn(hidden, H * d, sd=0.02),
               wg=randn(ffn, hidden, sd=0.02), wu=randn(ffn, hidden, sd=0.02), wd=randn(hidden, ffn, sd=0.02))
    x = randn(B, S, hidden)
    y = torch.empty_like(x)
    res = {}
    for causal in causals:
        cfg = rov.make_block_cfg(H, Hkv, d, hidden, ffn, p, causal=causal)
        weights = rov.make_block_weights(wts)
        ws = torch.empty(rov.block_workspace_bytes(cfg, B, S, 0), dtype=torch.uint8, device="cuda")
        m0 = torch.empty(rov.mask_shape(B, H, S), dtype=torch.int64, device="cuda")
        m1 = torch.empty_like(m0)
        off1 = rov.mask_philox_calls(B, H, S)
        rov.dropout_mask_generate(wl.SEED, 0, B, H, S, p, out=m0)
        sync()
        layer = [0]

        def seq():
            rov.block_forward(weights, x, y, cfg, rov.SCHED_SEQUENTIAL, wl.SEED, 0, m0, ws, main_s, side_s)

        def fus():
            rov.block_forward(weights, x, y, cfg, rov.SCHED_FUSED, wl.SEED, 0, None, ws, main_s, side_s)

        def ovl(sched=rov.SCHED_OVERLAP):   # steady state: this layer's mask was produced during the previous call
            cur, nxt = (m0, m1) if layer[0] % 2 == 0 else (m1, m0)
            rov.block_forward(weights, x, y, cfg, sched, wl.SEED, layer[0] * off1, cur, ws,
                              main_s, side_s, mask_ready=True, next_mask=nxt)
            layer[0] += 1

        def hyb():   # stored bits for the rows that fit beside the GEMMs, in-kernel Philox for the rest
            ovl(rov.SCHED_HYBRID)

        with torch.cuda.stream(main_s):
            t_seq = median_ms(seq, 2, 5, sync, ev_pair, inner=2)
            t_fus = median_ms(fus, 2, 5, sync, ev_pair, inner=2)
            t_ovl = median_ms(ovl, 2, 5, sync, ev_pair, inner=2)
            # hybrid in steady state needs the first rows of this layer's mask in the rows layout
            rows = rov.block_hybrid_mask_rows(cfg, B, S)
            t_hyb = None
            if 0 < rows < S:
                layer[0] = 0
                rov.dropout_mask_generate_rows(wl.SEED, 0, B, H, S, p, 0, rows, out=m0, stream=main_s)
                t_hyb = median_ms(hyb, 2, 5, sync, ev_pair, inner=2)
        res["causal" if causal else "noncausal"] = {
            "sequential_ms": t_seq, "fused_ms": t_fus, "overlap_ms": t_ovl,
            "speedup_overlap_vs_sequential": t_seq / t_ovl, "speedup_overlap_vs_fused": t_fus / t_ovl,
            "hybrid_mask_rows": rows, "hybrid_ms": t_hyb}
        if check:
            outs = []
            for fn in (seq, fus):
                sync()
                fn()
                sync()
                outs.append(y.clone())
            layer[0] = 0                                   # the overlap call that uses m0 with offset 0
            rov.dropout_mask_generate(wl.SEED, 0, B, H, S, p, out=m0)
            sync()
            ovl()
            sync()
            agree = torch.equal(outs[0], outs[1]) and torch.equal(outs[0], y)
            if 0 < rows < S:
                layer[0] = 0
                rov.dropout_mask_generate_rows(wl.SEED, 0, B, H, S, p, 0, rows, out=m0)
                sync()
                hyb()
                sync()
                agree = agree and torch.equal(outs[0], y)
            res["causal" if causal else "noncausal"]["schedules_agree_bit_for_bit"] = bool(agree)
        del ws, m0, m1
        torch.cuda.empty_cache()
    return res


def bench_fp8_layer(torch, rov, wl, main_s, side_s, sync, ev_pair):
    """All GEMMs of one Llama-3-70B-shaped layer in fp8 (e4m3, per-tensor scales; gate and up both
    run), the keep-mask of its GQA attention (64 query / 8 kv heads, S = 8192) and the attention, in
    the three schedules.  Inputs are drawn on the device; the GEMMs are independent of each other
    (the paper's silicon experiment, Sec. 6.1, with every GEMM of the layer beside the RNG)."""
    ci = 3
    c = wl.CONFIGS[ci]
    B, H, Hkv, S, d, p = c["B"], c["H"], c["Hkv"], c["S"], c["d"], c["p"]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1000 + ci)
    f8 = torch.float8_e4m3fn

    def quant(x):
        scale = float(x.abs().max()) / 448.0
        return (x / scale).to(f8), scale

    descs, keep, flop = [], [], 0.0
    shapes = [g for g in c["gemms"]] + [("ffn_gate",) + tuple(c["gemms"][2][1:])]
    for _, M, K, N in shapes:
        A8, sa = quant(torch.randn(M, K, device="cuda", generator=gen))
        W8, sw = quant(torch.randn(N, K, device="cuda", generator=gen) * 0.02)
        C = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        descs.append(rov.make_gemm_desc(A8, W8, C, scaleA=sa, scaleB=sw))
        keep += [A8, W8, C]
        flop += 2.0 * M * N * K
    bf = torch.bfloat16
    Q = torch.randn(B, S, H, d, device="cuda", generator=gen).to(bf)
    Kt = torch.randn(B, S, Hkv, d, device="cuda", generator=gen).to(bf)
    V = torch.randn(B, S, Hkv, d, device="cuda", generator=gen).to(bf)
    O = torch.empty_like(Q)
    mask = torch.empty(rov.mask_shape(B, H, S), dtype=torch.int64, device="cuda")
    ad = rov.make_attn_desc(Q, Kt, V, O, p)
    res = {}
    sync()   # the inputs were produced on torch's current stream
    with torch.cuda.stream(main_s):
        def gemms_only():
            for g in descs:
                rov.gemm_desc(g, stream=main_s)
        t_g = median_ms(gemms_only, 2, 5, sync, ev_pair, inner=2)
        t_r = median_ms(lambda: rov.dropout_mask_generate(wl.SEED, 0, B, H, S, p, out=mask, stream=main_s),
                        2, 5, sync, ev_pair, inner=2)
        for name, sched in (("sequential", rov.SCHED_SEQUENTIAL), ("fused", rov.SCHED_FUSED), ("overlap", rov.SCHED_OVERLAP)):
            res[name + "_ms"] = median_ms(
                lambda: rov.layer_step(sched, descs, ad, wl.SEED, 0, None if sched == rov.SCHED_FUSED else mask,
                                       main_s, side_s), 2, 5, sync, ev_pair, inner=2)
        # fewer Philox rounds (paper Sec. 5.2; its silicon numbers are for 7 rounds)
        sweep = {}
        for rounds in (7, 5, 3):
            r = {"rng_ms": median_ms(lambda: rov.dropout_mask_generate(wl.SEED, 0, B, H, S, p, out=mask, rounds=rounds,
                                                                               stream=main_s),
                                     2, 9, sync, ev_pair, inner=2)}
            for name, sched in (("sequential", rov.SCHED_SEQUENTIAL), ("fused", rov.SCHED_FUSED),
                                ("overlap", rov.SCHED_OVERLAP)):
                r[name + "_ms"] = median_ms(
                    lambda: rov.layer_step(sched, descs, ad, wl.SEED, 0, None if sched == rov.SCHED_FUSED else mask,
                                           main_s, side_s, rounds=rounds), 2, 9, sync, ev_pair, inner=2)
            r["speedup_overlap_vs_sequential"] = r["sequential_ms"] / r["overlap_ms"]
            r["speedup_overlap_vs_fused"] = r["fused_ms"] / r["overlap_ms"]
            # R16 on the whole step: the RNG time that no longer shows in the step
            r["rng_hidden_fraction_whole_step"] = (r["sequential_ms"] - r["overlap_ms"]) / r["rng_ms"]
            sweep["philox_%d" % rounds] = r
        res["rounds"] = sweep
        # narrower random numbers per element (paper Sec. 5.2)
        widths = {}
        for bits in (16, 8):
            r = {"rng_ms": median_ms(lambda: rov.dropout_mask_generate_bits(wl.SEED, 0, B, H, S, p, bits, out=mask,
                                                                            stream=main_s),
                                     2, 9, sync, ev_pair, inner=2)}
            for name, sched in (("sequential", rov.SCHED_SEQUENTIAL), ("fused", rov.SCHED_FUSED),
                                ("overlap", rov.SCHED_OVERLAP)):
                r[name + "_ms"] = median_ms(
                    lambda: rov.layer_step(sched, descs, ad, wl.SEED, 0, None if sched == rov.SCHED_FUSED else mask,
                                           main_s, side_s, bits=bits), 2, 9, sync, ev_pair, inner=2)
            r["speedup_overlap_vs_sequential"] = r["sequential_ms"] / r["overlap_ms"]
            r["speedup_overlap_vs_fused"] = r["fused_ms"] / r["overlap_ms"]
            r["rng_hidden_fraction_whole_step"] = (r["sequential_ms"] - r["overlap_ms"]) / r["rng_ms"]
            widths["bits_%d" % bits] = r
        res["widths"] = widths
    res["rng_hidden_fraction_whole_step"] = (res["sequential_ms"] - res["overlap_ms"]) / t_r
    res.update({"gemms_ms": t_g, "gemms_tflops": flop / t_g / 1e9, "gemms_fp8_mfma_frac": flop / t_g / 1e9 / 5000.0,
                "rng_ms": t_r, "speedup_overlap_vs_sequential": res["sequential_ms"] / res["overlap_ms"],
                "speedup_overlap_vs_fused": res["fused_ms"] / res["overlap_ms"]})
    return res


def cpu_baseline(wl, ci, q, k, v, a, w, nbits):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the step."""
    import torch
    from oracle import dense as OD
    from oracle import numerics as ON
    from oracle import philox as OP
    c = wl.CONFIGS[ci]
    B, H, S, p = c["B"], c["H"], c["S"], c["p"]
    t0 = time.perf_counter()
    words = OP.dropout_mask(wl.SEED, wl.OFFSET, B, H, S, p)          # full mask
    t_mask = time.perf_counter() - t0
    rows_g = 32
    ar = ON.bf16_round(a[:rows_g]).astype(np.float64)
    wr = ON.bf16_round(w).astype(np.float64)
    t0 = time.perf_counter()
    OD.gemm(ar, wr, transB=True)
    t_gemm = (time.perf_counter() - t0) * (a.shape[0] / rows_g)
    rows_a = wl.sample_rows(S, 16)
    keep = OP.unpack_keep(words, S)
    qr, kr, vr = [ON.bf16_round(x).astype(np.float64) for x in (q, k, v)]
    t0 = time.perf_counter()
    OD.attention_dropout(qr, kr, vr, keep, p, rows=rows_a)
    t_attn = (time.perf_counter() - t0) * (S / len(rows_a))
    total = t_mask + t_gemm + t_attn
    return {"value": nbits / total / 1e9, "unit": "Gbit/s", "cores": max(OP.num_threads(), torch.get_num_threads()),
            "kind": "oracle",
            "sample": "mask in full (%.3f s, %.2f Gbit/s); GEMM on %d of %d rows and attention on %d of %d query "
                      "rows of every head, each extrapolated by row count (GEMM %.1f s, attention %.1f s for the "
                      "full step)" % (t_mask, nbits / t_mask / 1e9, rows_g, a.shape[0], len(rows_a), S, t_gemm, t_attn),
            "mask_only_gbit_s": nbits / t_mask / 1e9}


if __name__ == "__main__":
    main()

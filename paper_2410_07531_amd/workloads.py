"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds shapes and random draws only - none of the method's
arithmetic - so both the HIP path and the CPU oracle can be fed from it.

The paper uses no dataset: its workloads are pure shapes (Sec. 4.1: head
dimension 128, batch 1, sequence 2K-64K, embedding 4K-16K).  The five
configurations below are the Llama-3-shaped instances of those shapes that
this build is measured on.
"""
import numpy as np

# name, B, H (query heads), Hkv, S, d, dropout p, dtype of the dense ops, hidden, ffn
CONFIGS = [
    dict(name="tiny", B=1, H=2, Hkv=2, S=128, d=64, p=0.1, dtype="fp32", hidden=128, ffn=256,
         gemms=[("square", 256, 256, 256)]),
    dict(name="llama3_8b_s2k", B=1, H=32, Hkv=32, S=2048, d=128, p=0.1, dtype="bf16",
         hidden=4096, ffn=14336, gemms=[("ffn_up", 2048, 4096, 14336)]),
    dict(name="llama3_8b_b2_s4k", B=2, H=32, Hkv=32, S=4096, d=128, p=0.1, dtype="bf16",
         hidden=4096, ffn=14336,
         gemms=[("qkv", 8192, 4096, 6144), ("ffn_down", 8192, 14336, 4096)]),
    dict(name="llama3_70b_s8k_fp8", B=1, H=64, Hkv=8, S=8192, d=128, p=0.1, dtype="fp8",
         hidden=8192, ffn=28672,
         gemms=[("qkv", 8192, 8192, 10240), ("o", 8192, 8192, 8192),
                ("ffn_up", 8192, 8192, 28672), ("ffn_down", 8192, 28672, 8192)]),
    dict(name="llama3_8b_block_s16k", B=1, H=32, Hkv=8, S=16384, d=128, p=0.1, dtype="bf16",
         hidden=4096, ffn=14336,
         gemms=[("qkv", 16384, 4096, 6144), ("o", 16384, 4096, 4096),
                ("ffn_up", 16384, 4096, 14336), ("ffn_down", 16384, 14336, 4096)]),
]

SEED = 1234          # Philox seed of every primary run
OFFSET = 0           # Philox offset of every primary run
CARRY_OFFSET = 2**32 - 64   # parity-only run: the call index carries into the second counter word


def rng_for(config_index):
    return np.random.default_rng(1000 + config_index)


def qkv(rng, B, S, H, Hkv, d):
    """Q [B,S,H,d], K and V [B,S,Hkv,d], each ~ N(0, 1), float32."""
    q = rng.standard_normal((B, S, H, d), dtype=np.float32)
    k = rng.standard_normal((B, S, Hkv, d), dtype=np.float32)
    v = rng.standard_normal((B, S, Hkv, d), dtype=np.float32)
    return q, k, v


def gemm_operands(rng, M, K, N):
    """Activations A [M,K] ~ N(0,1) and weights stored [N,K] ~ N(0, 0.02), float32."""
    a = rng.standard_normal((M, K), dtype=np.float32)
    w = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.02)
    return a, w


def block_weights(rng, H, Hkv, d, hidden, ffn):
    """Random-init block weights ~ N(0, 0.02); RMSNorm weights = 1."""
    def w(n, k):
        return rng.standard_normal((n, k), dtype=np.float32) * np.float32(0.02)
    return dict(
        norm1=np.ones(hidden, dtype=np.float32),
        norm2=np.ones(hidden, dtype=np.float32),
        wqkv=w((H + 2 * Hkv) * d, hidden),
        wo=w(hidden, H * d),
        wg=w(ffn, hidden),
        wu=w(ffn, hidden),
        wd=w(hidden, ffn),
    )


def block_input(rng, B, S, hidden):
    return rng.standard_normal((B, S, hidden), dtype=np.float32)


def sample_rows(S, n=16):
    """Deterministic query-row sample: first, last and evenly spread rows."""
    if S <= n:
        return list(range(S))
    idx = sorted(set([0, S - 1] + [int(round(i * (S - 1) / (n - 1))) for i in range(n)]))
    return idx

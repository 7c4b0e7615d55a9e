"""GPU parity: attention forward with dropout vs the float64 oracle.

Bar: max|gpu - ref| / max|ref| <= 2e-2 for bf16 (fp32 accumulation; the probabilities are
rounded to bf16 before the second product), 1e-4 for fp32 (hardware exp2).  The keep bits are
integers: the mask-reading and the fused kernels must give bit-identical outputs.
"""
import numpy as np
import pytest
import torch

from oracle import dense as OD
from oracle import philox as OP
from paper_2410_07531_amd import binding as rov
from paper_2410_07531_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = {torch.bfloat16: 2e-2, torch.float32: 1e-4}


def _inputs(seed, B, S, H, Hkv, d, dtype):
    rng = np.random.default_rng(seed)
    q, k, v = wl.qkv(rng, B, S, H, Hkv, d)
    return [torch.from_numpy(x).to(dtype).cuda() for x in (q, k, v)]


def _f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def _check(O, Q, K, V, keep, p, causal, dtype, rows=None):
    ref = OD.attention_dropout(_f64(Q), _f64(K), _f64(V), keep, p, causal=causal, rows=rows)
    got = _f64(O) if rows is None else _f64(O)[:, rows]
    err = float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))
    assert err <= TOL[dtype], err
    return err


CASES = [
    # B, S, H, Hkv, d, dtype
    (1, 128, 2, 2, 64, torch.float32),      # tiny workload (generic kernel)
    (2, 100, 3, 1, 40, torch.float32),      # ragged everything, GQA, odd head dim
    (1, 256, 2, 2, 128, torch.bfloat16),    # one query block, 4 KV tiles
    (1, 320, 2, 1, 128, torch.bfloat16),    # S % 256 != 0 (fused path regenerates per tile), GQA
    (2, 200, 2, 2, 128, torch.bfloat16),    # ragged S: partial KV tile and partial query block
    (1, 512, 4, 2, 64, torch.bfloat16),     # head dim 64
    (1, 1, 1, 1, 128, torch.bfloat16),      # single token
    (1, 96, 2, 2, 48, torch.bfloat16),      # bf16 on the generic kernel
]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,S,H,Hkv,d,dtype", CASES)
def test_attention_matches_oracle(B, S, H, Hkv, d, dtype, causal):
    print("attn", B, S, H, Hkv, d, dtype, causal, flush=True)
    p, seed, offset = 0.1, wl.SEED, 77
    Q, K, V = _inputs(S + d, B, S, H, Hkv, d, dtype)
    words = OP.dropout_mask(seed, offset, B, H, S, p)
    keep = OP.unpack_keep(words, S)
    mask = rov.dropout_mask_generate(seed, offset, B, H, S, p)
    assert np.array_equal(mask.cpu().numpy().view(np.uint64), words)
    O_mask = rov.attention_fwd_dropout(Q, K, V, p, mask=mask, causal=causal)
    O_fused = rov.attention_fwd_dropout(Q, K, V, p, mask=None, seed=seed, offset=offset, causal=causal)
    O_none = rov.attention_fwd_dropout(Q, K, V, 0.0, causal=causal)
    torch.cuda.synchronize()
    _check(O_mask, Q, K, V, keep, p, causal, dtype)
    _check(O_none, Q, K, V, None, 0.0, causal, dtype)
    assert torch.equal(O_mask, O_fused)           # same bits, same arithmetic


def test_attention_strided_views_and_carry_offset():
    # Q, K, V as slices of one fused [B, S, (H+2Hkv)*d] projection output, offset crossing 2^32
    B, S, H, Hkv, d = 1, 256, 4, 2, 128
    rng = np.random.default_rng(5)
    qkv = torch.from_numpy(rng.standard_normal((B, S, (H + 2 * Hkv) * d), dtype=np.float32)).bfloat16().cuda()
    Q = qkv[..., : H * d].view(B, S, H, d)
    K = qkv[..., H * d: (H + Hkv) * d].view(B, S, Hkv, d)
    V = qkv[..., (H + Hkv) * d:].view(B, S, Hkv, d)
    p, seed, offset = 0.2, 99, wl.CARRY_OFFSET
    keep = OP.unpack_keep(OP.dropout_mask(seed, offset, B, H, S, p), S)
    mask = rov.dropout_mask_generate(seed, offset, B, H, S, p)
    O1 = rov.attention_fwd_dropout(Q, K, V, p, mask=mask)
    O2 = rov.attention_fwd_dropout(Q, K, V, p, seed=seed, offset=offset)
    torch.cuda.synchronize()
    _check(O1, Q, K, V, keep, p, False, torch.bfloat16)
    assert torch.equal(O1, O2)


def test_attention_token_stride_beyond_32_bit_offsets():
    # K and V rows 2 GiB apart: the bf16 kernel addresses a (batch, kv head) with 32-bit byte offsets,
    # so this call must take the generic kernel (64-bit addressing) and still match the oracle
    B, S, H, d = 1, 3, 1, 128
    stride = (1 << 30) + 8                                    # elements between consecutive tokens
    Q, K0, V0 = _inputs(11, B, S, H, H, d, torch.bfloat16)
    bufs = [torch.zeros((S - 1) * stride + d, dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    K, V = [b.as_strided((B, S, H, d), (S * stride, stride, d, 1)) for b in bufs]
    K.copy_(K0)
    V.copy_(V0)
    p, seed = 0.25, 5
    keep = OP.unpack_keep(OP.dropout_mask(seed, 0, B, H, S, p), S)
    mask = rov.dropout_mask_generate(seed, 0, B, H, S, p)
    O = rov.attention_fwd_dropout(Q, K, V, p, mask=mask)
    torch.cuda.synchronize()
    _check(O, Q, K0, V0, keep, p, False, torch.bfloat16)
    del K, V, bufs
    torch.cuda.empty_cache()


def test_attention_constant_v_and_full_drop_rows():
    # V == c: O = c * kept softmax mass / (1-p); with p close to 1 many rows lose everything -> 0
    B, S, H, d = 1, 128, 2, 128
    Q, K, V = _inputs(1, B, S, H, H, d, torch.bfloat16)
    V[:] = 1.5
    p = 0.99
    words = OP.dropout_mask(3, 0, B, H, S, p)
    keep = OP.unpack_keep(words, S)
    mask = rov.dropout_mask_generate(3, 0, B, H, S, p)
    O = rov.attention_fwd_dropout(Q, K, V, p, mask=mask)
    torch.cuda.synchronize()
    ref = OD.attention_dropout(_f64(Q), _f64(K), _f64(V), keep, p)
    got = _f64(O)
    assert np.max(np.abs(got - ref)) / np.max(np.abs(ref)) <= 2e-2
    dead = ~keep.any(axis=-1)                      # [B, H, S]
    if dead.any():
        assert np.all(got.transpose(0, 2, 1, 3)[dead] == 0.0)


@pytest.mark.parametrize("direction", ["rising", "falling", "steps"])
def test_attention_scores_that_move_the_exponent_reference(direction):
    # scores that grow (or fall) by far more than any fixed margin along the keys: the online
    # softmax has to move its reference many times (rising), never after the first tile
    # (falling), or in steps below its margin (about 3 log2 units per 64-key tile: two absorbed,
    # the third not); rows are compared with the exact softmax of the oracle
    B, S, H, d = 1, 1024, 2, 128
    rng = np.random.default_rng(5)
    u = rng.standard_normal(d).astype(np.float32)
    u /= np.linalg.norm(u)
    q = (np.sqrt(d) * 4.0 * u)[None, None, None, :] + 0.1 * rng.standard_normal((B, S, H, d)).astype(np.float32)
    ramp = np.linspace(0.0, 1.0, S, dtype=np.float32)
    if direction == "falling":
        ramp = ramp[::-1].copy()
    if direction == "steps":
        ramp = (np.floor(np.arange(S) / 64.0) / (S / 64.0)).astype(np.float32) * 0.6
    # score(q, k_j) / sqrt(d) ~ 4 * 15 * ramp_j nats: 0 .. 60 nats (87 log2 units)
    k = (15.0 * ramp)[None, :, None, None] * u[None, None, None, :] + 0.05 * rng.standard_normal((B, S, H, d)).astype(np.float32)
    v = rng.standard_normal((B, S, H, d)).astype(np.float32)
    Q, K, V = [torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).cuda() for x in (q, k, v)]
    p, seed = 0.1, 11
    keep = OP.unpack_keep(OP.dropout_mask(seed, 0, B, H, S, p), S)
    for causal in (False, True):
        O_none = rov.attention_fwd_dropout(Q, K, V, 0.0, causal=causal)
        O_fused = rov.attention_fwd_dropout(Q, K, V, p, seed=seed, offset=0, causal=causal)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(O_none.float()).all()) and bool(torch.isfinite(O_fused.float()).all())
        _check(O_none, Q, K, V, None, 0.0, causal, torch.bfloat16)
        _check(O_fused, Q, K, V, keep, p, causal, torch.bfloat16)


def test_attention_llama8b_s2k_sampled_rows():
    # second workload at full size, as the benchmark runs it; the oracle evaluates 16 query rows
    # (first, last, spread) of every head against all 2048 keys
    c = wl.CONFIGS[1]
    B, S, H, Hkv, d, p = c["B"], c["S"], c["H"], c["Hkv"], c["d"], c["p"]
    print("attn cfg2", flush=True)
    Q, K, V = _inputs(1001, B, S, H, Hkv, d, torch.bfloat16)
    rows = wl.sample_rows(S, 16)
    mask = rov.dropout_mask_generate(wl.SEED, wl.OFFSET, B, H, S, p)
    words = mask.cpu().numpy().view(np.uint64)
    assert np.array_equal(words, OP.dropout_mask(wl.SEED, wl.OFFSET, B, H, S, p))
    keep = OP.unpack_keep(words, S)
    for causal in (False, True):
        O = rov.attention_fwd_dropout(Q, K, V, p, mask=mask, causal=causal)
        Of = rov.attention_fwd_dropout(Q, K, V, p, seed=wl.SEED, offset=wl.OFFSET, causal=causal)
        torch.cuda.synchronize()
        _check(O, Q, K, V, keep, p, causal, torch.bfloat16, rows=rows)
        assert torch.equal(O, Of)


def test_attention_error_paths():
    import ctypes
    L = rov.load()
    Q, K, V = _inputs(0, 1, 64, 2, 2, 64, torch.bfloat16)
    O = torch.full_like(Q, 3.0)
    st = rov._strides12(Q, K, V, O)
    s = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())
    call = lambda H, Hkv, p, dt: L.rov_attention_fwd_dropout(ptr(Q), ptr(K), ptr(V), ptr(O), 1, H, Hkv, 64, 64,
                                                            st, dt, 0, p, ctypes.c_void_p(0), 1, 0, s)
    assert call(2, 2, 1.0, rov.BF16) == rov.ERR_INVALID
    assert call(3, 2, 0.1, rov.BF16) == rov.ERR_INVALID        # H not a multiple of Hkv
    assert call(2, 2, 0.1, 7) == rov.ERR_INVALID
    assert call(2, 2, 0.1, rov.FP8_E4M3) == rov.ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert bool((O == 3.0).all())

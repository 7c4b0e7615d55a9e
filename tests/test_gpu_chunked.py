"""GPU parity for sequence chunking (paper Sec. 7.2): rows of the mask, attention on a range of
query rows, and the chunk-pipelined overlap schedule.

Chunking must not change a single bit: the mask rows are slices of the oracle's full mask, and
the chunked attention output equals the unchunked one exactly (and the oracle within the bf16 bar).
"""
import numpy as np
import pytest
import torch

from oracle import dense as OD
from oracle import philox as OP
from paper_2410_07531_amd import binding as rov
from paper_2410_07531_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def _dev(x, dtype=torch.bfloat16):
    return torch.from_numpy(x).to(dtype).cuda()


@pytest.mark.parametrize("B,H,S,p,seed,offset,q_begin,q_rows", [
    (1, 2, 128, 0.1, wl.SEED, wl.OFFSET, 0, 128),                   # the whole tiny mask as one chunk
    (1, 2, 128, 0.1, wl.SEED, wl.OFFSET, 32, 64),
    (2, 3, 200, 0.3, 99, 5, 96, 64),                                 # ragged S, 7 tiles per side (odd)
    (2, 3, 200, 0.3, 99, 5, 160, 500),                               # runs past S: clipped to the last rows
    (1, 5, 70, 0.25, 2**40 + 7, 2**32 - 64 * 16 - 3, 64, 32),        # last, partial tile row + carry
    (1, 4, 1024, 0.1, wl.SEED, 2**64 - 640, 256, 512),               # 64-bit wrap of the call index
    (2, 3, 4000, 0.1, 5, 640, 1024, 1504),                           # 125 tiles per side, 47 tile rows: many chunks per (batch, head) segment
    (1, 2, 4096, 0.5, 6, 0, 3072, 1024),                             # power-of-two tile rows, last quarter
])
def test_mask_rows_are_slices_of_the_full_mask(B, H, S, p, seed, offset, q_begin, q_rows):
    print("mask rows", B, H, S, p, seed, offset, q_begin, q_rows, flush=True)
    full = OP.dropout_mask(seed, offset, B, H, S, p)                 # [B, H, T, T, 16]
    qt0 = q_begin // 32
    nqt = (min(q_begin + q_rows, S) - q_begin + 31) // 32
    poison = torch.full((B, H, nqt, full.shape[3], 16), 0x2AAAAAAAAAAAAAAA, dtype=torch.int64, device="cuda")
    got = rov.dropout_mask_generate_rows(seed, offset, B, H, S, p, q_begin, q_rows, out=poison)
    assert np.array_equal(got.cpu().numpy().view(np.uint64), full[:, :, qt0:qt0 + nqt])
    assert rov.mask_words_rows(B, H, S, q_begin, q_rows) == got.numel()


def test_mask_rows_invalid_arguments():
    out = torch.zeros((1, 1, 1, 2, 16), dtype=torch.int64, device="cuda")
    for q_begin, q_rows in [(16, 32), (64, 32), (-32, 32), (0, 0)]:   # unaligned, past S, negative, empty
        with pytest.raises(rov.RovError):
            rov.dropout_mask_generate_rows(1, 0, 1, 1, 64, 0.1, q_begin, q_rows, out=out)
        assert rov.mask_words_rows(1, 1, 64, q_begin, q_rows) == 0
    assert int(out.abs().sum()) == 0


@pytest.mark.parametrize("dtype,B,S,H,Hkv,d,causal,chunks", [
    (torch.bfloat16, 1, 512, 4, 2, 128, False, [(0, 256), (256, 256)]),
    (torch.bfloat16, 2, 300, 4, 4, 64, True, [(0, 96), (96, 160), (256, 64)]),     # ragged S, uneven chunks
    (torch.float32, 1, 128, 2, 2, 64, False, [(0, 32), (32, 96)]),                  # generic kernel
])
@pytest.mark.parametrize("fused", [False, True])
def test_attention_rows_equals_full_attention(dtype, B, S, H, Hkv, d, causal, chunks, fused):
    print("attention rows", dtype, B, S, H, Hkv, d, causal, fused, flush=True)
    rng = np.random.default_rng(5)
    q, k, v = wl.qkv(rng, B, S, H, Hkv, d)
    Q, K, V = _dev(q, dtype), _dev(k, dtype), _dev(v, dtype)
    p, seed, offset = 0.2, 77, 12345
    mask = rov.dropout_mask_generate(seed, offset, B, H, S, p)
    full = rov.attention_fwd_dropout(Q, K, V, p, mask=None if fused else mask, seed=seed, offset=offset,
                                     causal=causal)
    O = torch.full_like(Q, 7.0)
    for q_begin, q_rows in chunks:
        rows = None if fused else rov.dropout_mask_generate_rows(seed, offset, B, H, S, p, q_begin, q_rows)
        rov.attention_fwd_dropout_rows(Q, K, V, p, q_begin, q_rows, O, mask_rows=rows, seed=seed, offset=offset,
                                       causal=causal)
        torch.cuda.synchronize()
    assert torch.equal(O, full)
    keep = OP.unpack_keep(OP.dropout_mask(seed, offset, B, H, S, p), S)
    ref = OD.attention_dropout(_f64(Q), _f64(K), _f64(V), keep, p, causal=causal)
    tol = 2e-2 if dtype == torch.bfloat16 else 1e-4
    assert np.max(np.abs(_f64(O) - ref)) / np.max(np.abs(ref)) <= tol


def test_attention_rows_leaves_other_rows_alone():
    B, S, H, d = 1, 256, 2, 128
    rng = np.random.default_rng(6)
    q, k, v = wl.qkv(rng, B, S, H, H, d)
    Q, K, V = _dev(q), _dev(k), _dev(v)
    O = torch.full_like(Q, 3.0)
    rows = rov.dropout_mask_generate_rows(1, 0, B, H, S, 0.1, 64, 96)
    rov.attention_fwd_dropout_rows(Q, K, V, 0.1, 64, 96, O, mask_rows=rows, seed=1, offset=0)
    torch.cuda.synchronize()
    assert bool((O[:, :64] == 3.0).all()) and bool((O[:, 160:] == 3.0).all())
    assert not bool((O[:, 64:160] == 3.0).all())


@pytest.mark.parametrize("dtype,B,S,H,Hkv,d,gemm,chunk,causal", [
    (torch.bfloat16, 1, 1024, 4, 2, 128, (512, 256, 768), 256, False),   # 4 chunks: the ring is reused
    (torch.bfloat16, 1, 1024, 4, 2, 128, (512, 256, 768), 1024, False),  # one chunk
    (torch.bfloat16, 2, 608, 2, 2, 64, (256, 128, 256), 160, True),      # ragged S, last chunk short
    (torch.float32, 1, 128, 2, 2, 64, (256, 256, 256), 32, False),       # tiny workload, generic kernels
])
def test_layer_step_chunked_equals_overlap_schedule(dtype, B, S, H, Hkv, d, gemm, chunk, causal):
    print("layer_step_chunked", dtype, B, S, H, Hkv, d, chunk, causal, flush=True)
    rng = np.random.default_rng(12)
    q, k, v = wl.qkv(rng, B, S, H, Hkv, d)
    Q, K, V = _dev(q, dtype), _dev(k, dtype), _dev(v, dtype)
    M, Kd, N = gemm
    a, w = wl.gemm_operands(rng, M, Kd, N)
    A, W = _dev(a, dtype), _dev(w, dtype)
    cdt = torch.float32 if dtype == torch.float32 else torch.bfloat16
    p, seed, offset = 0.1, wl.SEED, wl.OFFSET
    main, side = torch.cuda.Stream(), torch.cuda.Stream()
    O0, C0 = torch.zeros_like(Q), torch.zeros((M, N), dtype=cdt, device="cuda")
    mask = torch.zeros(rov.mask_shape(B, H, S), dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()   # inputs were produced on torch's current stream; the library runs on main / side
    rov.layer_step(rov.SCHED_OVERLAP, [rov.make_gemm_desc(A, W, C0)], rov.make_attn_desc(Q, K, V, O0, p, causal=causal),
                   seed, offset, mask, main, side)
    torch.cuda.synchronize()
    O1, C1 = torch.zeros_like(Q), torch.zeros((M, N), dtype=cdt, device="cuda")
    slot = rov.mask_words_rows(B, H, S, 0, chunk)
    ring = torch.full((2 * slot,), 0x2AAAAAAAAAAAAAAA, dtype=torch.int64, device="cuda")   # poison
    assert 2 * slot <= mask.numel() or chunk >= S // 2
    torch.cuda.synchronize()
    for _ in range(2):   # twice: events and ring slots are reused
        rov.layer_step_chunked([rov.make_gemm_desc(A, W, C1)], rov.make_attn_desc(Q, K, V, O1, p, causal=causal),
                               seed, offset, chunk, ring, main, side)
    torch.cuda.synchronize()
    assert torch.equal(O0, O1) and torch.equal(C0, C1)
    keep = OP.unpack_keep(OP.dropout_mask(seed, offset, B, H, S, p), S)
    ref = OD.attention_dropout(_f64(Q), _f64(K), _f64(V), keep, p, causal=causal)
    tol = 2e-2 if dtype == torch.bfloat16 else 1e-4
    assert np.max(np.abs(_f64(O1) - ref)) / np.max(np.abs(ref)) <= tol


def test_layer_step_chunked_invalid_arguments():
    Q = torch.zeros((1, 64, 2, 64), dtype=torch.bfloat16, device="cuda")
    O = torch.zeros_like(Q)
    ring = torch.zeros(2 * rov.mask_words_rows(1, 2, 64, 0, 32), dtype=torch.int64, device="cuda")
    s, t = torch.cuda.Stream(), torch.cuda.Stream()
    with pytest.raises(rov.RovError):
        rov.layer_step_chunked([], rov.make_attn_desc(Q, Q, Q, O, 0.1), 1, 0, 48, ring, s, t)    # not a multiple of 32
    with pytest.raises(rov.RovError):
        rov.layer_step_chunked([], rov.make_attn_desc(Q, Q, Q, O, 0.1), 1, 0, 32, ring, s, s)    # same stream
    with pytest.raises(rov.RovError):
        rov.layer_step_chunked([], rov.make_attn_desc(Q, Q, Q, O, 0.0), 1, 0, 32, ring, s, t)    # no dropout

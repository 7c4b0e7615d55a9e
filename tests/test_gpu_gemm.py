"""GPU parity: rov_gemm vs the float64 oracle on the same dtype-rounded inputs.

Tolerance (stated for this path): max|gpu - ref| / max|ref| <= 2e-2 for bf16 with fp32
accumulation; the arithmetic predicts about 2^-9 (one bf16 rounding of the result), so a tighter
sanity bound of 6e-3 is asserted too.  fp32: 1e-5 of the output scale.
"""
import numpy as np
import pytest
import torch

from oracle import dense as OD
from paper_2410_07531_amd import binding as rov
from paper_2410_07531_amd import workloads as wl

pytestmark = pytest.mark.gpu

BF16_TOL = 2e-2
BF16_EXPECTED = 6e-3


def _to_dev(x, dtype):
    return torch.from_numpy(x).to(dtype).cuda()


def _f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def _rel_err(got, ref):
    return float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))


@pytest.mark.parametrize("M,N,K,transB", [
    (256, 256, 64, True),        # one tile, one LDS slot (128 bytes of k per row = two k-steps)
    (256, 256, 128, True),       # two slots (both LDS stages)
    (512, 768, 448, True),       # several tiles, odd number of slots
    (2304, 256, 192, True),      # 9 tile rows over 3 slots: every cyclic start of the k walk, wrapping
    (300, 520, 192, True),       # ragged M and N (N % 4 == 0): MFMA kernel with clamped edges
    (1, 4, 64, True),            # degenerate sizes on the MFMA path
    (77, 130, 100, True),        # N % 4 != 0, K % 64 != 0: generic kernel
    (130, 96, 72, False),        # [K, N] weights: generic kernel
])
def test_gemm_bf16_matches_oracle(M, N, K, transB):
    print("gemm bf16", M, N, K, transB, flush=True)
    rng = np.random.default_rng(M * 131 + N * 17 + K)
    a, w = wl.gemm_operands(rng, M, K, N)
    A = _to_dev(a, torch.bfloat16)
    W = _to_dev(w if transB else np.ascontiguousarray(w.T), torch.bfloat16)
    C = rov.gemm(A, W, transB=transB)
    torch.cuda.synchronize()
    ref = OD.gemm(_f64(A), _f64(W), transB=transB)
    err = _rel_err(_f64(C), ref)
    assert err <= BF16_TOL and err <= BF16_EXPECTED, err


@pytest.mark.parametrize("cols", [128, 160, 192, 224, 256])
def test_gemm_bf16_every_tile_width(cols):
    # each width of the matrix-core kernel on a shape with several tiles in both directions, a
    # ragged last tile for every width (N = 1000), clamped rows (M = 600) and an odd slot count;
    # all widths give the same bits (same k order per element)
    M, N, K = 600, 1000, 448
    print("gemm bf16 width", cols, flush=True)
    rng = np.random.default_rng(11)
    a, w = wl.gemm_operands(rng, M, K, N)
    A, W = _to_dev(a, torch.bfloat16), _to_dev(w, torch.bfloat16)
    prev = rov.set_gemm_tile_cols(cols)
    try:
        C = rov.gemm(A, W, transB=True)
        torch.cuda.synchronize()
    finally:
        rov.set_gemm_tile_cols(prev)
    ref = OD.gemm(_f64(A), _f64(W), transB=True)
    err = _rel_err(_f64(C), ref)
    assert err <= BF16_TOL and err <= BF16_EXPECTED, err
    C0 = rov.gemm(A, W, transB=True)       # width chosen from the shape
    torch.cuda.synchronize()
    assert torch.equal(C.view(torch.int16), C0.view(torch.int16))


@pytest.mark.parametrize("M,N,K", [
    (256, 128, 64),         # one 128-column tile, one slot-step
    (600, 1000, 448),       # ragged rows and columns (last tile: 104 of 128), odd slot count
    (300, 72, 192),         # fewer columns than one wave's half of a 64-column tile
    (2304, 192, 128),       # nine tile rows (every k start), narrow output
    (512, 4096, 256),       # 64 tiles of 128 columns
])
@pytest.mark.parametrize("form", [0, 128, 256])       # the launch's choice, the narrow tile, the wide tile
def test_gemm_swiglu_matches_oracle(M, N, K, form):
    # silu(A Wg^T) * (A Wu^T) from the dual product: the oracle's two products and its silu
    print("gemm swiglu", M, N, K, form, flush=True)
    rng = np.random.default_rng(M + 3 * N + K)
    a, wg = wl.gemm_operands(rng, M, K, N)
    _, wu = wl.gemm_operands(rng, M, K, N)
    wg, wu = wg * np.float32(40.0), wu * np.float32(40.0)     # gate values of order 1: the silu's curve matters
    A, Wg, Wu = _to_dev(a, torch.bfloat16), _to_dev(wg, torch.bfloat16), _to_dev(wu, torch.bfloat16)
    prev = rov.set_gemm_tile_cols(form)
    try:
        C = rov.gemm_swiglu(A, Wg, Wu)
        torch.cuda.synchronize()
    finally:
        rov.set_gemm_tile_cols(prev)
    g = OD.gemm(_f64(A), _f64(Wg), transB=True)
    u = OD.gemm(_f64(A), _f64(Wu), transB=True)
    ref = OD.silu(g) * u
    err = _rel_err(_f64(C), ref)
    assert err <= BF16_TOL and err <= BF16_EXPECTED, err
    # gate and up are not interchangeable
    assert _rel_err(_f64(rov.gemm_swiglu(A, Wu, Wg)), ref) > 0.1


def test_gemm_tile_width_knob_rejects_other_values():
    prev = rov.set_gemm_tile_cols(0)
    for bad in (-32, 64, 96, 130, 288):
        with pytest.raises(rov.RovError):
            rov.set_gemm_tile_cols(bad)
    assert rov.set_gemm_tile_cols(prev) == 0


def test_gemm_bf16_scale_and_one_hot():
    # alpha = scaleA*scaleB is applied; one-hot activations copy weight rows exactly (bf16 in, bf16 out)
    rng = np.random.default_rng(3)
    _, w = wl.gemm_operands(rng, 256, 128, 256)
    W = _to_dev(w, torch.bfloat16)
    A = torch.zeros((256, 128), dtype=torch.bfloat16, device="cuda")
    idx = torch.arange(256, device="cuda") % 128
    A[torch.arange(256, device="cuda"), idx] = 1.0
    C = rov.gemm(A, W, transB=True)
    assert torch.equal(C, W[:, idx.cpu()].T.contiguous().cuda() if False else W.T[idx])
    C2 = rov.gemm(A, W, transB=True, scaleA=0.5, scaleB=4.0)
    assert torch.equal(C2.float(), 2.0 * C.float())


def test_gemm_fp32_tiny_workload():
    c = wl.CONFIGS[0]
    _, M, K, N = c["gemms"][0]
    a = wl.rng_for(0).standard_normal((M, K), dtype=np.float32)
    b = wl.rng_for(0).standard_normal((K, N), dtype=np.float32)
    for transB in (False, True):
        A, Bm = _to_dev(a, torch.float32), _to_dev(b if not transB else np.ascontiguousarray(b.T), torch.float32)
        C = rov.gemm(A, Bm, transB=transB)
        ref = OD.gemm(a.astype(np.float64), b.astype(np.float64))
        assert _rel_err(_f64(C), ref) <= 1e-5


def test_gemm_bf16_llama8b_ffn_up_sampled():
    # full-size second workload (2048 x 4096 x 14336) in the configuration the benchmark times;
    # the oracle evaluates 64 sampled rows in full and 4096 single entries
    _, M, K, N = wl.CONFIGS[1]["gemms"][0]
    print("gemm cfg2", M, K, N, flush=True)
    rng = wl.rng_for(1)
    a, w = wl.gemm_operands(rng, M, K, N)
    A, W = _to_dev(a, torch.bfloat16), _to_dev(w, torch.bfloat16)
    C = rov.gemm(A, W, transB=True)
    torch.cuda.synchronize()
    Ah, Wh, Ch = _f64(A), _f64(W), _f64(C)
    srng = np.random.default_rng(7)
    rows = np.sort(srng.choice(M, 64, replace=False))
    rows[0], rows[-1] = 0, M - 1
    ref_rows = OD.gemm(Ah[rows], Wh, transB=True)
    scale = float(np.max(np.abs(ref_rows)))
    err = float(np.max(np.abs(Ch[rows] - ref_rows)) / scale)
    assert err <= BF16_TOL and err <= BF16_EXPECTED, err
    rr, cc = srng.integers(0, M, 4096), srng.integers(0, N, 4096)
    ent = OD.gemm_entries(Ah, Wh, rr, cc, transB=True)
    assert float(np.max(np.abs(Ch[rr, cc] - ent)) / scale) <= BF16_EXPECTED


def test_gemm_error_paths():
    import ctypes
    L = rov.load()
    A = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    C = torch.full((64, 64), 7.0, dtype=torch.bfloat16, device="cuda")
    s = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    assert L.rov_gemm(p(A), p(A), p(C), 0, 64, 64, rov.BF16, 1, 1.0, 1.0, s) == rov.ERR_INVALID
    assert L.rov_gemm(ctypes.c_void_p(0), p(A), p(C), 64, 64, 64, rov.BF16, 1, 1.0, 1.0, s) == rov.ERR_INVALID
    assert L.rov_gemm(p(A), p(A), p(C), 64, 64, 64, 9, 1, 1.0, 1.0, s) == rov.ERR_INVALID
    assert L.rov_gemm(ctypes.c_void_p(A.data_ptr() + 2), p(A), p(C), 32, 32, 32, rov.BF16, 1, 1.0, 1.0, s) == rov.ERR_INVALID
    torch.cuda.synchronize()
    assert bool((C == 7.0).all())


# ----------------------------------------------------------------------------- fp8 (OCP e4m3)
FP8_TOL = 6e-2          # the workload definition's bar for fp8 GEMM outputs
FP8_EXPECTED = 6e-3     # fp8 x fp8 products are exact in fp32; only the bf16 result rounding remains


def _quantise(x):
    """Per-tensor scale = amax/448; codes by the library conversion (plumbing); both sides get the codes."""
    amax = float(np.max(np.abs(x)))
    scale = float(np.float32(amax / 448.0))
    codes = torch.from_numpy((x / np.float32(scale)).astype(np.float32)).to(torch.float8_e4m3fn)
    return codes.view(torch.uint8), scale


def test_gemm_fp8_decodes_every_code_as_ocp_e4m3():
    from oracle import numerics as ON
    table = ON.e4m3_decode_table()
    K, N, M = 128, 256, 128
    A = torch.zeros((M, K), dtype=torch.uint8)
    A[torch.arange(M), torch.arange(M)] = 0x38                      # 1.0
    W = torch.zeros((N, K), dtype=torch.uint8)
    W[torch.arange(N), torch.arange(N) % K] = torch.arange(N, dtype=torch.int32).to(torch.uint8)
    W[0x7F, 0x7F] = 0                                               # the two NaN codes are left out
    W[0xFF, 0xFF % K] = 0
    C = rov.gemm(A.cuda(), W.cuda(), transB=True)
    torch.cuda.synchronize()
    got = _f64(C)
    for n in range(N):
        if n in (0x7F, 0xFF):
            continue
        assert got[n % K, n] == table[n], (n, got[n % K, n], table[n])
    assert np.count_nonzero(got) == 256 - 4                         # +-0 and the two skipped codes


@pytest.mark.parametrize("M,N,K", [
    (256, 256, 128),        # one tile, one k-step
    (512, 768, 896),        # several tiles, odd number of k-steps
    (300, 520, 384),        # ragged M and N
    (77, 130, 100),         # generic kernel (N % 4 != 0, K % 128 != 0)
])
def test_gemm_fp8_matches_oracle(M, N, K):
    from oracle import numerics as ON
    print("gemm fp8", M, N, K, flush=True)
    rng = np.random.default_rng(M + N + K)
    a, w = wl.gemm_operands(rng, M, K, N)
    Aq, sa = _quantise(a)
    Wq, sb = _quantise(w)
    C = rov.gemm(Aq.cuda(), Wq.cuda(), transB=True, scaleA=sa, scaleB=sb)
    torch.cuda.synchronize()
    ref = sa * sb * OD.gemm(ON.e4m3_decode(Aq.numpy()), ON.e4m3_decode(Wq.numpy()), transB=True)
    err = _rel_err(_f64(C), ref)
    assert err <= FP8_TOL and err <= FP8_EXPECTED, err
    # the oracle's own encoder picks the same codes as the plumbing conversion (zero sign aside)
    mine = ON.e4m3_encode(a / np.float32(sa))
    nz = (mine & 0x7F) != 0
    assert np.array_equal(mine[nz], Aq.numpy()[nz])


@pytest.mark.parametrize("cols", [128, 160, 192, 224, 256])
def test_gemm_fp8_every_tile_width(cols):
    # each width of the matrix-core kernel: ragged last tile for every width, clamped rows, odd
    # number of k-steps; and every e4m3 code decoded exactly through that width
    from oracle import numerics as ON
    print("gemm fp8 width", cols, flush=True)
    M, N, K = 600, 1000, 640
    rng = np.random.default_rng(13)
    a, w = wl.gemm_operands(rng, M, K, N)
    Aq, sa = _quantise(a)
    Wq, sb = _quantise(w)
    table = ON.e4m3_decode_table()
    Kd, Nd, Md = 128, 256, 128
    Ad = torch.zeros((Md, Kd), dtype=torch.uint8)
    Ad[torch.arange(Md), torch.arange(Md)] = 0x38                   # 1.0
    Wd = torch.zeros((Nd, Kd), dtype=torch.uint8)
    Wd[torch.arange(Nd), torch.arange(Nd) % Kd] = torch.arange(Nd, dtype=torch.int32).to(torch.uint8)
    Wd[0x7F, 0x7F] = 0                                              # the two NaN codes are left out
    Wd[0xFF, 0xFF % Kd] = 0
    prev = rov.set_gemm_tile_cols(cols)
    try:
        C = rov.gemm(Aq.cuda(), Wq.cuda(), transB=True, scaleA=sa, scaleB=sb)
        D = rov.gemm(Ad.cuda(), Wd.cuda(), transB=True)
        torch.cuda.synchronize()
    finally:
        rov.set_gemm_tile_cols(prev)
    ref = sa * sb * OD.gemm(ON.e4m3_decode(Aq.numpy()), ON.e4m3_decode(Wq.numpy()), transB=True)
    err = _rel_err(_f64(C), ref)
    assert err <= FP8_TOL and err <= FP8_EXPECTED, err
    got = _f64(D)
    for n in range(Nd):
        if n not in (0x7F, 0xFF):
            assert got[n % Kd, n] == table[n], (n, got[n % Kd, n], table[n])
    assert np.count_nonzero(got) == 256 - 4


def test_gemm_fp8_llama70b_qkv_sampled():
    # fourth workload's QKV projection at full size: 8192 x 8192 x 10240, fp8 e4m3, per-tensor scales
    from oracle import numerics as ON
    _, M, K, N = wl.CONFIGS[3]["gemms"][0]
    print("gemm fp8 cfg4 qkv", M, K, N, flush=True)
    rng = wl.rng_for(3)
    a, w = wl.gemm_operands(rng, M, K, N)
    Aq, sa = _quantise(a)
    Wq, sb = _quantise(w)
    C = rov.gemm(Aq.cuda(), Wq.cuda(), transB=True, scaleA=sa, scaleB=sb)
    torch.cuda.synchronize()
    Ch = _f64(C)
    srng = np.random.default_rng(9)
    rows = np.sort(srng.choice(M, 32, replace=False))
    rows[0], rows[-1] = 0, M - 1
    Wd = ON.e4m3_decode(Wq.numpy())
    ref = sa * sb * OD.gemm(ON.e4m3_decode(Aq.numpy()[rows]), Wd, transB=True)
    scale = float(np.max(np.abs(ref)))
    err = float(np.max(np.abs(Ch[rows] - ref)) / scale)
    assert err <= FP8_TOL and err <= FP8_EXPECTED, err
    # reported only: distance to the unquantised product
    full = OD.gemm(a[rows].astype(np.float64), w.astype(np.float64), transB=True)
    print("fp8 vs unquantised product: rel err %.4f" % (np.max(np.abs(Ch[rows] - full)) / np.max(np.abs(full))), flush=True)


@pytest.mark.parametrize("M,N,K", [
    (256, 128, 128),        # one 128-column tile, one k-step
    (600, 1000, 896),       # ragged rows and columns, odd number of k-steps
    (300, 72, 384),         # fewer columns than one wave's half of a 64-column tile
    (512, 4096, 256),       # 64 tiles of 128 columns
])
@pytest.mark.parametrize("form", [128, 256])          # the narrow and the wide tile
def test_gemm_swiglu_fp8_codes_match_oracle(M, N, K, form):
    # e4m3( silu(sA sWg A Wg^T) * (sA sWu A Wu^T) / sC ): the codes the kernel writes against the
    # oracle's nearest-code choice on the float64 value.  The kernel takes the decision on its own
    # fp32 value (matrix-core accumulation of sums with cancelling terms, fast exponential), which is
    # the exact one up to about 3e-5 of the output scale: where the codes differ (few places), the
    # kernel's code must be as close to the exact value as the best code up to twice that bound.
    from oracle import numerics as ON
    print("gemm swiglu fp8", M, N, K, form, flush=True)
    rng = np.random.default_rng(5 * M + N + K)
    a, wg = wl.gemm_operands(rng, M, K, N)
    _, wu = wl.gemm_operands(rng, M, K, N)
    Aq, sa = _quantise(a)
    Gq, sg = _quantise(wg * np.float32(40.0))      # gate values of order 1: the silu's curve matters
    Uq, su = _quantise(wu * np.float32(40.0))
    g = sa * sg * OD.gemm(ON.e4m3_decode(Aq.numpy()), ON.e4m3_decode(Gq.numpy()), transB=True)
    u = sa * su * OD.gemm(ON.e4m3_decode(Aq.numpy()), ON.e4m3_decode(Uq.numpy()), transB=True)
    v = OD.silu(g) * u
    sc = float(np.float32(np.max(np.abs(v)) / 600.0))          # the largest values saturate at 448
    prev = rov.set_gemm_tile_cols(form)
    try:
        C = rov.gemm_swiglu_fp8(Aq.cuda(), Gq.cuda(), Uq.cuda(), sa, sg, su, sc)
        torch.cuda.synchronize()
    finally:
        rov.set_gemm_tile_cols(prev)
    got = C.cpu().numpy()
    exp = ON.e4m3_encode(v / sc)
    assert np.any((exp & 0x7F) == 0x7E)                        # saturation is exercised
    same = (got == exp) | (((got | exp) & 0x7F) == 0)          # +0 and -0 are the same value
    bad = ~same
    assert bad.mean() <= 1e-2, bad.mean()
    dg, de = ON.e4m3_decode(got[bad]), ON.e4m3_decode(exp[bad])
    x = (v / sc)[bad]
    eps = 3e-5 * np.max(np.abs(v / sc))
    assert np.all(np.abs(dg - x) <= np.abs(de - x) + 2 * eps), np.max(np.abs(dg - x) - np.abs(de - x)) / eps
    ref = np.clip(v / sc, -448, 448)
    assert np.max(np.abs(ON.e4m3_decode(got) - ref)) / np.max(np.abs(ref)) <= FP8_TOL
    # gate and up are not interchangeable
    C2 = rov.gemm_swiglu_fp8(Aq.cuda(), Uq.cuda(), Gq.cuda(), sa, su, sg, sc)
    torch.cuda.synchronize()
    assert (C2.cpu().numpy() != exp).mean() > 0.5


def test_gemm_swiglu_fp8_error_paths():
    A = torch.zeros((256, 128), dtype=torch.uint8, device="cuda")
    W = torch.zeros((128, 128), dtype=torch.uint8, device="cuda")
    for kw, code in ((dict(scaleC=0.0), rov.ERR_INVALID), (dict(scaleC=-1.0), rov.ERR_INVALID)):
        with pytest.raises(rov.RovError) as e:
            rov.gemm_swiglu_fp8(A, W, W, 1.0, 1.0, 1.0, kw["scaleC"])
        assert e.value.code == code
    with pytest.raises(rov.RovError) as e:      # K not a multiple of 128
        rov.gemm_swiglu_fp8(A[:, :64].contiguous(), W[:, :64].contiguous(), W[:, :64].contiguous(), 1.0, 1.0, 1.0, 1.0)
    assert e.value.code == rov.ERR_UNSUPPORTED

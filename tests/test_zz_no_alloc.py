"""rov_block_forward_static: the block forward on the library's static device scratch.

Called through the C ABI and compared with rov_block_forward (caller's workspace) on the same
inputs: identical kernels on another buffer, so the outputs must be bit-identical (which is
inside every tolerance the block has against the oracle).  Two calls in a row, the second on a
smaller input, because the scratch keeps the first call's contents.
"""
import numpy as np
import pytest
import torch

from paper_2410_07531_amd import binding as rov
from paper_2410_07531_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _setup(B, S, H, Hkv, d, hidden, ffn, seed):
    rng = np.random.default_rng(seed)
    w = wl.block_weights(rng, H, Hkv, d, hidden, ffn)
    x = wl.block_input(rng, B, S, hidden)
    to = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    return to(x), {k: to(v) for k, v in w.items()}


def _pair(B, S, H, Hkv, d, hidden, ffn, sched, causal, main, side, seed):
    """y from rov_block_forward and from rov_block_forward_static, and both next-layer masks."""
    p, pseed, offset = 0.1, wl.SEED, 1280
    x, wd = _setup(B, S, H, Hkv, d, hidden, ffn, seed)
    cfg = rov.make_block_cfg(H, Hkv, d, hidden, ffn, p, causal=causal)
    weights = rov.make_block_weights(wd)
    need = rov.block_workspace_bytes(cfg, B, S, 0)
    assert 0 < need <= rov.block_static_scratch_bytes()
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    out = []
    for static in (False, True):
        y = torch.zeros_like(x)
        mask = None if sched == rov.SCHED_FUSED else torch.zeros(rov.mask_shape(B, H, S), dtype=torch.int64, device="cuda")
        nxt = torch.zeros(rov.mask_shape(B, H, S), dtype=torch.int64, device="cuda") if sched == rov.SCHED_OVERLAP else None
        torch.cuda.synchronize()   # inputs were produced on torch's current stream
        if static:
            rov.block_forward_static(weights, x, y, cfg, sched, pseed, offset, mask, main, side, next_mask=nxt)
        else:
            rov.block_forward(weights, x, y, cfg, sched, pseed, offset, mask, ws, main, side, next_mask=nxt)
        torch.cuda.synchronize()
        out.append((y, nxt))
    return out


@pytest.mark.parametrize("sched", [rov.SCHED_SEQUENTIAL, rov.SCHED_FUSED, rov.SCHED_OVERLAP])
def test_static_scratch_block_equals_workspace_block_twice(sched):
    main, side = torch.cuda.Stream(), torch.cuda.Stream()
    H, Hkv, d, hidden, ffn = 4, 2, 128, 512, 1024
    # first a larger block, then a smaller one on the scratch the first one left behind
    for n, (S, causal) in enumerate(((384, False), (160, True))):
        print("static block", sched, S, causal, flush=True)
        (y_ws, nxt_ws), (y_st, nxt_st) = _pair(1, S, H, Hkv, d, hidden, ffn, sched, causal, main, side, 40 + n)
        assert torch.isfinite(y_st.float()).all()
        assert float(y_st.float().abs().max()) > 0.0
        assert torch.equal(y_ws, y_st), (sched, S)
        if nxt_ws is not None:
            assert torch.equal(nxt_ws, nxt_st)


def test_static_scratch_refuses_blocks_beyond_its_size():
    # 64 MiB holds 1024 tokens of the hidden-4096 / ffn-14336 block; 2048 tokens must be refused
    # before anything is enqueued (the output stays as it was)
    H, Hkv, d, hidden, ffn = 32, 8, 128, 4096, 14336
    cfg = rov.make_block_cfg(H, Hkv, d, hidden, ffn, 0.1)
    assert rov.block_workspace_bytes(cfg, 1, 1024, 0) <= rov.block_static_scratch_bytes()
    assert rov.block_workspace_bytes(cfg, 1, 2048, 0) > rov.block_static_scratch_bytes()
    x = torch.zeros((1, 2048, hidden), dtype=torch.bfloat16, device="cuda")
    y = torch.full_like(x, 3.0)
    wd = dict(norm1=torch.ones(hidden, dtype=torch.bfloat16, device="cuda"), norm2=torch.ones(hidden, dtype=torch.bfloat16, device="cuda"),
              wqkv=torch.zeros(((H + 2 * Hkv) * d, hidden), dtype=torch.bfloat16, device="cuda"),
              wo=torch.zeros((hidden, H * d), dtype=torch.bfloat16, device="cuda"),
              wg=torch.zeros((ffn, hidden), dtype=torch.bfloat16, device="cuda"),
              wu=torch.zeros((ffn, hidden), dtype=torch.bfloat16, device="cuda"),
              wd=torch.zeros((hidden, ffn), dtype=torch.bfloat16, device="cuda"))
    main, side = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    with pytest.raises(rov.RovError) as e:
        rov.block_forward_static(rov.make_block_weights(wd), x, y, cfg, rov.SCHED_FUSED, wl.SEED, 0, None, main, side)
    assert e.value.code == rov.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((y == 3.0).all())

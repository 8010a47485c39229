"""rq_block_forward_noalloc (scratch in a fixed device array of the library) against rq_block_forward (caller workspace)."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import repquant_oracle as orc
from paper_2402_05628_amd import synth
from tests.helpers import block_to_device, cfg_dict, dev

pytestmark = pytest.mark.gpu


def test_noalloc_matches_workspace_entry_point_twice_in_a_row():
    """Two calls in a row on the same GPU, the second with a smaller input that leaves the first call's bytes behind it in
    the shared array: each must equal the existing entry point bit for bit (same kernels, same plan) and the oracle to the
    block's bar.  A third shape too large for the array is refused with RQ_ERR_WORKSPACE before any GPU work."""
    from paper_2402_05628_amd import binding as b
    ctx = b.Context(0)
    cap = b.noalloc_scratch_bytes()
    assert cap == 32 << 20
    big_cfg, small_cfg = synth.CONFIGS[1].with_batch(6), synth.CONFIGS[1].with_batch(2)
    raw = synth.make_block(big_cfg, cfg_id=1, seed=0)
    P = orc.calibrate_block(raw, cfg_dict(big_cfg))
    for path in (b.ATTN_AUTO, b.ATTN_THREE_KERNELS):       # the second path keeps logits and codes in the scratch
        blk = b.Block(ctx, big_cfg, block_to_device(P), attn_path=path)
        for cfg in (big_cfg, small_cfg):
            print("case path", path, "batch", cfg.batch, flush=True)
            need = b._rq_block_ws(C.byref(blk.bp), cfg.batch, cfg.seq)
            assert 0 < need <= cap
            x_np = raw["x"][: cfg.tokens]
            x = dev(x_np)
            y_ws = torch.zeros_like(x)
            blk.forward(x, y_ws, cfg.batch, cfg.seq)
            y_na = torch.full_like(x, float("nan"))
            free_before = torch.cuda.mem_get_info()[0]
            b.rq_block_forward_noalloc(blk, x, y_na, cfg.batch, cfg.seq)
            torch.cuda.synchronize()
            assert torch.cuda.mem_get_info()[0] == free_before          # nothing was allocated on the device
            assert torch.equal(y_na, y_ws)
            Ps = dict(P)
            Ps["cfg"] = cfg_dict(cfg)
            want = orc.block_forward(Ps, x_np)
            got = y_na.cpu().numpy().astype(np.float64)
            assert np.abs(got - want).max() <= 1e-3 * np.abs(want).max()
    # beyond the array: refused, and y untouched
    huge = synth.CONFIGS[1]
    assert b._rq_block_ws(C.byref(blk.bp), huge.batch, huge.seq) > cap
    x = torch.zeros((huge.tokens, huge.D), device="cuda")
    y = torch.full_like(x, 7.0)
    with pytest.raises(b.RqError) as ei:
        b.rq_block_forward_noalloc(blk, x, y, huge.batch, huge.seq)
    assert ei.value.status == 4 and "scratch" in str(ei.value)
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())

"""rq_block_forward against the oracle block, with the oracle's calibrated parameters handed to both sides."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import repquant_oracle as orc
from paper_2402_05628_amd import synth
from tests.helpers import block_to_device, cfg_dict, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rq():
    from paper_2402_05628_amd import binding
    return binding, binding.Context(0)


SMALL = {
    "vit_s_tiny_w8a8": synth.CONFIGS[0],                                            # the full correctness config
    "vit_b_w4a4_b2": synth.CONFIGS[1].with_batch(2),
    "swin_b_window_w6a6_b16": synth.CONFIGS[2].with_batch(16),
    "llama_like_w4a8": dataclasses.replace(synth.CONFIGS[3], seq=320, D=512, H=4, Dm=1024),
    "clip_vit_l14_w4a4_b2": synth.CONFIGS[4].with_batch(2),
}


@pytest.mark.parametrize("name", list(SMALL))
@pytest.mark.parametrize("chunk_mb", [64, 1])
def test_block_forward_matches_oracle(rq, name, chunk_mb):
    b, ctx = rq
    cfg = SMALL[name]
    print("case", name, chunk_mb, flush=True)
    raw = synth.make_block(cfg, cfg_id=list(SMALL).index(name), seed=0)
    P = orc.calibrate_block(raw, cfg_dict(cfg))
    want, t = orc.block_forward(P, raw["x"], keep=True)
    b.set_attn_chunk_bytes(chunk_mb << 20)
    try:
        blk = b.Block(ctx, cfg, block_to_device(P))
        x = dev(raw["x"])
        y = torch.zeros_like(x)
        blk.forward(x, y, cfg.batch, cfg.seq)
        torch.cuda.synchronize()
    finally:
        b.set_attn_chunk_bytes(64 << 20)
    got = y.cpu().numpy().astype(np.float64)
    ref = np.abs(want).max()
    err = np.abs(got - want).max()
    print("  max|d| / max|ref| = %.3g" % (err / ref), flush=True)
    assert err <= 1e-3 * ref
    # fraction of elements outside the element-wise bar (downstream of a tie flip): reported, bounded loosely
    bar = 1e-3 * np.maximum(np.abs(want), 1e-3 * ref)
    frac = float(np.mean(np.abs(got - want) > bar))
    print("  elements beyond the element-wise bar: %.3g" % frac, flush=True)
    assert frac < 0.02

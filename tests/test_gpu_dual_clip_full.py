"""Dual-clipping learner at the benchmark's size and launch configuration (ViT-B LayerNorm-1 activation, 12 608 tokens x
768 channels, 4 bits, 100 iterations): channels are independent problems, so the oracle runs on a sample of them."""
import numpy as np
import pytest
import torch

from oracle import dual_clip_oracle as dco
from oracle import repquant_oracle as orc
from paper_2402_05628_amd import synth
from tests.helpers import dev

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(300)
def test_full_size_sampled_channels():
    from paper_2402_05628_amd import binding as b
    ctx = b.Context()
    cfg = synth.CONFIGS[1]
    raw = synth.make_block(cfg, 1, 0)
    print("case full size", cfg.tokens, cfg.D, flush=True)
    got = b.rq_dual_clip_learn(ctx, dev(raw["x"]), cfg.bits_a, gamma=dev(raw["ln1_gamma"]), beta=dev(raw["ln1_beta"]),
                               norm_kind=cfg.norm, eps=cfg.eps, iters=100, lr=0.01, alpha0=4.0)
    torch.cuda.synchronize()
    Xp = orc.layernorm(raw["x"].astype(np.float64), raw["ln1_gamma"].astype(np.float64), raw["ln1_beta"].astype(np.float64),
                       cfg.eps, cfg.norm)
    pick = np.random.default_rng(0).choice(cfg.D, size=48, replace=False)
    pick[:4] = [0, 1, cfg.D - 2, cfg.D - 1]
    want = dco.learn(Xp[:, pick], cfg.bits_a, iters=100, lr=0.01, alpha0=4.0)
    for k in ("alpha1", "alpha2"):
        np.testing.assert_allclose(got[k].cpu().numpy()[pick], want[k], rtol=0, atol=1e-7, err_msg=k)
    for k in ("up", "lo", "loss0", "loss"):
        np.testing.assert_allclose(got[k].cpu().numpy()[pick], want[k], rtol=1e-7, err_msg=k)
    # every channel: the factors stay within reach of 100 Adam steps and the error does not grow overall
    a1, a2 = got["alpha1"].cpu().numpy(), got["alpha2"].cpu().numpy()
    assert np.all(np.isfinite(a1)) and np.all(np.isfinite(a2))
    assert np.all(np.abs(a1 - 4.0) <= 100 * 0.01 * 3.17) and np.all(np.abs(a2 - 4.0) <= 100 * 0.01 * 3.17)
    assert got["loss"].sum().item() < got["loss0"].sum().item()
    ctx.close()

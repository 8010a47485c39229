"""GPU parity of the dual-clipping learner (Section "Per-channel dual clipping") against the float64 oracle.

Both sides compute in float64 and differ only in the order of the sums (and in how exp / sqrt round), so the learnt
factors agree to ~1e-12 unless a value sits within an ulp of a rounding tie, where one code -- and with it a gradient
term -- can flip; the tolerance leaves room for a few such flips (each moves alpha by far less than one Adam step)."""
import numpy as np
import pytest
import torch

from oracle import dual_clip_oracle as dco
from oracle import repquant_oracle as orc
from paper_2402_05628_amd import synth
from tests.helpers import dev

pytestmark = pytest.mark.gpu

ALPHA_TOL = 1e-7
REL_TOL = 1e-7


@pytest.fixture(scope="module")
def rq():
    from paper_2402_05628_amd import binding as b
    ctx = b.Context()
    yield b, ctx
    ctx.close()


def _check(got, want, D):
    g = {k: v.cpu().numpy() for k, v in got.items() if not k.startswith("_")}
    for k in ("alpha1", "alpha2"):
        np.testing.assert_allclose(g[k], want[k], rtol=0, atol=ALPHA_TOL, err_msg=k)
    for k in ("up", "lo", "loss0", "loss"):
        np.testing.assert_allclose(g[k], want[k], rtol=REL_TOL, atol=1e-300, err_msg=k)
    np.testing.assert_allclose(g["clip_up"], want["clip_up"].astype(np.float32), rtol=2e-7)
    np.testing.assert_allclose(g["clip_lo"], want["clip_lo"].astype(np.float32), rtol=2e-7)


# T spans one wavefront, several workgroup shapes, rows held in registers and rows re-read every pass
@pytest.mark.parametrize("T,D,bits,alpha0,iters", [
    (197, 24, 4, 4.0, 100), (1000, 40, 4, 0.0, 100), (3001, 16, 6, 1.0, 60), (50, 8, 8, 2.0, 30), (1, 8, 4, 4.0, 5),
    (30000, 6, 4, 0.5, 25), (9000, 300, 4, 1.5, 20), (2, 3, 4, 1.0, 10), (64, 1, 16, 3.0, 10), (500, 5, 2, 0.0, 40)])
def test_learner_matches_oracle_on_given_activations(rq, T, D, bits, alpha0, iters):
    b, ctx = rq
    print("case", T, D, bits, alpha0, iters, flush=True)
    X = synth.make_rows_asymmetric(T, D, seed=T + D)
    if D >= 8:
        X[:, 3] = 1.25                                    # a constant channel
    want = dco.learn(X.astype(np.float64), bits, iters=iters, alpha0=alpha0)
    got = b.rq_dual_clip_learn(ctx, dev(X), bits, iters=iters, alpha0=alpha0)
    torch.cuda.synchronize()
    _check(got, want, D)


@pytest.mark.parametrize("kind", [orc.NORM_LAYERNORM, orc.NORM_RMSNORM])
def test_learner_with_the_normalization_inside(rq, kind):
    b, ctx = rq
    T, D, bits = 1500, 64, 4
    x = synth.make_rows(T, D, seed=5)
    g = np.random.default_rng(8)
    gamma = (1.0 + 0.1 * g.standard_normal(D)).astype(np.float32)
    beta = (0.1 * g.standard_normal(D)).astype(np.float32) if kind == orc.NORM_LAYERNORM else None
    Xp = orc.layernorm(x.astype(np.float64), gamma.astype(np.float64), 0.0 if beta is None else beta.astype(np.float64), 1e-6, kind)
    want = dco.learn(Xp, bits, iters=50, alpha0=2.0)
    got = b.rq_dual_clip_learn(ctx, dev(x), bits, gamma=dev(gamma), beta=None if beta is None else dev(beta), norm_kind=kind,
                               eps=1e-6, iters=50, alpha0=2.0)
    torch.cuda.synchronize()
    _check(got, want, D)


def test_learnt_factors_feed_the_channel_bounds(rq):
    """clip_up / clip_lo are the contraction factors the calibration takes: bounds rebuilt from them match up / lo."""
    b, ctx = rq
    X = synth.make_rows_asymmetric(2000, 32, seed=1)
    got = b.rq_dual_clip_learn(ctx, dev(X), 4, iters=40, alpha0=1.0)
    torch.cuda.synchronize()
    lo, up = orc.channel_bounds(X.astype(np.float64), got["clip_up"].cpu().numpy(), got["clip_lo"].cpu().numpy())
    np.testing.assert_allclose(up, got["up"].cpu().numpy(), rtol=1e-6)
    np.testing.assert_allclose(lo, got["lo"].cpu().numpy(), rtol=1e-6)

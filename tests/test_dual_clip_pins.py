"""Pins for the dual-clipping learner's oracle (Section "Per-channel dual clipping"): the plain quantizer definition,
a hand derivation of the straight-through gradient evaluated element by element, the clipping loss it tends to at high
resolution, the textbook Adam recursion, and the symmetries the formulas have.  CPU only."""
import math

import numpy as np
import pytest

from oracle import dual_clip_oracle as dco
from oracle import repquant_oracle as orc
from paper_2402_05628_amd import synth


def _sig(a):
    return 1.0 / (1.0 + np.exp(-np.asarray(a, dtype=np.float64)))


@pytest.mark.parametrize("bits", [4, 6, 8])
def test_loss_is_the_error_of_the_plain_channelwise_quantizer(bits):
    """Eq. for s and z + the uniform quantizer of Section 'Efficient quantizers', with the contracted bounds."""
    X = synth.make_rows_asymmetric(300, 12, 1).astype(np.float64)
    g = np.random.default_rng(0)
    a1, a2 = g.uniform(-1, 4, 12), g.uniform(-1, 4, 12)
    lo, up = orc.channel_bounds(X, _sig(a1), _sig(a2))
    s, z = orc.qparams_from_bounds(lo, up, bits)
    xhat = orc.uniform_dequant(orc.uniform_quant(X, s[None, :], z[None, :], bits), s[None, :], z[None, :])
    want = ((X - xhat) ** 2).sum(axis=0)
    got = dco.loss_per_channel(X, a1, a2, bits)
    np.testing.assert_allclose(got, want, rtol=1e-12)
    total, _, _ = dco.loss_and_grad(X, a1, a2, bits)
    assert abs(total - want.sum()) <= 1e-12 * want.sum()


def _hand_gradient(x, a1, a2, bits):
    """One channel, element by element.  With u = x/s and zf = -lo/s both rounded straight-through,
    v = round(u) + round(zf), q = clip(v), x^ = s (q - round(zf)):
      d x^/d s  = (q - z) + [v inside] (lo - x)/s - lo/s,     d x^/d lo = 1 - [v inside]   (s held fixed),
      s = (up - lo)/qmax,  up = max * sig(a1),  lo = min * sig(a2)."""
    qmax = 2 ** bits - 1
    M, m = max(x), min(x)
    s1, s2 = 1 / (1 + math.exp(-a1)), 1 / (1 + math.exp(-a2))
    up, lo = M * s1, m * s2
    s = (up - lo) / qmax
    z = float(np.rint(-lo / s))
    dL_ds = dL_dlo = 0.0
    for xv in x:
        v = float(np.rint(xv / s)) + z
        inside = 1.0 if 0 <= v <= qmax else 0.0
        q = min(max(v, 0.0), float(qmax))
        xh = s * (q - z)
        gout = -2.0 * (xv - xh)
        dL_ds += gout * ((q - z) + inside * (lo - xv) / s - lo / s)
        dL_dlo += gout * (1.0 - inside)
    dL_dup = dL_ds / qmax
    dL_dlo_total = dL_dlo - dL_ds / qmax
    return dL_dup * M * s1 * (1 - s1), dL_dlo_total * m * s2 * (1 - s2)


@pytest.mark.parametrize("bits,alpha", [(4, (4.0, 4.0)), (4, (0.3, -0.4)), (6, (1.0, 2.5)), (3, (-1.0, 0.5))])
def test_autograd_gradient_equals_the_hand_derivation(bits, alpha):
    X = synth.make_rows_asymmetric(41, 5, 7).astype(np.float64)
    a1 = np.full(5, alpha[0])
    a2 = np.full(5, alpha[1])
    _, g1, g2 = dco.loss_and_grad(X, a1, a2, bits)
    for d in range(5):
        w1, w2 = _hand_gradient(list(X[:, d]), alpha[0], alpha[1], bits)
        assert g1[d] == pytest.approx(w1, rel=1e-9, abs=1e-12)
        assert g2[d] == pytest.approx(w2, rel=1e-9, abs=1e-12)


def test_fine_resolution_limit_is_the_gradient_of_the_clipping_error():
    """With 16-bit codes rounding hardly matters: the loss tends to sum (x - clip(x, lo, up))^2 and its gradient to
    d/d up = -2 sum_{x > up} (x - up), d/d lo = -2 sum_{x < lo} (x - lo), chained through the Sigmoid."""
    X = synth.make_rows_asymmetric(4000, 6, 3).astype(np.float64)
    a1, a2 = np.full(6, 0.5), np.full(6, 0.2)
    _, g1, g2 = dco.loss_and_grad(X, a1, a2, 16)
    M, m = X.max(axis=0), X.min(axis=0)
    up, lo = M * _sig(a1), m * _sig(a2)
    d_up = -2.0 * np.where(X > up, X - up, 0.0).sum(axis=0)
    d_lo = -2.0 * np.where(X < lo, X - lo, 0.0).sum(axis=0)
    np.testing.assert_allclose(g1, d_up * M * _sig(a1) * (1 - _sig(a1)), rtol=2e-3)
    np.testing.assert_allclose(g2, d_lo * m * _sig(a2) * (1 - _sig(a2)), rtol=2e-3)


def test_first_adam_step_moves_every_factor_by_the_learning_rate():
    """After bias correction the first Adam update is lr * g / (|g| + eps): lr against the sign of the gradient."""
    X = synth.make_rows_asymmetric(500, 9, 5).astype(np.float64)
    _, g1, g2 = dco.loss_and_grad(X, np.full(9, 1.0), np.full(9, 1.0), 4)
    r = dco.learn(X, 4, iters=1, lr=0.01, alpha0=1.0)
    np.testing.assert_allclose(r["alpha1"], 1.0 - 0.01 * np.sign(g1), atol=1e-7)
    np.testing.assert_allclose(r["alpha2"], 1.0 - 0.01 * np.sign(g2), atol=1e-7)


def test_three_iterations_follow_the_textbook_adam_recursion():
    """m <- b1 m + (1-b1) g, v <- b2 v + (1-b2) g^2, alpha <- alpha - lr (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps)."""
    X = synth.make_rows_asymmetric(300, 4, 11).astype(np.float64)
    b1, b2, eps, lr = 0.9, 0.999, 1e-8, 0.01
    a = np.full((2, 4), 0.5)
    m = np.zeros((2, 4))
    v = np.zeros((2, 4))
    for t in range(1, 4):
        _, g1, g2 = dco.loss_and_grad(X, a[0], a[1], 4)
        g = np.stack([g1, g2])
        m = b1 * m + (1 - b1) * g
        v = b2 * v + (1 - b2) * g * g
        a = a - lr * (m / (1 - b1 ** t)) / (np.sqrt(v / (1 - b2 ** t)) + eps)
    r = dco.learn(X, 4, iters=3, lr=lr, alpha0=0.5)
    np.testing.assert_allclose(r["alpha1"], a[0], rtol=0, atol=1e-12)
    np.testing.assert_allclose(r["alpha2"], a[1], rtol=0, atol=1e-12)
    np.testing.assert_allclose(r["loss"], dco.loss_per_channel(X, a[0], a[1], 4), rtol=1e-12)


@pytest.mark.parametrize("alpha0", [4.0, 0.0])
def test_mirror_symmetry(alpha0):
    """Negating X' swaps the roles of the two bounds: codes become qmax - q, X'^ changes sign, so the learnt factors
    swap and the losses stay."""
    X = synth.make_rows_asymmetric(400, 8, 2).astype(np.float64)
    r = dco.learn(X, 4, iters=30, alpha0=alpha0)
    n = dco.learn(-X, 4, iters=30, alpha0=alpha0)
    np.testing.assert_allclose(n["alpha1"], r["alpha2"], atol=1e-9)
    np.testing.assert_allclose(n["alpha2"], r["alpha1"], atol=1e-9)
    np.testing.assert_allclose(n["loss"], r["loss"], rtol=1e-9)
    np.testing.assert_allclose(n["up"], -r["lo"], rtol=1e-9)


def test_channels_are_independent_and_token_order_is_irrelevant():
    X = synth.make_rows_asymmetric(350, 10, 4).astype(np.float64)
    r = dco.learn(X, 4, iters=25, alpha0=1.0)
    sub = dco.learn(X[:, [7, 2, 3]], 4, iters=25, alpha0=1.0)
    np.testing.assert_allclose(sub["alpha1"], r["alpha1"][[7, 2, 3]], atol=1e-10)
    np.testing.assert_allclose(sub["alpha2"], r["alpha2"][[7, 2, 3]], atol=1e-10)
    perm = np.random.default_rng(1).permutation(350)
    p = dco.learn(X[perm], 4, iters=25, alpha0=1.0)
    np.testing.assert_allclose(p["alpha1"], r["alpha1"], atol=1e-9)
    np.testing.assert_allclose(p["loss"], r["loss"], rtol=1e-9)


def test_power_of_two_rescaling_changes_nothing_but_the_loss_scale():
    X = synth.make_rows_asymmetric(300, 6, 9).astype(np.float64)
    r = dco.learn(X, 4, iters=20, alpha0=1.0)
    k = dco.learn(8.0 * X, 4, iters=20, alpha0=1.0)
    np.testing.assert_allclose(k["alpha1"], r["alpha1"], atol=1e-7)      # only Adam's eps sees the scale
    np.testing.assert_allclose(k["loss"], 64.0 * r["loss"], rtol=1e-6)


def test_learning_lowers_the_error_on_channels_with_outliers_and_spares_constant_ones():
    X = synth.make_rows_asymmetric(3000, 12, 6).astype(np.float64)
    X[:, 5] = 0.75                                                      # max == min: nothing to learn
    r = dco.learn(X, 4, iters=100, alpha0=4.0)
    assert r["loss"].sum() < r["loss0"].sum()
    assert r["alpha1"][5] == 4.0 and r["alpha2"][5] == 4.0 and r["loss"][5] == 0.0
    # an Adam step is at most lr (1 - b1) / sqrt(1 - b2) long
    assert np.all(np.abs(r["alpha1"] - 4.0) <= 100 * 0.01 * 0.1 / math.sqrt(0.001))
    # a lone outlier on the upper side of a long channel: the bulk's rounding error outweighs the one clipped value,
    # so the upper bound contracts (alpha_1 falls) while the lower one, which only cuts into the bulk, relaxes
    g = np.random.default_rng(3)
    col = g.standard_normal(20000)
    col[17] = 12.0
    one = dco.learn(col[:, None], 4, iters=100, alpha0=0.0)
    assert one["alpha1"][0] < -0.5 < 0.3 < one["alpha2"][0] and one["loss"][0] < 0.75 * one["loss0"][0]

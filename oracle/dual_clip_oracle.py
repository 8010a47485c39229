"""CPU oracle for the per-channel dual-clipping learner -- TEST INFRASTRUCTURE ONLY.

Section "Per-channel dual clipping" of arXiv 2402.05628: two learnable vectors alpha_1, alpha_2 in R^D contract the
channel extremes of the LayerNorm activation X' through a Sigmoid (Eqs. for X'_up and X'_low); the contracted bounds
give the channel-wise scale and zero-point (Eq. for s and z); the factors are learnt by minimizing ||X' - X'^||^2
(the arg-min Eq.) with Adam, 100 iterations, learning rate 0.01 (Section "Implementation details").

Plain float64 PyTorch on the CPU: the forward pass is the printed formulas, the gradient comes from autograd, the
optimizer is torch.optim.Adam.  Nothing here is shared with the HIP library (which derives the gradient by hand and
keeps its own Adam); only tests/, smoke() and the cpu_baseline leg of the benchmark may import this module.

Readings of points the paper leaves open (each is a convention fixed here):
  * rounding has no gradient; the straight-through estimator (derivative 1) is used for both roundings -- of X'/s
    and of the zero-point -lo/s; the clip passes the gradient inside [0, 2^b - 1], end points included;
  * the loss is the plain sum of squares over the calibration batch (not a mean);
  * Adam with the usual defaults beta = (0.9, 0.999), eps = 1e-8, bias correction, no weight decay;
  * alpha_1 = alpha_2 = alpha0 at the start (a parameter; Sigmoid(4) = 0.982 keeps almost the whole range);
  * rounding is round-half-to-even; the zero-point used in the forward pass is the rounded one;
  * a channel whose extremes coincide (max == min) cannot be quantized by the formula (s = 0): it is left at alpha0
    with loss 0.
Parity unpinned by the paper (no printed value exists for any of these): the learnt factors themselves; the pins are
closed forms, symmetries and special cases (tests/test_dual_clip_pins.py).
"""
from __future__ import annotations

import numpy as np
import torch

F64 = torch.float64


def _round_ste(v):
    """Round-half-to-even in the forward pass, identity in the backward pass."""
    return v + (torch.round(v) - v).detach()


def fake_quant(Xp, up, lo, bits):
    """X'^ = s (clip(round(X'/s) + z, 0, 2^b - 1) - z) with s = (up - lo) / (2^b - 1), z = round(-lo / s), per channel."""
    qmax = float(2 ** bits - 1)
    s = (up - lo) / qmax
    z = _round_ste(-lo / s)
    q = torch.clamp(_round_ste(Xp / s) + z, 0.0, qmax)
    return s * (q - z)


def bounds(cmax, cmin, alpha1, alpha2):
    """Eqs. for X'_up and X'_low: the channel extremes contracted by Sigmoid(alpha)."""
    return cmax * torch.sigmoid(alpha1), cmin * torch.sigmoid(alpha2)


def loss_per_channel(Xp, alpha1, alpha2, bits):
    """Sum over the tokens of (X' - X'^)^2 for every channel; the objective of the arg-min Eq. is the sum of these."""
    Xp = torch.as_tensor(np.asarray(Xp, dtype=np.float64))
    a1 = torch.as_tensor(np.asarray(alpha1, dtype=np.float64))
    a2 = torch.as_tensor(np.asarray(alpha2, dtype=np.float64))
    up, lo = bounds(Xp.max(dim=0).values, Xp.min(dim=0).values, a1, a2)
    return ((Xp - fake_quant(Xp, up, lo, bits)) ** 2).sum(dim=0).numpy()


def loss_and_grad(Xp, alpha1, alpha2, bits):
    """Objective and its straight-through gradient with respect to alpha_1 and alpha_2 (autograd)."""
    Xp = torch.as_tensor(np.asarray(Xp, dtype=np.float64))
    a1 = torch.tensor(np.asarray(alpha1, dtype=np.float64), requires_grad=True)
    a2 = torch.tensor(np.asarray(alpha2, dtype=np.float64), requires_grad=True)
    up, lo = bounds(Xp.max(dim=0).values, Xp.min(dim=0).values, a1, a2)
    loss = ((Xp - fake_quant(Xp, up, lo, bits)) ** 2).sum()
    loss.backward()
    return float(loss.detach()), a1.grad.numpy(), a2.grad.numpy()


def learn(Xp, bits, iters=100, lr=0.01, alpha0=4.0):
    """Learn the clipping factors of every channel of X' [T, D].

    Returns a dict: alpha1, alpha2 (float64 [D]), clip_up = Sigmoid(alpha1), clip_lo = Sigmoid(alpha2), up, lo (the
    contracted bounds), loss0 and loss (per-channel sum of squares before the first and after the last update).
    """
    Xp = torch.as_tensor(np.asarray(Xp, dtype=np.float64))
    D = Xp.shape[1]
    cmax, cmin = Xp.max(dim=0).values, Xp.min(dim=0).values
    live = cmax > cmin                                   # channels the formula can quantize
    Xl, cmaxl, cminl = Xp[:, live], cmax[live], cmin[live]
    a1 = torch.full((int(live.sum()),), float(alpha0), dtype=F64, requires_grad=True)
    a2 = torch.full((int(live.sum()),), float(alpha0), dtype=F64, requires_grad=True)
    opt = torch.optim.Adam([a1, a2], lr=lr)

    def channel_loss():
        up, lo = bounds(cmaxl, cminl, a1, a2)
        return ((Xl - fake_quant(Xl, up, lo, bits)) ** 2).sum(dim=0)

    loss0 = channel_loss().detach().clone()
    for _ in range(iters):
        opt.zero_grad()
        channel_loss().sum().backward()
        opt.step()
    loss = channel_loss().detach()

    def full(v, fill):
        out = np.full(D, fill, dtype=np.float64)
        out[live.numpy()] = v.detach().numpy()
        return out

    alpha1, alpha2 = full(a1, alpha0), full(a2, alpha0)
    sg = lambda a: 1.0 / (1.0 + np.exp(-a))
    return dict(alpha1=alpha1, alpha2=alpha2, clip_up=sg(alpha1), clip_lo=sg(alpha2),
                up=cmax.numpy() * sg(alpha1), lo=cmin.numpy() * sg(alpha2),
                loss0=full(loss0, 0.0), loss=full(loss, 0.0))

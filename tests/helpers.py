"""Shared glue for the GPU parity tests: oracle-side preparation of inputs, comparison bars."""
import dataclasses

import numpy as np
import torch

from oracle import repquant_oracle as orc

CODE_MISMATCH_BUDGET = 1e-4     # fraction of elements allowed to differ, and then by one code only


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def folded_ln_case(x, seed, bits, kind, dual_clip=False):
    """Channel-wise calibration + fold done by the oracle; returns float32/ints as stored on the ABI."""
    g = np.random.default_rng(seed)
    D = x.shape[1]
    gamma = g.normal(1.0, 0.1, size=D).astype(np.float32)
    beta = (g.normal(0.0, 0.1, size=D).astype(np.float32) if kind == orc.NORM_LAYERNORM else np.zeros(D, np.float32))
    Xp = orc.layernorm(x, gamma, beta, 1e-6, kind)
    cu = g.uniform(0.8, 1.0, size=D) if dual_clip else None
    cl = g.uniform(0.8, 1.0, size=D) if dual_clip else None
    lo, up = orc.channel_bounds(Xp, cu, cl)
    s_ch, _ = orc.qparams_from_bounds(lo, up, bits)
    s_ch = s_ch.astype(np.float32)
    z_ch = np.rint(-lo / s_ch.astype(np.float64)).astype(np.int64)
    W = np.zeros((1, D), np.float32)
    f = orc.reparam_fold(s_ch, z_ch, gamma, beta, W, np.zeros(1, np.float32))
    return dict(gamma=gamma, beta=beta, s_ch=s_ch, z_ch=z_ch, gamma_t=f["gamma_t"].astype(np.float32),
                beta_t=f["beta_t"].astype(np.float32), s_t=np.float32(f["s_t"]), z_t=int(f["z_t"]))


def assert_codes_close(got, want, what, budget=CODE_MISMATCH_BUDGET):
    got = np.asarray(got).astype(np.int64)
    want = np.asarray(want).astype(np.int64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    diff = np.abs(got - want)
    frac = float(np.mean(diff != 0)) if diff.size else 0.0
    assert diff.max(initial=0) <= 1, "%s: codes differ by more than one (max %d)" % (what, diff.max())
    assert frac <= budget, "%s: %.3g of the codes differ (budget %.1g)" % (what, frac, budget)
    return frac


def assert_float_close(got, want, what, rtol=1e-3):
    """|d| <= rtol * max(|ref|, rtol * max|ref|) element-wise, and max|d| / max|ref| <= rtol."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    ref = np.abs(want).max()
    d = np.abs(got - want)
    assert d.max() <= rtol * ref, "%s: max abs err %.3g vs ref max %.3g" % (what, d.max(), ref)
    bar = rtol * np.maximum(np.abs(want), 1e-3 * ref)
    bad = float(np.mean(d > bar))
    assert bad == 0.0, "%s: %.3g of elements beyond element-wise bar" % (what, bad)


def cfg_dict(cfg):
    return dataclasses.asdict(cfg)

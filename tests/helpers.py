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


# ---- numpy-side packing of oracle weight codes into the library's storage formats (independent of the product's
#      own packer, so it also checks the layout the header documents) --------------------------------------------
W_I8_BAKED, W_I8_CENTERED, W_U4 = 0, 1, 2


def pack_u4(codes):
    """[N, K] codes 0..15 -> [N, K/2] bytes: in each group of 8 codes, byte i = code[i] | code[i+4] << 4."""
    N, K = codes.shape
    g = codes.reshape(N, K // 8, 8).astype(np.uint8)
    return (g[:, :, 0:4] | (g[:, :, 4:8] << 4)).reshape(N, K // 2)


def gate_up_interleave(arr, Dm):
    """rows [gate(0..Dm-1); up(0..Dm-1)] -> groups of 32 gate rows followed by the matching 32 up rows."""
    gate, upp = arr[:Dm], arr[Dm:2 * Dm]
    sh = (Dm // 32, 32) + arr.shape[1:]
    return np.stack([gate.reshape(sh), upp.reshape(sh)], axis=1).reshape(arr.shape)


def lin_to_device(lin, bits, gated_Dm=0):
    """Oracle linear dict (codes, s_w, z_w, bias) -> dict of device tensors in the library's format."""
    codes, s_w, z_w = np.asarray(lin["codes"]), np.asarray(lin["s_w"], np.float32), np.asarray(lin["z_w"], np.int64)
    bias = lin.get("bias")
    bias = np.zeros(codes.shape[0], np.float32) if bias is None else np.asarray(bias, np.float32)
    if gated_Dm:
        codes, s_w, z_w, bias = (gate_up_interleave(a, gated_Dm) for a in (codes, s_w, z_w, bias))
    colsum = (codes - z_w[:, None]).sum(1)
    if bits == 4:
        fmt, w = W_U4, pack_u4(codes)
    elif bits == 8:
        fmt, w = W_I8_CENTERED, (codes - 128).astype(np.int8)
    else:
        fmt, w = W_I8_BAKED, (codes - z_w[:, None]).astype(np.int8)
    return dict(w=dev(w), s_w=dev(s_w), z_w=dev(z_w.astype(np.int32)), colsum_w=dev(colsum.astype(np.int32)),
                bias=dev(bias), N=codes.shape[0], K=codes.shape[1], bits=bits, format=fmt)


def block_to_device(P):
    """Oracle block parameters -> the dict paper_2402_05628_amd.binding.Block consumes."""
    c = P["cfg"]
    gated = c["act"] == orc.ACT_SILU_GATED
    out = {}
    for k in ("ln1", "ln2"):
        out[k] = dict(gamma_t=dev(P[k]["gamma_t"]), beta_t=dev(P[k]["beta_t"]), s=float(P[k]["s"]), z=int(P[k]["z"]))
    for k in ("qkv", "proj", "fc2"):
        out[k] = lin_to_device(P[k], c["bits_w"])
    out["fc1"] = lin_to_device(P["fc1"], c["bits_w"], c["Dm"] if gated else 0)
    for k in ("s_q", "s_k", "s_v", "s_o", "s_h", "s_log", "z_q", "z_k", "z_v", "z_o", "z_h"):
        out[k] = P[k]
    out["rel_bias"] = None if P.get("rel_bias") is None else dev(P["rel_bias"])
    return out


def random_linear(g, N, K, bits):
    """Random weight codes with per-channel scale / zero-point, as an oracle linear dict."""
    return dict(codes=g.integers(0, 2 ** bits, size=(N, K)), s_w=g.uniform(1e-3, 5e-3, size=N).astype(np.float32),
                z_w=g.integers(0, 2 ** bits, size=N), bias=g.normal(0, 0.5, size=N).astype(np.float32))


def float_block(raw, cfg):
    """The block without any quantization (float64): the reference that quantization error is measured against."""
    from oracle import repquant_oracle as orc
    X = raw["x"].astype(np.float64)
    D, H, seq, batch = cfg.D, cfg.H, cfg.seq, cfg.batch
    dh = D // H
    f = lambda k: 0.0 if raw.get(k) is None else raw[k].astype(np.float64)
    a = orc.layernorm(X, raw["ln1_gamma"].astype(np.float64), f("ln1_beta"), cfg.eps, cfg.norm)
    qkv = a @ raw["w_qkv"].astype(np.float64).T + f("b_qkv")
    out = np.empty_like(X)
    for b in range(batch):
        r = slice(b * seq, (b + 1) * seq)
        for h in range(H):
            L = qkv[r, h * dh:(h + 1) * dh] @ qkv[r, D + h * dh:D + (h + 1) * dh].T / np.sqrt(dh)
            if raw.get("rel_bias") is not None:
                L = L + raw["rel_bias"][h].astype(np.float64)
            if cfg.mask == orc.MASK_CAUSAL:
                L = np.where(np.tril(np.ones((seq, seq), dtype=bool)), L, -np.inf)
            out[r, h * dh:(h + 1) * dh] = orc.softmax_rows(L) @ qkv[r, 2 * D + h * dh:2 * D + (h + 1) * dh]
    xbar = out @ raw["w_proj"].astype(np.float64).T + f("b_proj") + X
    a2 = orc.layernorm(xbar, raw["ln2_gamma"].astype(np.float64), f("ln2_beta"), cfg.eps, cfg.norm)
    hid = orc.mlp_activation(a2 @ raw["w_fc1"].astype(np.float64).T + f("b_fc1"), cfg.act, cfg.Dm)
    return hid @ raw["w_fc2"].astype(np.float64).T + f("b_fc2") + xbar

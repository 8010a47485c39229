"""Preparation kernels against the oracle: fold, weight quantization + packing, row sums, min/max."""
import numpy as np
import pytest
import torch

from oracle import repquant_oracle as orc
from paper_2402_05628_amd import synth
from tests.helpers import dev, gate_up_interleave, pack_u4

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rq():
    from paper_2402_05628_amd import binding
    return binding, binding.Context(0)


def _ulp_close(got, want64):
    """got (float32) equals float32(want64) up to one unit in the last place."""
    w = want64.astype(np.float32)
    return np.all(np.abs(got.astype(np.float64) - w.astype(np.float64)) <= np.spacing(np.abs(w)).astype(np.float64))


@pytest.mark.parametrize("D,D_out", [(384, 1152), (128, 384), (4096, 64), (52, 8)])
def test_reparam_fold(rq, D, D_out):
    b, ctx = rq
    g = np.random.default_rng(D)
    s_ch = np.exp(g.normal(size=D)).astype(np.float32) * np.float32(0.01)
    z_ch = g.integers(0, 256, size=D)
    gamma, beta = g.normal(1, 0.1, size=D).astype(np.float32), g.normal(0, 0.1, size=D).astype(np.float32)
    W, bb = g.normal(0, 0.02, size=(D_out, D)).astype(np.float32), g.normal(0, 0.02, size=D_out).astype(np.float32)
    f = orc.reparam_fold(s_ch, z_ch, gamma, beta, W, bb)
    out = b.rq_reparam_fold(ctx, dev(s_ch), dev(z_ch.astype(np.int32)), dev(gamma), dev(beta), dev(W), dev(bb), s_log=0.7)
    assert int(out["z_tilde"].item()) == f["z_t"]
    assert _ulp_close(out["s_tilde"].cpu().numpy(), np.array([f["s_t"]]))
    for k in ("gamma_t", "beta_t", "W_t"):
        assert _ulp_close(out[k].cpu().numpy(), f[k]), k
    # b~ is a length-D dot product: compare with the error bound of the float32 store plus summation order
    bt = out["b_t"].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(bt - f["b_t"]) <= 2e-7 * np.abs(f["b_t"]) + 1e-12 * np.abs(W).sum(1).max())
    pair = out["s_log_pair"].cpu().numpy()
    assert pair[0] == np.float32(0.7) and _ulp_close(pair[1:], np.array([np.float64(np.float32(0.7)) * np.sqrt(2.0)]))
    # no beta / no bias inputs (RMSNorm, bias-free Linear): the folded shift is still materialised
    f0 = orc.reparam_fold(s_ch, z_ch, gamma, np.zeros(D), W, np.zeros(D_out))
    out0 = b.rq_reparam_fold(ctx, dev(s_ch), dev(z_ch.astype(np.int32)), dev(gamma), None, dev(W), None)
    assert _ulp_close(out0["beta_t"].cpu().numpy(), f0["beta_t"])
    assert np.abs(out0["b_t"].cpu().numpy() - f0["b_t"]).max() <= 2e-7 * np.abs(f0["b_t"]).max() + 1e-9


@pytest.mark.parametrize("N,K,bits", [(96, 384, 8), (64, 768, 4), (40, 128, 6), (8, 11008, 4), (33, 64, 4)])
def test_weight_quant_pack(rq, N, K, bits):
    b, ctx = rq
    g = np.random.default_rng(N + K)
    W = g.normal(0, 0.02, size=(N, K)).astype(np.float32)
    bias = g.normal(size=N).astype(np.float32)
    codes, s_w, z_w = orc.weight_quant(W, bits)
    out = b.rq_weight_quant_pack(ctx, dev(W), dev(bias), bits)
    assert np.array_equal(out["s_w"].cpu().numpy(), s_w)
    assert np.array_equal(out["z_w"].cpu().numpy(), z_w)
    assert np.array_equal(out["colsum_w"].cpu().numpy(), (codes - z_w[:, None]).sum(1))
    assert np.array_equal(out["bias"].cpu().numpy(), bias)
    w = out["w"].cpu().numpy()
    if bits == 4:
        assert np.array_equal(w, pack_u4(codes))
    elif bits == 8:
        assert np.array_equal(w.astype(np.int64) + 128, codes)
    else:
        assert np.array_equal(w.astype(np.int64) + z_w[:, None], codes)


@pytest.mark.parametrize("bits", [4, 6, 8])
def test_weight_quant_pack_rows_of_one_sign(rq, bits):
    """All-positive, all-negative and all-zero rows: the zero-point stays a code (0, 2^b - 1, 0), and a 4-bit GEMM over
    such rows gives the exact accumulators (the packed operands subtract the zero-point byte-wise)."""
    b, ctx = rq
    g = np.random.default_rng(bits)
    N, K, M = 64, 128, 96
    W = g.normal(0, 0.02, size=(N, K)).astype(np.float32)
    W[0::4] = np.abs(W[0::4]) + np.float32(0.01)
    W[1::4] = -np.abs(W[1::4]) - np.float32(0.01)
    W[2] = 0
    codes, s_w, z_w = orc.weight_quant(W, bits)
    qmax = 2 ** bits - 1
    assert np.all(z_w[0::4] == 0) and np.all(z_w[1::4] == qmax) and z_w[2] == 0 and s_w[2] == 1.0
    out = b.rq_weight_quant_pack(ctx, dev(W), None, bits)
    assert np.array_equal(out["s_w"].cpu().numpy(), s_w)
    assert np.array_equal(out["z_w"].cpu().numpy(), z_w)
    assert np.array_equal(out["colsum_w"].cpu().numpy(), (codes - z_w[:, None]).sum(1))
    if bits == 4:
        assert np.array_equal(out["w"].cpu().numpy(), pack_u4(codes))
    # the GEMM on these weights: true accumulators
    bits_a = 4 if bits == 4 else 8
    qa = 2 ** bits_a - 1
    z_a = qa // 2
    A = g.integers(0, qa + 1, size=(M, K))
    off = b.store_offset(bits_a, z_a)
    acc = torch.zeros((M, N), dtype=torch.int32, device="cuda")
    stored = (A - off).astype(np.int8)
    rowsum = dev(stored.astype(np.int64).sum(axis=1).astype(np.int32)) if out["format"] == b.W_I8_CENTERED else None
    b.rq_qgemm(ctx, dev(stored), off, z_a, 0.1, out, out_acc=acc, rowsum_a=rowsum)
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), orc.int_matmul_nt(A - z_a, codes - z_w[:, None]))


def test_weight_quant_pack_gate_up_interleave(rq):
    b, ctx = rq
    Dm, K = 64, 128
    g = np.random.default_rng(3)
    W = g.normal(0, 0.02, size=(2 * Dm, K)).astype(np.float32)
    codes, s_w, z_w = orc.weight_quant(W, 4)
    out = b.rq_weight_quant_pack(ctx, dev(W), None, 4, gate_up_rows=Dm)
    assert np.array_equal(out["w"].cpu().numpy(), pack_u4(gate_up_interleave(codes, Dm)))
    assert np.array_equal(out["s_w"].cpu().numpy(), gate_up_interleave(s_w, Dm))
    assert np.array_equal(out["z_w"].cpu().numpy(), gate_up_interleave(z_w, Dm))
    assert np.all(out["bias"].cpu().numpy() == 0)


def test_rowsum_and_minmax(rq):
    b, ctx = rq
    g = np.random.default_rng(4)
    A = g.integers(-128, 128, size=(301, 768)).astype(np.int8)
    rs = torch.zeros(301, dtype=torch.int32, device="cuda")
    b.rq_rowsum_i8(ctx, dev(A), rs)
    assert np.array_equal(rs.cpu().numpy(), A.astype(np.int64).sum(1))
    v = g.normal(size=(513, 300)).astype(np.float32)
    mm = b.rq_minmax_f32(ctx, dev(v)[:, :257]).cpu().numpy()
    assert mm[0] == v[:, :257].min() and mm[1] == v[:, :257].max()


@pytest.mark.parametrize("T,D,kind", [(333, 384, 0), (100, 4096, 1), (50, 128, 0)])
def test_ln_channel_minmax(rq, T, D, kind):
    b, ctx = rq
    x = synth.make_rows(T, D, seed=D)
    g = np.random.default_rng(D)
    gamma, beta = g.normal(1, 0.1, size=D).astype(np.float32), g.normal(0, 0.1, size=D).astype(np.float32)
    Xp = orc.layernorm(x, gamma, beta, 1e-6, kind)
    cmin, cmax = b.rq_ln_channel_minmax(ctx, dev(x), dev(gamma), dev(beta), norm_kind=kind)
    assert np.allclose(cmin.cpu().numpy(), Xp.min(0), rtol=1e-11, atol=1e-12)
    assert np.allclose(cmax.cpu().numpy(), Xp.max(0), rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("T,D,kind,q", [(333, 384, 0, (0.01, 0.99)), (1000, 128, 1, (0.001, 0.9999)), (50, 64, 0, (0.0, 1.0)),
                                        (12608, 48, 0, (0.00001, 0.99999)), (7, 8, 0, (0.5, 0.5)), (1, 4, 0, (0.1, 0.9)),
                                        (2, 4, 1, (0.3, 0.7))])
def test_ln_channel_percentile(rq, T, D, kind, q):
    """Percentile calibration bounds (exact selection + linear interpolation) against numpy's definition."""
    b, ctx = rq
    print("case", T, D, kind, q, flush=True)
    x = synth.make_rows(T, D, seed=D + 1)
    x[: T // 3, 2] = x[0, 2]                                   # repeated values in one channel
    g = np.random.default_rng(D)
    gamma, beta = g.normal(1, 0.1, size=D).astype(np.float32), g.normal(0, 0.1, size=D).astype(np.float32)
    Xp = orc.layernorm(x, gamma, beta, 1e-6, kind)
    want_lo, want_hi = orc.channel_percentile_bounds(Xp, *q)
    lo, hi, _ = b.rq_ln_channel_percentile(ctx, dev(x), q[0], q[1], dev(gamma), dev(beta), norm_kind=kind)
    torch.cuda.synchronize()
    scale = np.abs(Xp).max(axis=0)
    assert np.all(np.abs(lo.cpu().numpy() - want_lo) <= 1e-11 * scale)
    assert np.all(np.abs(hi.cpu().numpy() - want_hi) <= 1e-11 * scale)
    # without a normalization the input is taken as X' itself
    lo2, hi2, _ = b.rq_ln_channel_percentile(ctx, dev(x), q[0], q[1])
    torch.cuda.synchronize()
    w_lo, w_hi = orc.channel_percentile_bounds(x.astype(np.float64), *q)
    assert np.allclose(lo2.cpu().numpy(), w_lo, rtol=1e-13, atol=0) and np.allclose(hi2.cpu().numpy(), w_hi, rtol=1e-13, atol=0)

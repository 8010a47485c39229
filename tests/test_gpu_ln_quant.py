"""rq_ln_quant against the oracle: codes equal except at ties (<= 1e-4 of elements, off by one)."""
import numpy as np
import pytest
import torch

from oracle import repquant_oracle as orc
from paper_2402_05628_amd import synth
from tests.helpers import assert_codes_close, dev, folded_ln_case

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rq():
    from paper_2402_05628_amd import binding
    return binding, binding.Context(0)


@pytest.mark.parametrize("T,D", [(333, 384), (1031, 768), (517, 128), (130, 1024), (67, 4096), (45, 100), (9, 8192),
                                 (1, 768), (700, 52)])
@pytest.mark.parametrize("bits", [4, 6, 8])
@pytest.mark.parametrize("kind", [orc.NORM_LAYERNORM, orc.NORM_RMSNORM])
def test_ln_quant_matches_oracle(rq, T, D, bits, kind):
    b, ctx = rq
    print("case", T, D, bits, kind, flush=True)
    xc = synth.make_rows(T + 40, D, seed=T + D + bits)       # calibrate on more rows than are run
    p = folded_ln_case(xc, seed=bits + D, bits=bits, kind=kind, dual_clip=(D % 3 == 0))
    x = np.ascontiguousarray(xc[:T])
    want = orc.ln_quant(x, p["gamma_t"], p["beta_t"], p["s_t"], p["z_t"], bits, 1e-6, kind)
    q = torch.full((T, D), 77, dtype=torch.int8, device="cuda")
    rs = torch.zeros(T, dtype=torch.int32, device="cuda")
    off = b.rq_ln_quant(ctx, dev(x), dev(p["gamma_t"]), dev(p["beta_t"]), float(p["s_t"]), p["z_t"], bits, q,
                        norm_kind=kind, eps=1e-6, rowsum=rs)
    torch.cuda.synchronize()
    got = q.cpu().numpy().astype(np.int64) + off
    assert got.min() >= 0 and got.max() <= 2 ** bits - 1
    assert_codes_close(got, want, "ln_quant T=%d D=%d b=%d" % (T, D, bits))
    assert np.array_equal(rs.cpu().numpy(), q.cpu().numpy().astype(np.int64).sum(1))
    # the layer-wise codes are the channel-wise codes (the paper's invariance claim), up to float32 storage of the fold
    q_def = orc.ln_quant_channelwise(x, p["gamma"], p["beta"], p["s_ch"], p["z_ch"], bits, 1e-6, kind)
    assert np.abs(got - q_def).max() <= 1 and np.mean(got != q_def) < 2e-3


@pytest.mark.parametrize("T,D", [(24601, 768), (24700, 1024), (24603, 520), (24580, 2048), (24599, 1300), (24601, 512)])
@pytest.mark.parametrize("bits,kind", [(4, orc.NORM_LAYERNORM), (8, orc.NORM_RMSNORM)])
def test_ln_quant_many_rows_through_the_lds_ring(rq, T, D, bits, kind):
    """Enough rows for the LDS-ring kernel (rows of 2, 3, 4, 6 and 8 KiB, ragged widths): every row's codes lie in range and
    its row sum matches its codes; the first, the last and 400 scattered rows (first turns, steady state and the ragged
    last turns of the wavefronts) against the oracle."""
    b, ctx = rq
    print("case", T, D, bits, kind, flush=True)
    xc = synth.make_rows(2000, D, seed=D + bits)
    p = folded_ln_case(xc, seed=bits + D, bits=bits, kind=kind, dual_clip=(D % 3 == 0))
    g = np.random.default_rng(T + D)
    x = xc[g.integers(0, 2000, size=T)] * g.uniform(0.5, 1.5, size=(T, 1)).astype(np.float32) + g.normal(0, 0.05, size=(T, 1)).astype(np.float32)
    x = np.ascontiguousarray(x.astype(np.float32))
    q = torch.full((T, D), 77, dtype=torch.int8, device="cuda")
    rs = torch.zeros(T, dtype=torch.int32, device="cuda")
    off = b.rq_ln_quant(ctx, dev(x), dev(p["gamma_t"]), dev(p["beta_t"]), float(p["s_t"]), p["z_t"], bits, q,
                        norm_kind=kind, eps=1e-6, rowsum=rs)
    torch.cuda.synchronize()
    qh = q.cpu().numpy().astype(np.int64)
    got = qh + off
    assert got.min() >= 0 and got.max() <= 2 ** bits - 1
    assert np.array_equal(rs.cpu().numpy(), qh.sum(1))
    rows = np.unique(np.concatenate([np.arange(300), np.arange(T - 300, T), g.integers(0, T, size=400)]))
    want = orc.ln_quant(x[rows], p["gamma_t"], p["beta_t"], p["s_t"], p["z_t"], bits, 1e-6, kind)
    assert_codes_close(got[rows], want, "ln_quant ring T=%d D=%d b=%d" % (T, D, bits))


@pytest.mark.parametrize("T", [50, 24700])
def test_ln_quant_strided_rows_and_no_beta(rq, T):
    b, ctx = rq
    D = 384
    x = synth.make_rows(T, D + 64, seed=3)
    p = folded_ln_case(x[:, :D], seed=1, bits=8, kind=orc.NORM_RMSNORM)
    xd = dev(x)
    q = torch.zeros((T, D + 32), dtype=torch.int8, device="cuda")
    off = b.rq_ln_quant(ctx, xd[:, :D], dev(p["gamma_t"]), None, float(p["s_t"]), p["z_t"], 8, q[:, :D],
                        norm_kind=orc.NORM_RMSNORM)
    want = orc.ln_quant(x[:, :D], p["gamma_t"], np.zeros(D), p["s_t"], p["z_t"], 8, 1e-6, orc.NORM_RMSNORM)
    assert_codes_close(q[:, :D].cpu().numpy().astype(np.int64) + off, want, "strided")
    assert torch.all(q[:, D:] == 0)

"""GPU parity of rq_gptq_quant_pack (Algorithm 1, weight-quantization step) against the float64 elimination-form oracle.
Both sides are float64; they differ in the formulation (Cholesky factor in blocks vs explicit inverse-Hessian
elimination), so updated weights agree to ~1e-10 and a code can differ only next to a rounding tie -- the budget below
allows one such output channel (a flipped code changes the rest of that channel's row, nothing else)."""
import numpy as np
import pytest
import torch

from oracle import gptq_oracle as gq
from paper_2402_05628_amd import synth
from tests.helpers import dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rq():
    from paper_2402_05628_amd import binding as b
    ctx = b.Context()
    yield b, ctx
    ctx.close()


def _inputs(N, K, T, bits_a, seed):
    """Correlated calibration activations (shared factors across channels) and small random weights."""
    g = np.random.Generator(np.random.Philox(key=0x6B70 + seed))
    W = (g.standard_normal((N, K)) * 0.02).astype(np.float32)
    F = g.standard_normal((T, 8))
    X = F @ g.standard_normal((8, K)) * 0.5 + g.standard_normal((T, K))
    qmax = 2 ** bits_a - 1
    z_a = qmax // 2 + 1
    codes = np.clip(np.rint(X * (qmax / 8.0)) + z_a, 0, qmax).astype(np.int64)
    return W, codes, z_a


def _unpack(b, out, bits):
    w = out["w"].cpu().numpy()
    z = out["z_w"].cpu().numpy().astype(np.int64)
    if out["format"] == b.W_U4:
        N, K2 = w.shape
        g = w.reshape(N, K2 // 4, 4)
        lo, hi = g & 0xF, g >> 4
        return np.concatenate([lo, hi], axis=2).reshape(N, K2 * 2).astype(np.int64)
    off = 128 if out["format"] == b.W_I8_CENTERED else z[:, None]
    return w.astype(np.int64) + off


def _check(b, out, want, bits, max_bad_rows):
    codes, s, z = want
    got = _unpack(b, out, bits)
    assert np.array_equal(out["s_w"].cpu().numpy(), s)
    assert np.array_equal(out["z_w"].cpu().numpy().astype(np.int64), z)
    bad_rows = np.flatnonzero((got != codes).any(axis=1))
    assert len(bad_rows) <= max_bad_rows, (len(bad_rows), bad_rows[:8])
    good = np.setdiff1d(np.arange(codes.shape[0]), bad_rows)
    assert np.array_equal(out["colsum_w"].cpu().numpy()[good], (codes - z[:, None]).sum(axis=1)[good])
    return len(bad_rows)


@pytest.mark.parametrize("N,K,T,bits_w,bits_a", [(96, 128, 500, 4, 4), (200, 192, 1000, 4, 8), (64, 64, 100, 3, 4), (130, 256, 777, 8, 8),
                                                  (33, 320, 64, 6, 6), (1, 64, 1, 4, 4), (17, 64, 3, 2, 8),
                                                  (40, 1152, 300, 4, 4),    # 18 panels / sweep blocks: every wavefront of the sweep gets several column chunks
                                                  (24, 1600, 200, 4, 4),    # 25 panels: the first steps have more trailing tiles than CUs (separate launches)
                                                  (13, 2048, 150, 4, 4)])   # rows this long: 8 channels per workgroup of the sweep
def test_gptq_matches_oracle(rq, N, K, T, bits_w, bits_a):
    b, ctx = rq
    print("case", N, K, T, bits_w, bits_a, flush=True)
    W, codes_a, z_a = _inputs(N, K, T, bits_a, seed=N + K)
    codes_a[:, 5] = z_a                                   # a dead input channel
    off = z_a if bits_a < 8 else 128
    A = dev((codes_a - off).astype(np.int8))
    want = gq.gptq(W, codes_a - z_a, bits_w)
    out = b.rq_gptq_quant_pack(ctx, dev(W), None, bits_w, A, off, z_a)
    torch.cuda.synchronize()
    _check(b, out, want, bits_w, max_bad_rows=1)


def test_gptq_gated_rows_and_bias(rq):
    b, ctx = rq
    Dm, K, T = 64, 128, 300
    W, codes_a, z_a = _inputs(2 * Dm, K, T, 4, seed=9)
    bias = np.arange(2 * Dm, dtype=np.float32)
    want = gq.gptq(W, codes_a - z_a, 4)
    out = b.rq_gptq_quant_pack(ctx, dev(W), dev(bias), 4, dev((codes_a - z_a).astype(np.int8)), z_a, z_a, gate_up_rows=Dm)
    torch.cuda.synchronize()
    n = np.arange(2 * Dm)
    j = np.where(n < Dm, n, n - Dm)
    r = (j // 32) * 64 + np.where(n < Dm, 0, 32) + j % 32
    perm = np.empty(2 * Dm, dtype=np.int64)
    perm[r] = n                                           # output row r holds input row perm[r]
    _check(b, out, (want[0][perm], want[1][perm], want[2][perm]), 4, max_bad_rows=1)
    assert np.array_equal(out["bias"].cpu().numpy(), bias[perm])


@pytest.mark.timeout(300)
def test_gptq_full_size_vit_b_qkv(rq):
    """The benchmark's launch: QKV weights of the ViT-B block (2304 x 768) against 12 608 tokens of 4-bit codes."""
    b, ctx = rq
    N, K, T = 2304, 768, 12608
    print("case full size", N, K, T, flush=True)
    W, codes_a, z_a = _inputs(N, K, T, 4, seed=1)
    want = gq.gptq(W, codes_a - z_a, 4)
    out = b.rq_gptq_quant_pack(ctx, dev(W), None, 4, dev((codes_a - z_a).astype(np.int8)), z_a, z_a)
    torch.cuda.synchronize()
    bad = _check(b, out, want, 4, max_bad_rows=2)
    print("  rows with a differing code:", bad, flush=True)
    got = _unpack(b, out, 4)
    e_gpu = gq.output_error(W[:64], got[:64], want[1][:64], want[2][:64], codes_a - z_a)
    e_orc = gq.output_error(W[:64], want[0][:64], want[1][:64], want[2][:64], codes_a - z_a)
    assert abs(e_gpu - e_orc) <= 1e-6 * e_orc

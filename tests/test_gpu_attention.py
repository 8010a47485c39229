"""Q.K^T accumulators (bit-exact), Softmax-log2 codes and shift-dequantized P.V against the oracle."""
import math

import numpy as np
import pytest
import torch

from oracle import repquant_oracle as orc
from tests.helpers import assert_codes_close, assert_float_close, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rq():
    from paper_2402_05628_amd import binding
    return binding, binding.Context(0)


def _ld(n):
    return (n + 15) // 16 * 16


@pytest.mark.parametrize("batch,H,seq,dh,bits,causal", [(2, 3, 197, 64, 4, False), (1, 2, 49, 32, 6, False), (3, 2, 257, 64, 4, False),
                                                        (1, 2, 300, 128, 8, True), (2, 2, 64, 64, 8, False), (1, 1, 1, 32, 8, False),
                                                        (1, 2, 33, 64, 8, True)])
def test_qk_accumulators_bit_exact(rq, batch, H, seq, dh, bits, causal):
    b, ctx = rq
    print("case", batch, H, seq, dh, bits, causal, flush=True)
    g = np.random.default_rng(seq + dh + bits)
    D = H * dh
    codes = g.integers(0, 2 ** bits, size=(batch * seq, 3 * D))
    z_q, z_k = int(g.integers(0, 2 ** bits)), int(g.integers(0, 2 ** bits))
    offq, offk = b.store_offset(bits, z_q), b.store_offset(bits, z_k)
    st = codes.copy()
    st[:, :D] -= offq
    st[:, D:2 * D] -= offk
    st[:, 2 * D:] -= 128 if bits == 8 else 0
    qkv = dev(st.astype(np.int8))
    ld = _ld(seq)
    acc = torch.full((batch * H, seq, ld), 12345, dtype=torch.int32, device="cuda")
    b.rq_qk(ctx, qkv, batch, seq, H, dh, 0, D, offq, z_q, offk, z_k, acc, ld, causal=causal)
    got = acc.cpu().numpy()
    for bi in range(batch):
        r = slice(bi * seq, (bi + 1) * seq)
        for h in range(H):
            want = orc.int_matmul_nt(codes[r, h * dh:(h + 1) * dh] - z_q, codes[r, D + h * dh:D + (h + 1) * dh] - z_k)
            sub = got[bi * H + h, :, :seq]
            if causal:
                m = np.tril(np.ones((seq, seq), bool))
                assert np.array_equal(sub[m], want[m])
            else:
                assert np.array_equal(sub, want)


@pytest.mark.parametrize("G,H,N,bits,bias,causal", [(6, 3, 197, 4, False, False), (8, 4, 49, 6, True, False), (4, 2, 257, 4, False, False),
                                                    (2, 2, 2048, 8, False, True), (3, 3, 64, 8, False, False), (2, 1, 1, 4, False, False),
                                                    (2, 2, 1000, 6, True, True), (2, 2, 4096, 8, False, False), (5, 5, 20, 8, True, True)])
def test_softmax_log2_codes(rq, G, H, N, bits, bias, causal):
    b, ctx = rq
    print("case", G, H, N, bits, bias, causal, flush=True)
    g = np.random.default_rng(G + N + bits)
    dh = 64
    # accumulators of 4..8-bit q, k whose de-quantized values are ~N(0,1): heavy-tailed probabilities
    sq = 8.0 / 2 ** 8
    acc = np.rint(g.normal(size=(G, N, N)) * math.sqrt(dh) / (sq * sq)).astype(np.int64)
    ld = _ld(N)
    accp = np.full((G, N, ld), 7777, np.int32)
    accp[:, :, :N] = acc
    scale = sq * sq / math.sqrt(dh)
    bias_a = (g.normal(0, 0.5, size=(H, N, N)).astype(np.float32)) if bias else None
    s_log = np.float32(0.8)
    want = np.empty((G, N, N), np.int64)
    for gi in range(G):
        L = acc[gi].astype(np.float64) * scale
        if bias:
            L = L + bias_a[gi % H].astype(np.float64)
        if causal:
            L = np.where(np.arange(N)[None, :] > np.arange(N)[:, None], -np.inf, L)
        want[gi] = orc.softmax_log_quant(L, s_log, bits)
    codes = torch.full((G, N, ld), 99, dtype=torch.uint8, device="cuda")
    b.rq_softmax_log2_quant(ctx, dev(accp), G, H, N, N, ld, scale, codes, bits, s_log=float(s_log),
                            bias=None if bias_a is None else dev(bias_a), mask=b.MASK_CAUSAL if causal else b.MASK_NONE)
    got = codes.cpu().numpy()
    assert_codes_close(got[:, :, :N], want, "softmax codes N=%d b=%d" % (N, bits))
    assert np.all(got[:, :, N:] == 2 ** bits - 1)


@pytest.mark.parametrize("G,H,nq,nk,bits,bias", [(4, 2, 50, 197, 4, True), (3, 3, 197, 40, 6, False), (2, 2, 7, 1500, 8, True),
                                                 (2, 1, 300, 33, 4, False)])
def test_softmax_log2_codes_rectangular(rq, G, H, nq, nk, bits, bias):
    """Rows of nk keys for nq queries with nq != nk (accumulators [G, nq, ld], bias planes [H, nq, nk])."""
    b, ctx = rq
    print("case", G, H, nq, nk, bits, bias, flush=True)
    g = np.random.default_rng(G + nq * 3 + nk + bits)
    acc = np.rint(g.normal(size=(G, nq, nk)) * 8000).astype(np.int64)
    scale = 1.0 / 2048
    ld = _ld(nk)
    accp = np.full((G, nq, ld), -31337, np.int32)
    accp[:, :, :nk] = acc
    bias_a = g.normal(0, 0.7, size=(H, nq, nk)).astype(np.float32) if bias else None
    s_log = np.float32(1.0)
    want = np.empty((G, nq, nk), np.int64)
    for gi in range(G):
        L = acc[gi].astype(np.float64) * scale
        if bias:
            L = L + bias_a[gi % H].astype(np.float64)
        want[gi] = orc.softmax_log_quant(L, s_log, bits)
    codes = torch.full((G, nq, ld), 99, dtype=torch.uint8, device="cuda")
    b.rq_softmax_log2_quant(ctx, dev(accp), G, H, nq, nk, ld, scale, codes, bits, s_log=float(s_log),
                            bias=None if bias_a is None else dev(bias_a))
    got = codes.cpu().numpy()
    assert_codes_close(got[:, :, :nk], want, "softmax codes %d x %d b=%d" % (nq, nk, bits))
    assert np.all(got[:, :, nk:] == 2 ** bits - 1)


@pytest.mark.parametrize("batch,H,seq,dh,bits_p,bits_v,causal", [(2, 3, 197, 64, 4, 4, False), (2, 2, 49, 32, 6, 6, False),
                                                                 (1, 2, 257, 64, 4, 4, False), (1, 2, 600, 128, 8, 8, True),
                                                                 (2, 2, 64, 64, 8, 8, False), (1, 1, 1, 32, 4, 8, False),
                                                                 (1, 2, 300, 64, 4, 8, True),
                                                                 # wide codes on rows beyond 256 keys: the bfloat16 kernel
                                                                 (1, 2, 300, 64, 6, 8, False), (2, 1, 700, 32, 8, 6, True),
                                                                 (1, 1, 1025, 128, 8, 8, False), (1, 2, 257, 128, 5, 4, True)])
def test_attn_pv(rq, batch, H, seq, dh, bits_p, bits_v, causal):
    _attn_pv_case(rq, batch, H, seq, dh, bits_p, bits_v, causal, False)


@pytest.mark.parametrize("batch,H,seq,dh,bits_p,bits_v,causal", [(2, 2, 197, 64, 4, 4, False), (2, 2, 49, 32, 6, 6, False),
                                                                 (1, 2, 257, 64, 4, 8, True), (1, 2, 300, 64, 6, 8, False),
                                                                 (1, 1, 520, 128, 8, 8, True), (1, 2, 40, 32, 3, 4, False)])
def test_attn_pv_zero_at_max_code(rq, batch, H, seq, dh, bits_p, bits_v, causal):
    """RQ_LOG_ZERO_AT_MAX_CODE: keys whose code is the saturated one contribute nothing (every kernel variant of rq_attn_pv)."""
    _attn_pv_case(rq, batch, H, seq, dh, bits_p, bits_v, causal, True)


def _attn_pv_case(rq, batch, H, seq, dh, bits_p, bits_v, causal, zero_max):
    b, ctx = rq
    print("case", batch, H, seq, dh, bits_p, bits_v, causal, zero_max, flush=True)
    g = np.random.default_rng(seq + dh + bits_p)
    D = H * dh
    ld = _ld(seq)
    # codes with a realistic spread: most mass on large codes, a few small ones
    A = orc.softmax_rows(g.normal(size=(batch * H, seq, seq)) * 3)
    codes = orc.logsqrt2_quant_base2(A, 1.0, bits_p)
    if zero_max:         # make sure the saturated code is there, also where the softmax of this draw rarely reaches it
        codes[g.random(codes.shape) < 0.05] = 2 ** bits_p - 1
    cp = np.full((batch * H, seq, ld), 3, np.uint8)      # padding holds a small code on purpose: it must be ignored
    cp[:, :, :seq] = codes
    qv = g.integers(0, 2 ** bits_v, size=(batch * seq, D))
    z_v = int(g.integers(0, 2 ** bits_v))
    offv = b.store_offset(bits_v, z_v)
    qkv = np.zeros((batch * seq, 3 * D), np.int8)
    qkv[:, 2 * D:] = (qv - offv).astype(np.int8)
    s_log, s_v = np.float32(0.9), np.float32(0.043)
    want = np.empty((batch * seq, D))
    for bi in range(batch):
        r = slice(bi * seq, (bi + 1) * seq)
        for h in range(H):
            want[r, h * dh:(h + 1) * dh] = orc.attn_pv(codes[bi * H + h], qv[r, h * dh:(h + 1) * dh], s_log, s_v, z_v, causal,
                                                       bits_p, zero_max)
    s_o = np.float32((want.max() - want.min()) / (2 ** bits_v - 1))
    z_o = int(np.rint(-want.min() / np.float64(s_o)))
    off_o = b.store_offset(bits_v, z_o)
    qd = dev(qkv)
    outf = torch.zeros((batch * seq, D), dtype=torch.float32, device="cuda")
    outq = torch.zeros((batch * seq, D), dtype=torch.int8, device="cuda")
    b.rq_attn_pv(ctx, dev(cp), ld, qd.data_ptr() + 2 * D, 3 * D, batch, H, seq, seq, dh, float(s_log), float(s_v), z_v, offv, bits_p,
                 mask=b.MASK_CAUSAL if causal else b.MASK_NONE, out_f32=outf, out_q=outq, s_o=float(s_o), z_o=z_o, off_o=off_o,
                 bits_o=bits_v, flags=b.LOG_ZERO_AT_MAX_CODE if zero_max else 0)
    # exact integer sums everywhere except for wide codes on long rows, which accumulate in float32 on the bfloat16
    # matrix cores: n terms of magnitude <= |v| p_j each round to 2^-24 of the running sum
    assert_float_close(outf.cpu().numpy(), want, "attn_pv", rtol=1e-4 if (bits_p > 4 and seq > 256) else 1e-5)
    assert_codes_close(outq.cpu().numpy().astype(np.int64) + off_o, orc.uniform_quant(want, s_o, z_o, bits_v), "attn_pv codes")


@pytest.mark.parametrize("batch,H,nq,nk,dh,bits_p,bits_v", [(2, 2, 50, 197, 64, 4, 4), (1, 3, 197, 40, 32, 4, 8), (2, 1, 70, 300, 64, 8, 8),
                                                           (1, 2, 330, 100, 128, 6, 6), (1, 1, 1, 513, 64, 8, 4), (1, 2, 290, 270, 64, 4, 4)])
def test_attn_pv_rectangular(rq, batch, H, nq, nk, dh, bits_p, bits_v):
    """Query and key counts that differ (the codes of one group are [nq, nk]; V has batch * nk rows, the output batch * nq)."""
    b, ctx = rq
    print("case", batch, H, nq, nk, dh, bits_p, bits_v, flush=True)
    g = np.random.default_rng(nq * 7 + nk + dh + bits_p)
    D = H * dh
    ld = _ld(nk)
    codes = orc.logsqrt2_quant_base2(orc.softmax_rows(g.normal(size=(batch * H, nq, nk)) * 3), 1.0, bits_p)
    cp = np.full((batch * H, nq, ld), 2, np.uint8)
    cp[:, :, :nk] = codes
    qv = g.integers(0, 2 ** bits_v, size=(batch * nk, D))
    z_v = int(g.integers(0, 2 ** bits_v))
    offv = b.store_offset(bits_v, z_v)
    s_log, s_v = np.float32(1.1), np.float32(0.021)
    want = np.empty((batch * nq, D))
    for bi in range(batch):
        for h in range(H):
            want[bi * nq:(bi + 1) * nq, h * dh:(h + 1) * dh] = orc.attn_pv(codes[bi * H + h], qv[bi * nk:(bi + 1) * nk, h * dh:(h + 1) * dh],
                                                                         s_log, s_v, z_v)
    vd = dev((qv - offv).astype(np.int8))
    outf = torch.zeros((batch * nq, D), dtype=torch.float32, device="cuda")
    b.rq_attn_pv(ctx, dev(cp), ld, vd.data_ptr(), D, batch, H, nq, nk, dh, float(s_log), float(s_v), z_v, offv, bits_p, out_f32=outf)
    # narrow codes: exact integer sums, rounded once.  Wide codes: float32 sums (the per-window integer sums of short rows
    # are each rounded to 2^-24 of themselves before they are added; long rows accumulate in float32 on the bfloat16
    # matrix cores), so an output that cancels to nearly zero keeps an error of ~1e-7 of the row's magnitude
    assert_float_close(outf.cpu().numpy(), want, "attn_pv rectangular", rtol=1e-4 if bits_p > 4 else 1e-5)


@pytest.mark.parametrize("batch,H,seq,dh,bits,bits_p,bias,causal", [(2, 3, 197, 64, 4, 4, False, False), (3, 2, 49, 32, 6, 6, True, False),
                                                                    (2, 2, 257, 64, 4, 4, False, False), (1, 2, 288, 128, 8, 8, False, True),
                                                                    (2, 2, 64, 64, 8, 8, False, False), (1, 1, 1, 32, 8, 4, False, False),
                                                                    (1, 2, 33, 64, 8, 6, True, True), (2, 1, 130, 128, 6, 4, False, False),
                                                                    # bias with codes of at most 6 bits: float32 logits
                                                                    (2, 4, 49, 32, 6, 4, True, False), (1, 3, 197, 64, 4, 4, True, False),
                                                                    (1, 2, 100, 128, 6, 6, True, False),
                                                                    # rows beyond 288 keys: the two-sweep kernel
                                                                    (1, 2, 289, 64, 4, 4, False, False), (2, 1, 320, 128, 8, 8, False, True),
                                                                    (1, 3, 500, 32, 6, 6, False, True), (1, 1, 1000, 64, 8, 4, False, False),
                                                                    (1, 2, 1025, 128, 8, 8, False, True), (2, 2, 384, 64, 4, 3, False, True)])
def test_fused_qk_softmax_codes(rq, batch, H, seq, dh, bits, bits_p, bias, causal):
    """The single-kernel Q.K^T + Softmax-log2 path against the oracle's integer logits and log-sqrt2 codes."""
    b, ctx = rq
    print("case", batch, H, seq, dh, bits, bits_p, bias, causal, flush=True)
    g = np.random.default_rng(seq * 7 + dh + bits)
    D = H * dh
    qmax = 2 ** bits - 1
    # q, k codes of ~N(0,1) values quantized on [-4, 4]
    s_qk = 8.0 / qmax
    z_q, z_k = int(g.integers(qmax // 3, 2 * qmax // 3 + 1)), int(g.integers(qmax // 3, 2 * qmax // 3 + 1))
    codes = np.empty((batch * seq, 3 * D), np.int64)
    codes[:, :D] = np.clip(np.rint(g.normal(size=(batch * seq, D)) / s_qk) + z_q, 0, qmax)
    codes[:, D:2 * D] = np.clip(np.rint(g.normal(size=(batch * seq, D)) / s_qk) + z_k, 0, qmax)
    codes[:, 2 * D:] = 0
    offq, offk = b.store_offset(bits, z_q), b.store_offset(bits, z_k)
    st = codes.copy()
    st[:, :D] -= offq
    st[:, D:2 * D] -= offk
    qkv = dev(st.astype(np.int8))
    ld = _ld(seq)
    scale = s_qk * s_qk / math.sqrt(dh)
    bias_a = g.normal(0, 0.5, size=(H, seq, seq)).astype(np.float32) if bias else None
    s_log = np.float32(0.8)
    want = np.empty((batch * H, seq, seq), np.int64)
    for bi in range(batch):
        r = slice(bi * seq, (bi + 1) * seq)
        for h in range(H):
            acc = orc.int_matmul_nt(codes[r, h * dh:(h + 1) * dh] - z_q, codes[r, D + h * dh:D + (h + 1) * dh] - z_k)
            L = acc.astype(np.float64) * scale
            if bias:
                L = L + bias_a[h].astype(np.float64)
            if causal:
                L = np.where(np.arange(seq)[None, :] > np.arange(seq)[:, None], -np.inf, L)
            want[bi * H + h] = orc.softmax_log_quant(L, s_log, bits_p)
    out = torch.full((batch * H, seq, ld), 99, dtype=torch.uint8, device="cuda")
    b.rq_qk_softmax_log2_quant(ctx, qkv, batch, seq, H, dh, 0, D, offq, z_q, offk, z_k, scale, out, ld, bits_p, s_log=float(s_log),
                               bias=None if bias_a is None else dev(bias_a), mask=b.MASK_CAUSAL if causal else b.MASK_NONE)
    got = out.cpu().numpy()
    assert_codes_close(got[:, :, :seq], want, "fused codes N=%d b=%d" % (seq, bits_p))
    assert np.all(got[:, :, seq:] == 2 ** bits_p - 1)


@pytest.mark.parametrize("batch,H,seq,dh,bits,bits_p", [(2, 3, 197, 64, 4, 4), (3, 2, 49, 32, 6, 4), (1, 2, 224, 64, 4, 4),
                                                        (2, 2, 64, 128, 8, 4), (1, 1, 1, 32, 8, 3), (2, 1, 288, 32, 4, 4),
                                                        (5, 2, 100, 64, 8, 2), (2, 2, 257, 64, 4, 4), (1, 3, 256, 64, 8, 4),
                                                        (2, 1, 288, 64, 4, 4), (1, 2, 160, 128, 4, 4), (1, 2, 288, 128, 8, 4),
                                                        (3, 3, 270, 64, 8, 4), (2, 3, 259, 32, 8, 3), (5, 1, 257, 64, 8, 2)])
def test_attn_fused_whole(rq, batch, H, seq, dh, bits, bits_p):
    """rq_attn_fused (one kernel) against the oracle's logits -> log-sqrt2 codes -> shift de-quantized P.V -> uniform codes."""
    _attn_fused_case(rq, batch, H, seq, dh, bits, bits_p, False)


@pytest.mark.parametrize("batch,H,seq,dh,bits,bits_p,bias", [(4, 4, 49, 32, 6, 6, True), (3, 2, 49, 32, 4, 4, True), (2, 3, 64, 32, 6, 5, False),
                                                             (2, 2, 144, 32, 6, 6, True), (1, 2, 160, 64, 8, 6, False), (2, 1, 100, 128, 6, 6, True),
                                                             (1, 1, 1, 32, 6, 6, True), (2, 2, 33, 64, 4, 3, True)])
def test_attn_fused_whole_windows(rq, batch, H, seq, dh, bits, bits_p, bias):
    """The one-kernel attention with a relative-position bias and / or codes of 5 or 6 bits (bfloat16 P.V): window attention."""
    _attn_fused_case(rq, batch, H, seq, dh, bits, bits_p, bias)


@pytest.mark.parametrize("batch,H,seq,dh,bits,bits_p,bias", [(2, 3, 197, 64, 4, 4, False), (2, 2, 257, 64, 4, 4, False),
                                                             (3, 2, 49, 32, 6, 6, True), (2, 2, 64, 128, 8, 3, False)])
def test_attn_fused_zero_at_max_code(rq, batch, H, seq, dh, bits, bits_p, bias):
    """RQ_LOG_ZERO_AT_MAX_CODE in the one-kernel attention (int8 and bfloat16 P.V variants)."""
    _attn_fused_case(rq, batch, H, seq, dh, bits, bits_p, bias, True)


def _attn_fused_case(rq, batch, H, seq, dh, bits, bits_p, bias, zero_max=False):
    b, ctx = rq
    flags = b.LOG_ZERO_AT_MAX_CODE if zero_max else 0
    print("case", batch, H, seq, dh, bits, bits_p, bias, zero_max, flush=True)
    assert b.attn_fused_supported(seq, dh, bits_p, bias)
    g = np.random.default_rng(seq * 3 + dh + bits)
    D = H * dh
    qmax = 2 ** bits - 1
    s_qk = 8.0 / qmax
    z = [int(g.integers(qmax // 3, 2 * qmax // 3 + 1)) for _ in range(3)]
    codes = np.empty((batch * seq, 3 * D), np.int64)
    for i in range(3):
        codes[:, i * D:(i + 1) * D] = np.clip(np.rint(g.normal(size=(batch * seq, D)) / s_qk) + z[i], 0, qmax)
    off = [b.store_offset(bits, zz) for zz in z]
    st = codes.copy()
    for i in range(3):
        st[:, i * D:(i + 1) * D] -= off[i]
    qkv = dev(st.astype(np.int8))
    ld = _ld(seq)
    scale = s_qk * s_qk / math.sqrt(dh)
    s_log, s_v = np.float32(0.8), np.float32(s_qk)
    bias_a = g.normal(0, 0.5, size=(H, seq, seq)).astype(np.float32) if bias else None
    want_codes = np.empty((batch * H, seq, seq), np.int64)
    want = np.empty((batch * seq, D))
    for bi in range(batch):
        r = slice(bi * seq, (bi + 1) * seq)
        for h in range(H):
            c = slice(h * dh, (h + 1) * dh)
            acc = orc.int_matmul_nt(codes[r, c] - z[0], codes[r, D + h * dh:D + (h + 1) * dh] - z[1])
            L = acc.astype(np.float64) * scale
            if bias:
                L = L + bias_a[h].astype(np.float64)
            pc = orc.softmax_log_quant(L, s_log, bits_p)
            want_codes[bi * H + h] = pc
            want[r, c] = orc.attn_pv(pc, codes[r, 2 * D + h * dh:2 * D + (h + 1) * dh], s_log, s_v, z[2], False, bits_p, zero_max)
    s_o = np.float32((want.max() - want.min()) / qmax)
    z_o = int(np.rint(-want.min() / np.float64(s_o)))
    off_o = b.store_offset(bits, z_o)
    outc = torch.full((batch * H, seq, ld), 99, dtype=torch.uint8, device="cuda")
    outf = torch.zeros((batch * seq, D), dtype=torch.float32, device="cuda")
    outq = torch.zeros((batch * seq, D), dtype=torch.int8, device="cuda")
    b.rq_attn_fused(ctx, qkv, batch, seq, H, dh, off[0], z[0], off[1], z[1], off[2], z[2], scale, float(s_log), float(s_v), bits_p,
                    codes=outc, ld=ld, out_f32=outf, out_q=outq, s_o=float(s_o), z_o=z_o, off_o=off_o, bits_o=bits,
                    bias=None if bias_a is None else dev(bias_a), flags=flags)
    got_codes = outc.cpu().numpy()[:, :, :seq]
    frac = assert_codes_close(got_codes, want_codes, "fused attention codes")
    # float32 epilogue on exact integer sums: the even- and odd-code terms can cancel, so an element far below the row's
    # scale carries the rounding of the larger terms (6e-8 of them) -- hence 1e-4 element-wise, not 1e-5
    if frac == 0.0:      # identical codes -> the P.V sums are the same exact integers: only float rounding differs
        assert_float_close(outf.cpu().numpy(), want, "fused attention out", rtol=1e-4)
        assert_codes_close(outq.cpu().numpy().astype(np.int64) + off_o, orc.uniform_quant(want, s_o, z_o, bits), "fused attention out codes")
    else:                # a tie flipped a code: compare P.V against the oracle's P.V of the codes the kernel produced
        for bi in range(batch):
            r = slice(bi * seq, (bi + 1) * seq)
            for h in range(H):
                c = slice(h * dh, (h + 1) * dh)
                want[r, c] = orc.attn_pv(got_codes[bi * H + h].astype(np.int64), codes[r, 2 * D + h * dh:2 * D + (h + 1) * dh], s_log,
                                         s_v, z[2], False, bits_p, zero_max)
        assert_float_close(outf.cpu().numpy(), want, "fused attention out", rtol=1e-4)
    # without the optional codes output the result is the same
    outq2 = torch.zeros_like(outq)
    b.rq_attn_fused(ctx, qkv, batch, seq, H, dh, off[0], z[0], off[1], z[1], off[2], z[2], scale, float(s_log), float(s_v), bits_p,
                    out_q=outq2, s_o=float(s_o), z_o=z_o, off_o=off_o, bits_o=bits, bias=None if bias_a is None else dev(bias_a),
                    flags=flags)
    assert torch.equal(outq, outq2)


def test_attn_fused_many_passes(rq):
    """257 keys, more groups than one pass of every workgroup takes (the persistent workgroups of the streamed kernel refill
    their LDS slots while they compute, and the last pass is partial): sampled batch items against the oracle, and every item
    bit-equal to a call on that item alone."""
    b, ctx = rq
    batch, H, seq, dh, bits, bits_p = 515, 2, 257, 32, 8, 4
    assert b.attn_fused_supported(seq, dh, bits_p, False)
    g = np.random.default_rng(77)
    D = H * dh
    qmax = 2 ** bits - 1
    s_qk = 8.0 / qmax
    z = [int(g.integers(qmax // 3, 2 * qmax // 3 + 1)) for _ in range(3)]
    codes = np.empty((batch * seq, 3 * D), np.int64)
    for i in range(3):
        codes[:, i * D:(i + 1) * D] = np.clip(np.rint(g.normal(size=(batch * seq, D)) / s_qk) + z[i], 0, qmax)
    off = [b.store_offset(bits, zz) for zz in z]
    st = codes.copy()
    for i in range(3):
        st[:, i * D:(i + 1) * D] -= off[i]
    qkv = dev(st.astype(np.int8))
    scale = s_qk * s_qk / math.sqrt(dh)
    s_log, s_v = np.float32(0.8), np.float32(s_qk)
    s_o, z_o = np.float32(0.004), 120
    off_o = b.store_offset(bits, z_o)
    outq = torch.zeros((batch * seq, D), dtype=torch.int8, device="cuda")
    outf = torch.zeros((batch * seq, D), dtype=torch.float32, device="cuda")
    print("case many passes", batch, H, seq, dh, flush=True)
    b.rq_attn_fused(ctx, qkv, batch, seq, H, dh, off[0], z[0], off[1], z[1], off[2], z[2], scale, float(s_log), float(s_v), bits_p,
                    out_f32=outf, out_q=outq, s_o=float(s_o), z_o=z_o, off_o=off_o, bits_o=bits)
    torch.cuda.synchronize()
    gotf = outf.cpu().numpy()
    for bi in (0, 1, 255, 256, 511, 512, 513, 514):
        r = slice(bi * seq, (bi + 1) * seq)
        one_q = torch.zeros((seq, D), dtype=torch.int8, device="cuda")
        b.rq_attn_fused(ctx, qkv[bi * seq:(bi + 1) * seq], 1, seq, H, dh, off[0], z[0], off[1], z[1], off[2], z[2], scale, float(s_log),
                        float(s_v), bits_p, out_q=one_q, s_o=float(s_o), z_o=z_o, off_o=off_o, bits_o=bits)
        assert torch.equal(one_q, outq[r]), "batch item %d differs from its own call" % bi
        want = np.empty((seq, D))
        flips = 0
        for h in range(H):
            c = slice(h * dh, (h + 1) * dh)
            acc = orc.int_matmul_nt(codes[r, c] - z[0], codes[r, D + h * dh:D + (h + 1) * dh] - z[1])
            pc = orc.softmax_log_quant(acc.astype(np.float64) * scale, s_log, bits_p)
            want[:, c] = orc.attn_pv(pc, codes[r, 2 * D + h * dh:2 * D + (h + 1) * dh], s_log, s_v, z[2], False, bits_p)
        # a code next to a rounding tie may differ (float32 against float64 sum); rows without one meet the float bar
        e = np.abs(gotf[r] - want).max(axis=1)
        ref = np.abs(want).max()
        assert np.mean(e > 1e-4 * ref) < 0.02, "batch item %d: %g of the rows off" % (bi, np.mean(e > 1e-4 * ref))
        assert e.max() < 0.05 * ref
    # every item, not only the sampled ones, was written
    assert int((outq.view(batch, seq * D) == 0).all(dim=1).sum()) == 0
